/*
 * msched.h -- C ABI of the MI355X-native MSched hot path (arXiv 2512.24637,
 * "Towards Fully-fledged GPU Multitasking via Proactive Memory Scheduling").
 *
 * One context = one GPU's HBM frame pool, its page table and the command
 * queues of the tasks that share it.  At every context switch the scheduler
 * calls msched_plan() with its task timeline and then msched_migrate(); both
 * run as HIP kernels on gfx950.  No torch types cross this boundary: callers
 * pass plain pointers (each marked HOST or DEVICE below) and sizes.
 *
 * Threading: a context is used by one thread at a time (the paper's
 * coordinator is a single daemon, Sec. 6.2).  All device work is issued on the
 * stream given at creation.
 *
 * Errors: every call returns MSCHED_OK (0) or a negative code and leaves the
 * context unchanged on error.
 */
#ifndef MSCHED_H
#define MSCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MSCHED_NOT_RESIDENT 0xFFFFFFFFu       /* page-table value of a page that is not in HBM */
#define MSCHED_NO_SLOT 0xFFFFFFFFu            /* host_slot value of a page without backing store */
#define MSCHED_MAX_ARGS 12                    /* 64-bit launch arguments per command */
#define MSCHED_MAX_RULES 8                    /* access rules per kernel template */
#define MSCHED_MAX_PRODUCT_ARGS 4             /* arguments multiplied in one formula */
#define MSCHED_MAX_TIMELINE_COMMANDS 3071     /* commands one plan may look ahead over */
#define MSCHED_MAX_TIMELINE_ENTRIES 1024

enum {
    MSCHED_OK = 0,
    MSCHED_E_INVAL = -1,           /* bad argument, unknown task or kernel, too long a timeline */
    MSCHED_E_RANGE = -2,           /* page >= n_virtual_pages, page without backing slot, rule names a missing argument */
    MSCHED_E_OVERFLOW = -3,        /* template arithmetic exceeds 64 bits */
    MSCHED_E_WSET_TOO_LARGE = -4,  /* the first command of the incoming task alone needs more than n_frames pages */
    MSCHED_E_STALE_PLAN = -5,      /* migrate with a plan that is not the latest, or already carried out */
    MSCHED_E_NOMEM = -6,
    MSCHED_E_HIP = -7,             /* a HIP call failed; see msched_last_hip_error() */
    MSCHED_E_TOO_LARGE = -8        /* request larger than a fixed-size buffer of the library (msched_pagetable_query_static) */
};

typedef struct msched_ctx msched_ctx;          /* opaque, library-owned */

typedef struct {
    uint32_t page_shift;          /* log2(page bytes), 6..30 */
    uint32_t n_frames;            /* F: frames in the HBM pool */
    uint64_t n_virtual_pages;     /* V: page-table length, < 2^32 - 1 */
    void *hbm_pool;               /* DEVICE, n_frames << page_shift bytes, 16-byte aligned, caller-owned */
    void *host_store;             /* HOST pinned and device-accessible, n_host_slots << page_shift bytes, caller-owned */
    uint64_t n_host_slots;        /* pages in host_store */
    const uint32_t *host_slot;    /* HOST, V entries (page -> slot, MSCHED_NO_SLOT = none) or NULL = identity; copied.
                                     No two pages may share a slot (E_INVAL); a slot >= n_host_slots is E_RANGE */
    void *stream;                 /* hipStream_t all device work is issued on (NULL = default stream) */
} msched_config;

/*
 * One access rule of a kernel template (Sec. 5.2, "Access pattern templates").
 * The region starts at the byte address held in launch argument base_arg.  Each
 * of size, stride and count is coeff * product(args[idx[0..n-1]]), empty product = 1,
 * evaluated in unsigned 64-bit arithmetic.
 *   FIXED   (T1) one range of size_coeff bytes (n_size_args must be 0)
 *   LINEAR  (T2) one range of `size` bytes
 *   STRIDED (T3) `count` ranges of `size` bytes, the j-th starting at base + j*stride
 *   LIST         the explicit page ids attached to the launch (sparse gathers, which the
 *                paper's templates do not cover); base/size/stride/count are ignored
 * A range of b bytes at address a touches pages floor(a/P) .. floor((a+b-1)/P); zero bytes touch nothing.
 */
enum { MSCHED_RULE_FIXED = 1, MSCHED_RULE_LINEAR = 2, MSCHED_RULE_STRIDED = 3, MSCHED_RULE_LIST = 4 };

typedef struct {
    uint8_t kind;
    uint8_t base_arg;
    uint8_t n_size_args, n_stride_args, n_count_args;
    uint8_t size_args[MSCHED_MAX_PRODUCT_ARGS];
    uint8_t stride_args[MSCHED_MAX_PRODUCT_ARGS];
    uint8_t count_args[MSCHED_MAX_PRODUCT_ARGS];
    uint8_t reserved[7];
    uint64_t size_coeff, stride_coeff, count_coeff;
} msched_rule;                                  /* 48 bytes */

/* One entry of the task scheduling timeline (Sec. 6.1): which task runs next and for how
 * many ticks.  Commands are taken from the task's queue while the latency accumulated in
 * the entry is below timeslice; a task listed again continues where it stopped. */
typedef struct { uint32_t task; uint32_t timeslice; } msched_timeline_entry;

typedef struct {
    uint32_t n_evict;             /* pages to copy out, in eviction order */
    uint32_t n_fetch;             /* pages to copy in, in order of first use */
    uint32_t n_free_used;         /* fetches that go to free frames (the first n_free_used of the list) */
    uint32_t covered_launches;    /* commands of entry 0 whose pages will all be resident (= g_cut) */
    uint32_t g_cut;
    uint32_t g_end0;              /* commands entry 0 holds; covered_launches < g_end0 means the slice was cut */
    uint32_t n_commands;          /* G: commands in the flattened timeline */
    uint32_t reserved;
    const uint32_t *evict_pages;  /* DEVICE, context-owned, valid until the next msched_plan; complete in stream order */
    const uint32_t *evict_frames; /* DEVICE */
    const uint32_t *fetch_pages;  /* DEVICE */
    const uint32_t *fetch_frames; /* DEVICE */
    uint64_t plan_id;
} msched_plan_t;

/* Create a context.  Nothing is resident, every frame is free.  *out is set on success. */
int msched_create(const msched_config *cfg, msched_ctx **out);
int msched_destroy(msched_ctx *ctx);

/* Register a kernel template of n_rules <= MSCHED_MAX_RULES rules (HOST array); *kernel_id receives its id.
 * Stands for one record of the offline description file (Sec. 4.1). */
int msched_kernel_register(msched_ctx *ctx, const msched_rule *rules, uint32_t n_rules, uint32_t *kernel_id);

/* Create a task (one process's command queue, Sec. 6.2 "Distributed metadata management"). */
int msched_task_create(msched_ctx *ctx, uint32_t *task_id);

/*
 * Append a launch to a task's queue (Sec. 5.2 "Memory access prediction": launch arguments are
 * captured when the command is issued; Sec. 6.2: the queue holds the command and its profiled
 * latency).  args: HOST, n_args <= MSCHED_MAX_ARGS values (32-bit arguments zero-extended).
 * id_list: DEVICE array of n_ids page ids for the kernel's LIST rule, or NULL; it is NOT copied.
 * It must stay valid and unchanged from this call until the launch has been retired AND the context's
 * stream has passed the last msched_plan / msched_migrate issued before that msched_launch_retire:
 * retiring is a host-side step that does not wait, and a migration may still have the list's preparation
 * queued behind its copy.  (Synchronise the stream, or free the list in stream order, after the retire.)
 * The template's formulas are evaluated here, once, with these arguments (Sec. 5.2: prediction at launch
 * time): E_RANGE / E_OVERFLOW launches are refused, and plans reuse the page ranges worked out here.
 * (Ids inside id_list are checked by msched_plan, which then returns E_RANGE.)
 */
int msched_launch_enqueue(msched_ctx *ctx, uint32_t task, uint32_t kernel_id,
                          const uint64_t *args, uint32_t n_args, uint32_t latency_ticks,
                          const uint32_t *id_list, uint32_t n_ids);

/* The first n_launches queued commands of the task have executed ("currently executing command"
 * of Sec. 6.2 moves forward). */
int msched_launch_retire(msched_ctx *ctx, uint32_t task, uint32_t n_launches);

/*
 * Plan the migration for a context switch (Sec. 6.2 "Enforcing the OPT memory scheduling").
 * tl: HOST, n_entries <= MSCHED_MAX_TIMELINE_ENTRIES, entry 0 is the incoming task.
 * Flattens the timeline into the order of future commands, expands every command's template
 * into pages, gives each page the position of its first future use, cuts entry 0 to the longest
 * command prefix whose pages fit the pool, and selects
 *   fetch  = wanted and not resident, ordered by (first use, page id)
 *   evict  = first max(0, n_fetch - free frames) resident pages that are not wanted, ordered by
 *            (first use descending with never-used first, page id)
 * Fetched page i takes the i-th lowest free frame, or the frame of evict[i - n_free_used].
 * Does not change the page table.  Blocks until the counts in *out are known - which is before the four
 * device lists are complete: the kernels that fill them may still be running on the context's stream when
 * the call returns.  Work on that stream (msched_migrate) sees them complete; so does any caller after
 * msched_plan_copy_lists, msched_state_copy or a synchronisation of the stream.
 */
int msched_plan(msched_ctx *ctx, const msched_timeline_entry *tl, uint32_t n_entries, msched_plan_t *out);

/*
 * Carry out the latest plan (Sec. 6.2 "Driver support": evict, then populate; Sec. 6.3: victim
 * copy-out and target copy-in proceed in parallel, target i reusing the space of victim i):
 * host_store[slot(evict[i])] <- pool[evict_frames[i]], pool[fetch_frames[i]] <- host_store[slot(fetch[i])],
 * then the page table and frame owners are updated.  Asynchronous on the context's stream; a plan
 * can be carried out once.
 * Behind the migration, on the same stream, the call may also bin the id lists of commands queued beyond the
 * planned ones (preparation for the next plans, hidden behind the host-link transfer): those lists are read
 * then, which is why they must be valid from msched_launch_enqueue on.  A failure of that preparation never
 * fails the call (it switches the look-ahead off).
 */
int msched_migrate(msched_ctx *ctx, const msched_plan_t *plan);

/* Frame of each page, or MSCHED_NOT_RESIDENT.  page_ids: HOST, out: HOST.  Waits for the stream. */
int msched_pagetable_query(msched_ctx *ctx, const uint64_t *page_ids, uint32_t n, uint32_t *out);

/*
 * msched_pagetable_query for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments, same result, but the ids and the answers are
 * staged in a fixed device array that is part of the library's code object, so the call never allocates or
 * frees memory, on the device or on the host, and never grows a buffer of the context.
 * n <= MSCHED_QUERY_STATIC_MAX, else MSCHED_E_TOO_LARGE (nothing is done).  Each GPU holds one copy of the
 * array (MSCHED_QUERY_STATIC_MAX * 12 bytes) from the first msched_create on it until the process ends.  Every
 * call on a GPU, from any context, uses that one array: calls that overlap on one GPU race (callers serialise
 * them; one context is single-threaded anyway).  Nothing in the array has to start at zero: a call overwrites
 * the n ids and n answers it uses and reads nothing else.  Waits for the stream like msched_pagetable_query.
 */
#define MSCHED_QUERY_STATIC_MAX 65536u
int msched_pagetable_query_static(msched_ctx *ctx, const uint64_t *page_ids, uint32_t n, uint32_t *out);

/* Copy the lists of the latest plan to HOST arrays (any may be NULL) of n_evict / n_fetch entries. */
int msched_plan_copy_lists(msched_ctx *ctx, const msched_plan_t *plan, uint32_t *evict_pages,
                           uint32_t *evict_frames, uint32_t *fetch_pages, uint32_t *fetch_frames);

/* Copy the whole page table (V entries) and frame-owner table (F entries) to HOST arrays (either may be NULL). */
int msched_state_copy(msched_ctx *ctx, uint32_t *page_table, uint32_t *frame_owner);

/*
 * Per-phase device times of the last plan and the last migrate, measured with HIP events on the
 * context's stream when profiling is on, and the host-clock split of the last msched_plan call (always
 * measured).  ms: HOST array of MSCHED_N_PHASES floats, all in milliseconds.
 */
enum { MSCHED_PHASE_EXPAND = 0,   /* next-use reset + template expansion + scatter-min */
       MSCHED_PHASE_COUNT = 1,    /* per-chunk class histograms over the page table */
       MSCHED_PHASE_CUT = 2,      /* totals, budget cut, victim threshold, output offsets */
       MSCHED_PHASE_EMIT = 3,     /* ordered compaction of both lists + frame assignment */
       MSCHED_PHASE_MIGRATE = 4,  /* copy kernel + page-table update */
       MSCHED_PHASE_PLAN = 5,     /* all planning kernels of one msched_plan, first launch to last */
       MSCHED_HOST_PREP = 6,      /* host clock: timeline flatten + repeat detection of the last plan */
       MSCHED_HOST_LAUNCH = 7,    /* host clock: issuing the plan's kernel launches */
       MSCHED_HOST_WAIT = 8,      /* host clock: waiting for the plan's kernels and reading the counts */
       MSCHED_PHASE_PREPARE = 9,  /* id-list preparation the last msched_migrate queued behind its copy (0 if none) */
       MSCHED_N_PHASES = 10 };
/* level 0: off; 1: time each plan as a whole and each migrate (two events per call); 2: also time the
 * four planning phases separately (the extra events between kernels add a few microseconds each). */
int msched_set_profiling(msched_ctx *ctx, int level);
int msched_get_phase_ms(msched_ctx *ctx, float *ms);

/*
 * Early execution (Sec. 6.3: pages migrate in predicted access order, and a kernel starts as soon as the pages
 * it depends on are resident instead of waiting for the whole working set).
 * With early start enabled, msched_plan also computes need[g] for every covered command g: the number of
 * leading fetch-list entries that hold the pages commands 0..g use; and the kernel of msched_migrate
 * publishes `landed`, the number of leading fetch entries that are complete (bytes in the frame, victim's
 * bytes in the host store, page table updated), advancing strictly in list order.  Command g may be
 * submitted once landed >= need[g]; after the migration, landed == n_fetch.
 *   msched_set_early_start   enable != 0 switches it on for later plans and migrations (off by default: the
 *                            in-order bookkeeping costs a fence and a few atomics per copied chunk).
 *   msched_plan_ready_need   need: HOST, covered_launches entries; E_STALE_PLAN unless `plan` is the latest
 *                            plan and was made with early start enabled.
 *   msched_progress          *landed of the latest early migration (0 before the first).  Does not wait for
 *                            the migration: it runs a one-thread kernel on a stream of its own and waits
 *                            for that.  Data of landed entries is visible to kernels launched afterwards.
 */
int msched_set_early_start(msched_ctx *ctx, int enable);
int msched_plan_ready_need(msched_ctx *ctx, const msched_plan_t *plan, uint32_t *need);
int msched_progress(msched_ctx *ctx, uint32_t *landed);

/*
 * The same hand-over without the host in between (Sec. 6.3 signals from the copy to the compute side on the
 * device): msched_gate_enqueue puts a one-wavefront kernel on `stream` (the stream the task's commands are
 * launched on; NOT the context's stream) that returns once landed >= need[g] of the latest plan, so that whatever
 * the caller launches on that stream afterwards - command g - starts when its pages are resident, while the
 * migration is still running on the context's stream.  g < covered_launches; the plan must be the latest one, made
 * with early start enabled, and msched_migrate must already have been called for it (else E_STALE_PLAN: a gate
 * queued ahead of its migration could sit in front of it in a hardware queue the two streams share, and would
 * then hold it up until the gate gives up); call it before the next msched_plan.  The wait is bounded: after timeout_us microseconds (0 = 2 seconds) on the device's wall
 * clock the kernel gives up and returns all the same, and the caller finds that out from msched_gate_result and
 * waits for the migration in the ordinary way (an event on the context's stream) before it launches the command.
 * msched_gate_result reports gate g of the latest plan, as its kernel left it in host memory (synchronise `stream`
 * first): *status 0 = has not finished, 1 = its pages were resident, 2 = gave up; *ready_ms = when it saw them
 * resident, in milliseconds after the migration kernel started (0 if it returned before the migration began, e.g.
 * need[g] == 0).  Either pointer may be NULL.
 */
int msched_gate_enqueue(msched_ctx *ctx, const msched_plan_t *plan, uint32_t g, void *stream, uint32_t timeout_us);
int msched_gate_result(msched_ctx *ctx, uint32_t g, uint32_t *status, float *ready_ms);

/*
 * Offline memory analyzer (Sec. 5.2, "Memory analyzer"): derive access rules from profiled invocations.
 * A batch holds n_kernels kernels, each with n_invocations profiled invocations.  Per invocation: the
 * launch arguments as 64-bit values (32-bit ones zero-extended), and the byte intervals (start, length)
 * the kernel touched: one per region a memory instruction covers, regions that begin at the same address merged;
 * sorted by start, starts distinct; intervals of different buffers may touch or overlap.  All arrays are DEVICE memory, owned by
 * the caller, read only:
 *   n_args      [K]                         arguments per kernel, <= MSCHED_MAX_ARGS
 *   int64_mask  [K]                         bit a set: argument a is a 64-bit integer (a possible pointer)
 *   args        [K][n_inv][MSCHED_MAX_ARGS] argument values (entries >= n_args ignored)
 *   intervals   [K][n_inv][max_intervals][2]
 *   n_intervals [K][n_inv]                  intervals in use, <= max_intervals
 * For each kernel: a 64-bit argument whose value starts a touched interval in every invocation is a base
 * pointer; the region at a base (one interval, or a run of equal intervals at a regular stride that ends
 * at a different length, an irregular gap or another base's address) is matched against T1, T2, T3 in this
 * order, each of size / stride / count as coeff * product of at most three non-pointer arguments with a
 * positive integer coeff; candidates are tried as: no argument, single arguments, pairs, triples, indices
 * ascending, first match wins.  An argument that equals a lower base in every invocation yields no rule.
 * Output (DEVICE, caller-owned): rules [K][MSCHED_MAX_RULES] in ascending base_arg (unused tail untouched),
 * n_rules [K], unexplained [K] = (invocation, interval) pairs that no rule accounts for.  The rules are
 * what msched_kernel_register takes.
 * Limits: 1 <= n_invocations <= 512; 1 <= max_intervals <= 65535; args and intervals 16-byte aligned,
 * rules 8-byte aligned.  The first call on a device also writes a small constant table and waits for it.
 * Asynchronous on `stream`
 * (a hipStream_t, NULL = the default stream).  Errors: MSCHED_E_INVAL (null pointer, limits), MSCHED_E_HIP.
 * Input whose intervals are not sorted by distinct starts gives unspecified rules but no out-of-bounds access.
 */
typedef struct {
    uint32_t n_kernels, n_invocations, max_intervals, reserved;
    const int32_t *n_args;
    const uint32_t *int64_mask;
    const uint64_t *args;
    const uint64_t *intervals;
    const uint32_t *n_intervals;
} msched_profile_batch;                         /* 56 bytes */
int msched_analyze(const msched_profile_batch *batch, msched_rule *rules, uint32_t *n_rules,
                   uint32_t *unexplained, void *stream);

const char *msched_strerror(int code);
int msched_last_hip_error(msched_ctx *ctx);     /* hipError_t of the last MSCHED_E_HIP, as int; ctx may be NULL
                                                    (then: the last one of any context, e.g. a failed create) */

#ifdef __cplusplus
}
#endif
#endif /* MSCHED_H */
