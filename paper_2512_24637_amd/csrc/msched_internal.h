// Internal declarations shared by the HIP translation units of libmsched.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <unordered_map>
#include <vector>

#include "msched.h"

namespace msched {

constexpr uint32_t kNone = 0xFFFFFFFFu;         // not resident / free frame / no next use
constexpr uint32_t kSkip = 0x80000000u;         // output offset of a class that is not emitted
constexpr int kWave = 64;                       // CDNA wavefront
constexpr uint32_t kMaxChunks = 2048;           // page-table chunks (one workgroup each)
constexpr uint32_t kSingleChunkPages = 8192;    // page tables up to this size are swept by one workgroup (one tile)
constexpr uint32_t kMaxBuckets = 4096;          // binned id lists: buckets of 32 Ki pages, counters in LDS
constexpr int kMaxWaves = 8;                    // wavefronts per sweep workgroup
constexpr int kMaxSteps = 16;                   // 64-page steps a wavefront keeps in registers per tile
constexpr uint32_t kNuShift = 12;               // nu entry = (epoch << kNuShift) | (kNuMask - g)
constexpr uint32_t kNuMask = (1u << kNuShift) - 1;
constexpr uint64_t kPtrMask = (1ull << 56) - 1; // record address without the skip mask in its top byte
constexpr uint32_t kMaxEpoch = (1u << (32 - kNuShift)) - 1;
static_assert(MSCHED_MAX_TIMELINE_COMMANDS < kNuMask, "g must fit the next-use encoding");
constexpr uint32_t kRowGroups = 16;             // row groups of the chunk x class count matrix
constexpr uint32_t kOffsetSplit = 8;            // slices of a row group: the column prefixes are taken slice by slice
constexpr uint32_t kSumRows = kRowGroups * (1 + kOffsetSplit);   // rows of per-key sums the first sweep keeps: row groups, then their slices

// status bits raised by device code while planning
constexpr uint32_t kStatRange = 1u;             // a LIST id >= V, or a touched page without backing slot
constexpr uint32_t kStatWset = 2u;              // first command alone exceeds the pool

// A queued launch as the expansion kernel reads it (lives in pinned, device-visible host memory).
struct alignas(16) CmdRec {
    uint32_t kernel, n_args, latency, n_ids;
    const uint32_t *ids;                        // device pointer (caller-owned) or null
    uint64_t reserved;                          // host copy: 0; device copy: mask of rules to skip in this plan
    uint64_t args[MSCHED_MAX_ARGS];
};
static_assert(sizeof(CmdRec) == 128, "CmdRec layout");

struct DevKernel {
    uint32_t n_rules, pad;
    msched_rule rules[MSCHED_MAX_RULES];
};

// Written by the cut kernel; read by later kernels (device copy) and by the host (pinned copy).
struct PlanHeader {
    uint32_t n_fetch, n_evict, n_free_used, g_cut;
    uint32_t n_resident, status, first_free;
    uint32_t seq;       // host copy only: written last, after everything else of the plan that the host reads has been written
};

// What a rule of a queued command describes, as an exact tuple (page range of a fixed / linear rule; the four
// strided parameters; address and length of an id list).
struct RegionSig {
    uint64_t a, b, c, d;
    bool operator==(const RegionSig &o) const { return a == o.a && b == o.b && c == o.c && d == o.d; }
};
struct RegionSigHash {
    size_t operator()(const RegionSig &s) const {
        uint64_t h = s.a * 0x9E3779B97F4A7C15ull ^ (s.b + 0x7F4A7C15ull) * 0xC2B2AE3D27D4EB4Full ^
                     (s.c * 0x165667B19E3779F9ull) ^ (s.d * 0x27D4EB2F165667C5ull);
        return (size_t)(h ^ (h >> 29));
    }
};

// One page range [lo, hi) of a queued command, evaluated when the launch was queued (Sec. 5.2: the predictor
// evaluates the formulas with the launch arguments at launch time).  `back` is the distance, in commands of the
// task, to the latest earlier command one of whose rules described the very same region (0: none): while that
// command is still queued it comes first in every timeline, so this range cannot lower any page's first use and
// a plan leaves it out.  All ranges of one rule share `back`; `cmd` is the command's program-order index in its
// task (low 32 bits: only differences between queued commands are ever taken).
struct RangeRec { uint32_t lo, hi, back, cmd; };
constexpr uint32_t kRuleEmpty = 0xFFFFFFFFu;
constexpr uint8_t kCmdList = 1;                 // the command has a live id list (a LIST rule and at least one id)
constexpr uint8_t kCmdNoPaint = 2;              // its ranges were too many to keep: plans that hold it scatter next uses per page

struct TaskQueue {
    CmdRec *recs = nullptr;                     // pinned host memory: what kernels read of a command (the per-page and binning paths)
    CmdRec *recs_dev = nullptr;                 // same memory, device address
    size_t cap = 0;                             // records allocated
    size_t base = 0;                            // program-order index of recs[0]
    size_t n = 0;                               // commands ever enqueued
    size_t cursor = 0;                          // first command not yet retired
    // What a plan walks: compact arrays in ordinary host memory, entry i - base for command i.  Everything a plan
    // needs of a command was worked out when it was queued; the plan only reads, in order.
    std::vector<uint32_t> lat;                  // profiled latency
    std::vector<uint64_t> range_end;            // the command's ranges have the running indices [range_end[i - 1], range_end[i])
    std::vector<uint32_t> n_ids;
    std::vector<const uint32_t *> ids;          // device pointer (caller-owned) or null
    std::vector<uint32_t> list_back;            // like RangeRec::back, for the id list (same address and length)
    std::vector<uint8_t> flag;                  // kCmdList, kCmdNoPaint
    std::vector<uint32_t> rule_back;            // [MSCHED_MAX_RULES per command] like RangeRec::back, per rule; kRuleEmpty: the rule describes nothing
    std::vector<uint64_t> prep;                 // 1 + ring offset of the command's prepared id list (0 = none)
    // The commands' page ranges in program order: a ring in pinned host memory, the range with running index q at
    // q & (rng_cap - 1), and a mirror of it in device memory that the sweeps of large tables read (brought up to
    // date behind every migration; a plan reads it only when all its ranges are there).  Ranges of retired commands are dead.
    RangeRec *rng = nullptr;                    // pinned host memory [rng_cap]
    RangeRec *rng_dev = nullptr;                // device memory [rng_cap]
    uint64_t rng_cap = 0;                       // a power of two
    uint64_t rng_end = 0;                       // running index behind the last range
    uint64_t rng_uploaded = 0;                  // ranges with a running index below this are in the mirror
    bool want_mirror = false;                   // a plan would have read this task's ranges from a mirror: keep one, filled behind migrations
    uint64_t ranges_base = 0;                   // running index of the first range of command `base`
    std::unordered_map<RegionSig, size_t, RegionSigHash> last_region;   // region -> latest command that described it
    size_t pruned_at = 0;                       // size of last_region after its last clean-up
    // prepared id lists of this task's queued commands: a ring in device memory, filled in program order
    uint8_t *prep_buf = nullptr;
    uint64_t prep_size = 0, prep_head = 0, prep_tail = 0;   // head / tail are running byte offsets (never wrap)
    size_t prep_scan = 0;                       // commands before this index have been looked at by the look-ahead preparation
    uint64_t range_begin(size_t i) const { return i == base ? ranges_base : range_end[i - base - 1]; }
    uint64_t ranges_live_from() const { return cursor == n ? rng_end : range_begin(cursor); }   // the oldest range still needed
    const RangeRec &range_at(uint64_t q) const { return rng[q & (rng_cap - 1)]; }
};

// A run of one timeline entry: commands [first, first + count) of `task` take the positions g0, g0 + 1, ...
// What a gate kernel (msched_gate_enqueue) reports: status 1 = pages resident, 2 = gave up; the fetch entries it saw
// landed; 100 MHz ticks from the start of the migration kernel to that moment (0 if the migration had not begun).
struct GateRec { uint32_t status, seen; uint64_t ticks; };

struct PlanRun { uint32_t task, g0, count; size_t first; };

// The ranges of a plan as the sweeps of large tables read them when nothing is staged: for each run of the flattened
// timeline the slice of its task's range mirror, and what turns an entry into a range of this plan (the command's
// position g = g0 + (cmd - cmd_first); a range that repeats a region of a command still queued - cmd - back at or
// behind the task's cursor - is left out).  Wavefront w of a sweep workgroup serves run w mod n for the whole
// launch, so it reads the run's description once, into scalar registers, and an entry then costs one load at an
// address worked out by arithmetic alone (anything looked up per entry - a run table in LDS or in the argument
// buffer - was measured at 0.5 us and more per row of 64 entries, several times the cost of the range test itself).
// The table travels in the launch's arguments; plans with more runs than a workgroup has wavefronts list their
// ranges on the host instead.
constexpr uint32_t kMaxRangeRuns = 16;
constexpr uint32_t kRangeRow = 64;
struct RangeRun {
    const RangeRec *ring;
    uint32_t mask, first;          // range k of the run is ring[(first + k) & mask]
    uint32_t count;                // ranges
    uint32_t cmd_first, g0, cursor;
    uint32_t dedupe;
    uint32_t share;                // set at launch, per wavefront: its rank among the wavefronts that serve the run | their number << 16
    uint32_t passes;               // set at launch: passes of kRangesPerThread rows per wavefront that cover the longest run
    uint32_t pad[5];
};
static_assert(sizeof(RangeRun) == 64, "a line of the table");
// What a launch carries: the runs, copied out once more per wavefront of a workgroup (entry w is the run wavefront w
// serves, with its share of it), so that a wavefront finds its 64-byte line of the table without having read
// anything else.
struct alignas(64) RangeRuns {
    uint32_t n;                    // runs (host side)
    uint32_t pad[15];
    RangeRun run[kMaxRangeRuns];   // by run (host side); by wavefront in the copy a launch carries
};
static_assert(sizeof(RangeRuns) == 64 + 64 * kMaxRangeRuns, "RangeRuns layout");
constexpr uint32_t kStagePieces = 512;      // segments of a bucket described in LDS at a time (16 bytes each)
constexpr uint32_t kRangesPerThread = 4;    // ranges a thread tests per pass over a plan's ranges

// One source of the id-list merge: a prepared (de-duplicated, grouped by bucket) piece of a command's list.
// A piece is prepared in `split` parts (prep_split), each by a workgroup of its own, part q taking the buckets
// q, q + split, q + 2 split, ... (every workgroup reads the whole piece and keeps the ids of its
// buckets): part q of the piece starts at block + q * part_words and holds
//   part[0] = 1 if the part saw an id it cannot plan (out of range - reported by part 0 - or without backing slot)
//   part[1 .. Bq + 1] = start of each of its buckets' ids (exclusive prefix, last = total), Bq = buckets per part
//   part[Bq + 2 ..] = the ids (room for every id of the piece)
struct ListSource { const uint32_t *block; uint32_t g, part_words; };
// A piece still to be prepared: n ids of a command's list, and where its block goes.
struct ListPrep { const uint32_t *ids; uint32_t *block; uint32_t n, pad[3]; };
constexpr uint32_t kMaxPrepSplit = 8;
// parts a piece is prepared in: at least 16 buckets per part, at most `most` parts (MSCHED_PREP_SPLIT)
inline uint32_t prep_split(uint32_t n_buckets, uint32_t most) {
    const uint32_t s = n_buckets / 16;
    return s < 1 ? 1u : (s > most ? most : s);
}
__host__ __device__ inline uint32_t prep_part_buckets(uint32_t n_buckets, uint32_t split) { return (n_buckets + split - 1) / split; }
// 32-bit words of one part of a piece of n ids
__host__ __device__ inline uint32_t prep_part_words(uint32_t n_buckets, uint32_t split, uint32_t n) {
    return prep_part_buckets(n_buckets, split) + 2 + n;
}
constexpr uint32_t kMaxListSources = 4096;
constexpr uint32_t kBucketShift = 13;           // id lists are grouped by bucket of this many (log2) consecutive pages
constexpr uint32_t kPrepBlock = 24576;          // ids per prepared piece (24 per thread of the workgroup that prepares it, in registers)

// A page range [lo, hi) first used by command g: what a fixed / linear rule, or one chunk of a strided
// rule, describes once its formulas are evaluated.
struct PageRange { uint32_t lo, hi, g, pad; };
constexpr uint32_t kMaxRanges = 4096;           // more ranges than this in one plan: next use is scattered per page instead
constexpr uint32_t kMaxResidentRanges = 4 * kMaxRanges;   // ... read from the mirrors, where repeats count until the reader drops them

struct PlanGeom {
    uint32_t G, g_end0, n_chunks, chunk_pages, n_keys;   // n_keys = 2 * (G + 1)
    uint32_t waves, steps, rounds;                       // sweep workgroup shape
    bool single;                                         // one workgroup sweeps the whole table (fused tail kernel)
    bool list_binned;                                    // id lists go through the bucket path
    bool list_prepared;                                  // ... from per-command prepared pieces (cached across plans)
    uint32_t n_list_sources, n_list_new;                 // pieces merged by this plan; of those, prepared by it
    uint32_t n_buckets, bucket_cap;                      // bucket_cap: pairs per sub-segment
    uint32_t split;                                      // parts a prepared piece consists of
    bool live_list;                                      // some command of the plan brings an id list that is not a repeat
    bool needs_records;                                  // some kernel of the plan reads whole command records (table of record addresses filled)
    bool painted;                                        // range rules arrive as a range list the sweeps paint into LDS
    bool resident;                                       // ... which the sweeps read from the tasks' range mirrors (nothing staged)
    bool use_nu;                                         // some next uses are in nu[] (id lists, or the scatter path)
    uint32_t n_ranges;
};

}  // namespace msched

struct msched_ctx {
    msched_config cfg;
    hipStream_t stream;
    int device = 0;                             // the GPU that was current at msched_create
    uint64_t V;
    uint32_t F, page_shift;
    void *host_dev = nullptr;                   // device address of cfg.host_store
    uint32_t migrate_chunk_shift = 21;          // bytes a workgroup moves per work unit (log2), at most a page
    uint32_t migrate_ticket = 0;                // hand work units out from a counter instead of dealing them round-robin
    uint32_t early_chunk_shift = 16;            // the same under early execution: small, so that entries complete in list order
    uint32_t migrate_max_blocks = 512;          // grid cap of the copy kernel (two workgroups per CU measured best)
    uint32_t migrate_hints = 0;                 // bit 0: plain host stores, bit 1: plain host loads (default: non-temporal)
    uint32_t expand_split = 0;                  // workgroups per (command, rule); 0 = by page-table size
    uint32_t max_chunks = msched::kMaxChunks;   // page-table chunks (sweep workgroups) at most
    uint32_t stage_threshold = 2048;            // expansion workgroups above which records are staged first
    bool dedupe_regions = true;                 // leave out rules that repeat a region an earlier queued command of the task describes
    std::vector<msched::PlanRun> runs;          // the flattened timeline of the plan being made, one run per entry
    msched::RangeRuns range_runs{};             // the same runs as slices of the tasks' range mirrors (plans that stage nothing)
    // The tasks' mirrors are small and every sweep workgroup reads several of them at once: carved out of one
    // allocation they share its pages and address translations.  A mirror that outgrows the arena gets memory of its own.
    uint8_t *mirror_arena = nullptr;
    size_t mirror_arena_used = 0;
    std::vector<size_t> pos;                    // per task: next command the flattening takes
    struct Reserved { uint32_t task; size_t cmd; uint64_t head; };
    std::vector<Reserved> reserved;             // ring blocks this plan handed out for id lists it prepares itself (undone if it fails)
    bool force_multi_kernel = false;            // test hook: never use the fused single-workgroup tail
    bool no_large_lds = false;                  // MSCHED_NO_LARGE_LDS: never ask for more than the default dynamic LDS
    bool has_list_rule = false;                 // some registered kernel has a LIST rule
    // binned id lists (allocated on first use)
    uint32_t *list_bucket_fill = nullptr;       // [kMaxBuckets][8]
    uint32_t *list_pairs = nullptr; size_t list_cap = 0;   // n_buckets x 8 x bucket_cap
    uint64_t list_binned_min_ids = 262144;      // plans with at least this many ids take the bucket path
    uint32_t list_prepared = 1;                 // 0: bin every plan's ids from scratch (MSCHED_LIST_PREPARED)
    uint32_t prep_split_max = 1;                // parts (workgroups) an id-list piece is prepared in, at most (MSCHED_PREP_SPLIT)
    uint64_t list_cache_bytes = 128ull << 20;   // ring of prepared pieces per task (MSCHED_LIST_CACHE_MB)
    msched::ListSource *list_src_host = nullptr;   // pinned [kMaxListSources]: the pieces this plan merges
    msched::ListSource *list_src_dev = nullptr;    // the same memory, device address
    msched::ListPrep *list_prep_host = nullptr;    // pinned [kMaxListSources]: the pieces this plan has to prepare first
    msched::ListPrep *list_prep_dev = nullptr;
    uint32_t *bucket_mark = nullptr;               // device [kMaxBuckets]: buckets some prepared piece has put an id in; then [kMaxChunks] chunk order
    msched::ListSource *list_src_stage = nullptr;  // device copy of the source table (every merge workgroup reads it)
    // look-ahead preparation: id lists of queued commands are binned behind a migration, off the plan's path
    uint32_t list_ahead = 128;                     // commands per task looked ahead at each migration (MSCHED_LIST_AHEAD, 0 = off)
    msched::ListPrep *list_ahead_host = nullptr;   // pinned [kMaxListSources]
    msched::ListPrep *list_ahead_dev = nullptr;
    hipEvent_t ahead_ev = nullptr; bool ahead_pending = false;   // the last look-ahead kernel still reads the table
    bool last_plan_prepared = false;               // the latest plan merged prepared pieces
    std::vector<uint8_t> kernel_has_list;          // per registered kernel
    uint32_t list_b0 = 4, list_b1 = 32;         // id lists: commands [0,b0), [b0,b1), [b1,G) run as ordered batches
    uint32_t *page_table = nullptr, *frame_owner = nullptr, *nu = nullptr, *slot = nullptr;  // device
    uint32_t *evict_pages = nullptr, *evict_frames = nullptr, *fetch_pages = nullptr, *fetch_frames = nullptr;
    uint32_t *flags = nullptr;                  // device status word
    uint32_t *matrix = nullptr; size_t matrix_cap = 0;       // [n_chunks][n_keys] counts; behind them [matrix_cap...) the chunks' start positions
    uint32_t *chunk_hint = nullptr;                          // [3][kMaxChunks]: what the first sweep saw per chunk for the second; the second sweep's chunk order;
                                                             // how a chunk's ranges were painted by the last plans (SweepGeom::paint_hint)
    uint32_t *partial = nullptr;                             // [kSumRows][n_keys] sums by row group, then by slice; all zero between plans
    uint32_t *offsets = nullptr;                // [2 * (MAX_G + 1)] per-class output offsets
    msched::PlanHeader *hdr_dev = nullptr;      // device
    msched::PlanHeader *hdr_host = nullptr;     // pinned
    const msched::CmdRec **cmd_ptrs_host = nullptr;          // pinned: record of the g-th future command
    const msched::CmdRec *const *cmd_ptrs_dev = nullptr;     // same memory, device address
    msched::CmdRec *cmd_dev = nullptr;                       // device: this plan's records, in g order
    uint32_t epoch = 0;                                      // next-use epoch of the latest plan
    msched::DevKernel *kernels_dev = nullptr; size_t kernels_cap = 0;
    std::vector<msched::DevKernel> kernels;
    std::vector<msched::TaskQueue> tasks;
    uint32_t max_rules = 0;
    uint32_t n_resident = 0;
    uint64_t plan_seq = 0, pending_plan = 0;    // pending_plan == 0: nothing to migrate
    msched::PlanHeader pending{};
    uint32_t *query_buf = nullptr; size_t query_cap = 0;     // device scratch for pagetable_query
    // early execution: in-order landing of the fetch list
    // range list of the latest plan (painted path)
    msched::PageRange *ranges_host = nullptr;   // pinned [kMaxRanges], written by the timeline flatten
    msched::PageRange *ranges_host_dev = nullptr;   // the same memory, device address
    msched::PageRange *ranges_dev = nullptr;    // device copy for sweeps of many workgroups
    uint16_t *key16 = nullptr;                  // device [V]: class key of every page (first sweep -> second sweep)
    uint32_t paint = 1;                         // 0: always scatter next uses per page (MSCHED_PAINT)
    uint32_t resident_ranges = 1;               // 0: every plan copies its range list to the device (MSCHED_RESIDENT_RANGES)
    int early = 0;                              // msched_set_early_start
    uint32_t *need_host = nullptr;              // pinned [MAX_G + 1]: need[g] of the latest plan (written by the cut kernel)
    uint32_t *page_done = nullptr;              // device [F]: tag of the migration that completed fetch entry i
    uint32_t *chunks_done = nullptr;            // device [F]: chunks of entry i copied so far (zero between migrations)
    uint32_t *landed = nullptr;                 // device: [0] leading fetch entries complete, [1] work units handed out,
                                                // [2..3] wall clock at which the latest early migration kernel started (0: not yet)
    msched::GateRec *gate_host = nullptr;       // pinned [MAX_G + 1]: what the gate kernel of command g left behind
    uint32_t *progress_host = nullptr;          // pinned: where msched_progress reads `landed` into
    hipStream_t poll_stream = nullptr;          // msched_progress works here, beside the migration
    uint32_t early_tag = 0;                     // nonzero tag of the latest early migration
    uint32_t hdr_seq = 0;                       // stamp of the header the host is waiting for (never 0)
    uint32_t order_emit = 1;                    // the second sweep takes the chunks it may have to list pages of first (MSCHED_ORDER_EMIT)
    uint32_t fuse_lists = 1;                    // prepared id lists are merged inside the first sweep (MSCHED_FUSE_LISTS, 0 = own kernel)
    uint32_t plan_spin = 1;                     // msched_plan returns when the counts have landed, not when the lists are complete
    bool plan_timing_pending = false;           // device times of the last plan have not been read from their events yet
    bool early_ready = false;                   // every piece of the early-execution bookkeeping exists
    int plan_early = 0;                         // the latest plan computed need[] and reset landed
    int profiling = 0;
    int migrate_timed = 0;                      // ev[5], ev[6] have been recorded
    int prepare_timed = 0;                      // ev[8], ev[9] have been recorded around the look-ahead preparation of the last migrate
    hipEvent_t ev[10] = {};
    float phase_ms[MSCHED_N_PHASES] = {};
    int last_hip = 0;
};

namespace msched {

// plan kernels (msched_plan.hip)
hipError_t launch_plan(msched_ctx *c, const PlanGeom &g);
hipError_t launch_nu_reset(msched_ctx *c);
void plan_geometry(const msched_ctx *c, uint32_t G, PlanGeom &g);
// migrate + query kernels (msched_migrate.hip)
hipError_t launch_migrate(msched_ctx *c, const PlanHeader &h);
hipError_t launch_query(msched_ctx *c, const uint32_t *ids_dev, uint32_t n, uint32_t *out_dev);
hipError_t launch_init_tables(msched_ctx *c);
hipError_t query_scratch_init(uint8_t **out);                                         // address of the static staging array on the current device
hipError_t query_static(msched_ctx *c, const uint64_t *page_ids, uint32_t n, uint32_t *out);
hipError_t launch_peek(msched_ctx *c);
hipError_t launch_gate(msched_ctx *c, uint32_t g, uint32_t need, uint64_t timeout_ticks, hipStream_t stream);
hipError_t launch_list_prepare(msched_ctx *c, const ListPrep *table_dev, uint32_t n, uint32_t n_buckets, uint32_t split);
//      // landed -> progress_host on the poll stream

extern int g_last_hip;                        // hipError_t of the last failed HIP call of any context

}  // namespace msched
