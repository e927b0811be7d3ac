/*
 * msched_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, single-threaded, deliberately slow CPU statement of what MSched's
 * proactive memory scheduling computes at one context switch, written from the
 * paper (arXiv 2512.24637).  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no code, header, table or helper with
 * the HIP library; the two are compared on the same seeded inputs.
 *
 * What each part follows:
 *   expansion   Sec. 5.2 "Access pattern templates" (T1 fixed, T2 linear, T3
 *               strided: base pointer argument + extent that is a coefficient
 *               times a product of launch arguments) and "Memory access
 *               prediction" (regions are aligned to page boundaries).  The
 *               result has a plain definition -- the set of pages overlapped by
 *               the described byte ranges -- and is computed as exactly that.
 *   flatten     Sec. 6.1 "Task scheduling timeline" + Sec. 6.2 "Distributed
 *               metadata management": the timeline (ordered task entries with
 *               timeslices) and each task's queue of (command, latency) resolve
 *               the global order of future commands.
 *   next use    Sec. 6.2 "Enforcing the OPT memory scheduling": the eviction
 *               order is the reverse of the access order (Belady).  Here every
 *               page gets the position of the first future command touching it;
 *               pages untouched by the timeline come first in eviction order.
 *   migrate     Sec. 6.2 "Driver support" (evict from the head of the eviction
 *               order until enough space is free, then populate the next task's
 *               working set) and Sec. 6.3 (unmap, copy out, copy in, map; target
 *               i lands in the space reclaimed from victim i).
 *
 * Readings taken where the paper is silent (each is listed in the design
 * notes): command-granular next use; ties broken by lowest page id; a timeslice
 * whose working set exceeds the pool is cut to its longest fitting command
 * prefix; a command belongs to the timeslice in which it starts; fetched pages
 * take free frames in ascending order first, then the victims' frames in
 * eviction order; every eviction copies the page back (no dirty tracking).
 *
 * Pins (tests/test_oracle_*.py): brute-force optimal fetch counts on tiny
 * caches, textbook MIN on one-page commands, the paper's three-task eviction
 * order example, a hand-derived periodic steady state, byte-marking brute force
 * for the expander, content round trips.  The per-switch lists of a one-round
 * horizon have no published value: parity unpinned beyond those.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define NONE32 0xFFFFFFFFu   /* page not resident / frame free / no next use */

enum { E_OK = 0, E_INVAL = -1, E_RANGE = -2, E_OVERFLOW = -3, E_WSET = -4, E_STALE = -5, E_NOMEM = -6 };
enum { K_FIXED = 1, K_LINEAR = 2, K_STRIDED = 3, K_LIST = 4 };
enum { F_SIZE = 0, F_STRIDE = 1, F_COUNT = 2 };

typedef struct {
    int kind, base_arg;
    int n_idx[3];
    int idx[3][4];
    uint64_t coeff[3];
} rule_t;

typedef struct { int n_rules; rule_t rules[8]; } kernel_t;

typedef struct {
    uint32_t kernel, n_args, latency, n_ids;
    uint64_t args[12];
    uint32_t *ids;            /* private copy */
} cmd_t;

typedef struct { cmd_t *cmds; size_t n, cap, cursor; } task_t;

typedef struct { uint32_t *v; size_t n, cap; } vec32;

typedef struct {
    int page_shift;
    uint64_t V;
    uint32_t F;
    uint32_t *page_table;     /* [V] frame or NONE32 */
    uint32_t *frame_owner;    /* [F] page or NONE32 */
    const uint32_t *host_slot;/* [V] or NULL = identity */
    uint64_t n_slots;
    uint8_t *pool, *host;     /* caller-owned byte images; NULL = metadata only */
    kernel_t *kernels; size_t n_kernels, cap_kernels;
    task_t *tasks; size_t n_tasks, cap_tasks;
    /* last plan */
    int plan_pending;
    uint32_t mig_done;                 /* fetch entries already carried out by orc_migrate_prefix */
    uint32_t n_fetch, n_evict, n_free_used, g_cut, g_end0, G;
    vec32 fetch_pages, fetch_frames, evict_pages, evict_frames;
    uint32_t *nu;             /* [V] scratch */
} orc_t;

static int push32(vec32 *a, uint32_t x) {
    if (a->n == a->cap) {
        size_t nc = a->cap ? a->cap * 2 : 1024;
        uint32_t *nv = (uint32_t *)realloc(a->v, nc * sizeof(uint32_t));
        if (!nv) return E_NOMEM;
        a->v = nv; a->cap = nc;
    }
    a->v[a->n++] = x;
    return E_OK;
}

orc_t *orc_create(int page_shift, uint64_t V, uint32_t F, const uint32_t *host_slot,
                  uint64_t n_slots, uint8_t *pool, uint8_t *host) {
    if (page_shift < 1 || page_shift > 30 || V == 0 || V >= NONE32 || F == 0) return NULL;
    orc_t *o = (orc_t *)calloc(1, sizeof(orc_t));
    if (!o) return NULL;
    o->page_shift = page_shift; o->V = V; o->F = F;
    o->host_slot = host_slot; o->n_slots = host_slot ? n_slots : V;
    o->pool = pool; o->host = host;
    o->page_table = (uint32_t *)malloc(V * sizeof(uint32_t));
    o->frame_owner = (uint32_t *)malloc((size_t)F * sizeof(uint32_t));
    o->nu = (uint32_t *)malloc(V * sizeof(uint32_t));
    if (!o->page_table || !o->frame_owner || !o->nu) return NULL;
    for (uint64_t p = 0; p < V; p++) o->page_table[p] = NONE32;
    for (uint32_t f = 0; f < F; f++) o->frame_owner[f] = NONE32;
    return o;
}

void orc_destroy(orc_t *o) {
    if (!o) return;
    for (size_t t = 0; t < o->n_tasks; t++) {
        for (size_t i = 0; i < o->tasks[t].n; i++) free(o->tasks[t].cmds[i].ids);
        free(o->tasks[t].cmds);
    }
    free(o->tasks); free(o->kernels); free(o->page_table); free(o->frame_owner); free(o->nu);
    free(o->fetch_pages.v); free(o->fetch_frames.v); free(o->evict_pages.v); free(o->evict_frames.v);
    free(o);
}

/* Rules arrive as flat arrays: kind[n], base_arg[n], n_idx[n][3], idx[n][3][4], coeff[n][3]
 * with field order size, stride, count. */
int orc_kernel_register(orc_t *o, int n_rules, const int *kind, const int *base_arg,
                        const int *n_idx, const int *idx, const uint64_t *coeff) {
    if (n_rules < 0 || n_rules > 8) return E_INVAL;
    kernel_t k; memset(&k, 0, sizeof k);
    k.n_rules = n_rules;
    for (int r = 0; r < n_rules; r++) {
        rule_t *q = &k.rules[r];
        if (kind[r] < K_FIXED || kind[r] > K_LIST) return E_INVAL;
        q->kind = kind[r]; q->base_arg = base_arg[r];
        for (int f = 0; f < 3; f++) {
            q->n_idx[f] = n_idx[r * 3 + f];
            if (q->n_idx[f] < 0 || q->n_idx[f] > 4) return E_INVAL;
            for (int j = 0; j < 4; j++) q->idx[f][j] = idx[(r * 3 + f) * 4 + j];
            q->coeff[f] = coeff[r * 3 + f];
        }
        if (q->kind == K_FIXED && q->n_idx[F_SIZE] != 0) return E_INVAL;
    }
    if (o->n_kernels == o->cap_kernels) {
        size_t nc = o->cap_kernels ? o->cap_kernels * 2 : 16;
        kernel_t *nk = (kernel_t *)realloc(o->kernels, nc * sizeof(kernel_t));
        if (!nk) return E_NOMEM;
        o->kernels = nk; o->cap_kernels = nc;
    }
    o->kernels[o->n_kernels] = k;
    return (int)o->n_kernels++;
}

int orc_task_create(orc_t *o) {
    if (o->n_tasks == o->cap_tasks) {
        size_t nc = o->cap_tasks ? o->cap_tasks * 2 : 8;
        task_t *nt = (task_t *)realloc(o->tasks, nc * sizeof(task_t));
        if (!nt) return E_NOMEM;
        o->tasks = nt; o->cap_tasks = nc;
    }
    memset(&o->tasks[o->n_tasks], 0, sizeof(task_t));
    return (int)o->n_tasks++;
}

/* value = coeff * product of the named launch arguments (empty product = 1). */
static int formula(const rule_t *q, int f, const cmd_t *c, uint64_t *out) {
    uint64_t v = q->coeff[f];
    for (int j = 0; j < q->n_idx[f]; j++) {
        int a = q->idx[f][j];
        if (a < 0 || (uint32_t)a >= c->n_args) return E_RANGE;
        if (__builtin_mul_overflow(v, c->args[a], &v)) return E_OVERFLOW;
    }
    *out = v;
    return E_OK;
}

/* Pages overlapped by bytes [a, a+len): floor(a/P) .. floor((a+len-1)/P). */
static int touch_bytes(const orc_t *o, uint64_t a, uint64_t len, vec32 *pages) {
    if (len == 0) return E_OK;
    uint64_t last;
    if (__builtin_add_overflow(a, len - 1, &last)) return E_OVERFLOW;
    uint64_t p0 = a >> o->page_shift, p1 = last >> o->page_shift;
    if (p1 >= o->V) return E_RANGE;
    for (uint64_t p = p0; p <= p1; p++) {
        if (o->host_slot && o->host_slot[p] == NONE32) return E_RANGE;
        int rc = push32(pages, (uint32_t)p);
        if (rc) return rc;
    }
    return E_OK;
}

static int cmp_u32(const void *a, const void *b) {
    uint32_t x = *(const uint32_t *)a, y = *(const uint32_t *)b;
    return (x > y) - (x < y);
}

/* The page set of one command: union over its kernel's rules, ascending, no repeats. */
static int expand_command(const orc_t *o, const cmd_t *c, vec32 *pages) {
    pages->n = 0;
    const kernel_t *k = &o->kernels[c->kernel];
    for (int r = 0; r < k->n_rules; r++) {
        const rule_t *q = &k->rules[r];
        int rc;
        if (q->kind == K_LIST) {
            for (uint32_t i = 0; i < c->n_ids; i++) {
                uint32_t p = c->ids[i];
                if (p >= o->V) return E_RANGE;
                if (o->host_slot && o->host_slot[p] == NONE32) return E_RANGE;
                if ((rc = push32(pages, p))) return rc;
            }
            continue;
        }
        if (q->base_arg < 0 || (uint32_t)q->base_arg >= c->n_args) return E_RANGE;
        uint64_t base = c->args[q->base_arg], size;
        if ((rc = formula(q, F_SIZE, c, &size))) return rc;
        if (q->kind == K_FIXED || q->kind == K_LINEAR) {
            if ((rc = touch_bytes(o, base, size, pages))) return rc;
        } else {
            uint64_t stride, count;
            if ((rc = formula(q, F_STRIDE, c, &stride))) return rc;
            if ((rc = formula(q, F_COUNT, c, &count))) return rc;
            if (size == 0) continue;
            for (uint64_t j = 0; j < count; j++) {
                uint64_t off, a;
                if (__builtin_mul_overflow(j, stride, &off)) return E_OVERFLOW;
                if (__builtin_add_overflow(base, off, &a)) return E_OVERFLOW;
                if ((rc = touch_bytes(o, a, size, pages))) return rc;
            }
        }
    }
    qsort(pages->v, pages->n, sizeof(uint32_t), cmp_u32);
    size_t w = 0;
    for (size_t i = 0; i < pages->n; i++)
        if (w == 0 || pages->v[i] != pages->v[w - 1]) pages->v[w++] = pages->v[i];
    pages->n = w;
    return E_OK;
}

int orc_launch_enqueue(orc_t *o, uint32_t task, uint32_t kernel, const uint64_t *args, uint32_t n_args,
                       uint32_t latency, const uint32_t *ids, uint32_t n_ids) {
    if (task >= o->n_tasks || kernel >= o->n_kernels || n_args > 12) return E_INVAL;
    if (n_ids && !ids) return E_INVAL;
    cmd_t c; memset(&c, 0, sizeof c);
    c.kernel = kernel; c.n_args = n_args; c.latency = latency; c.n_ids = n_ids;
    for (uint32_t i = 0; i < n_args; i++) c.args[i] = args[i];
    if (n_ids) {
        c.ids = (uint32_t *)malloc((size_t)n_ids * sizeof(uint32_t));
        if (!c.ids) return E_NOMEM;
        memcpy(c.ids, ids, (size_t)n_ids * sizeof(uint32_t));
    }
    vec32 tmp = {0, 0, 0};
    int rc = expand_command(o, &c, &tmp);     /* reject unusable launches at the door */
    free(tmp.v);
    if (rc) { free(c.ids); return rc; }
    task_t *t = &o->tasks[task];
    if (t->n == t->cap) {
        size_t nc = t->cap ? t->cap * 2 : 64;
        cmd_t *nv = (cmd_t *)realloc(t->cmds, nc * sizeof(cmd_t));
        if (!nv) { free(c.ids); return E_NOMEM; }
        t->cmds = nv; t->cap = nc;
    }
    t->cmds[t->n++] = c;
    return E_OK;
}

int orc_launch_retire(orc_t *o, uint32_t task, uint32_t n) {
    if (task >= o->n_tasks) return E_INVAL;
    task_t *t = &o->tasks[task];
    if (t->cursor + n > t->n) return E_RANGE;
    t->cursor += n;
    return E_OK;
}

/* Pages of a queued command (absolute index in the task's program order). Returns the
 * count, or a negative error; writes at most cap ids. */
int64_t orc_command_pages(orc_t *o, uint32_t task, uint64_t index, uint32_t *out, uint64_t cap) {
    if (task >= o->n_tasks || index >= o->tasks[task].n) return E_INVAL;
    vec32 tmp = {0, 0, 0};
    int rc = expand_command(o, &o->tasks[task].cmds[index], &tmp);
    if (rc) { free(tmp.v); return rc; }
    for (size_t i = 0; i < tmp.n && i < cap; i++) out[i] = tmp.v[i];
    int64_t n = (int64_t)tmp.n;
    free(tmp.v);
    return n;
}

typedef struct { uint32_t nu, page; } sortkey_t;

static int cmp_fetch(const void *a, const void *b) {      /* next use ascending, then page id */
    const sortkey_t *x = (const sortkey_t *)a, *y = (const sortkey_t *)b;
    if (x->nu != y->nu) return x->nu < y->nu ? -1 : 1;
    return (x->page > y->page) - (x->page < y->page);
}

static int cmp_victim(const void *a, const void *b) {     /* next use descending (never = first), then page id */
    const sortkey_t *x = (const sortkey_t *)a, *y = (const sortkey_t *)b;
    if (x->nu != y->nu) return x->nu > y->nu ? -1 : 1;
    return (x->page > y->page) - (x->page < y->page);
}

/* One context switch: decide what to evict and what to fetch.  State is not changed. */
int orc_plan(orc_t *o, const uint32_t *tl_task, const uint32_t *tl_slice, uint32_t n_entries) {
    o->plan_pending = 0;
    o->mig_done = 0;
    for (uint32_t e = 0; e < n_entries; e++) if (tl_task[e] >= o->n_tasks) return E_INVAL;

    /* 1. Flatten the timeline into the global order of future commands. */
    size_t *pos = (size_t *)malloc((o->n_tasks + 1) * sizeof(size_t));
    size_t total = 0;
    for (size_t t = 0; t < o->n_tasks; t++) { pos[t] = o->tasks[t].cursor; total += o->tasks[t].n - pos[t]; }
    const cmd_t **seq = (const cmd_t **)malloc((total + 1) * sizeof(cmd_t *));
    uint32_t G = 0, g_end0 = 0;
    for (uint32_t e = 0; e < n_entries; e++) {
        task_t *t = &o->tasks[tl_task[e]];
        uint64_t elapsed = 0;
        while (pos[tl_task[e]] < t->n && elapsed < tl_slice[e]) {   /* a command runs in the slice it starts in */
            seq[G++] = &t->cmds[pos[tl_task[e]]];
            elapsed += t->cmds[pos[tl_task[e]]].latency;
            pos[tl_task[e]]++;
        }
        if (e == 0) g_end0 = G;
    }
    free(pos);

    /* 2-3. Next use of every page = position of the first command that touches it. */
    uint32_t *nu = o->nu;
    for (uint64_t p = 0; p < o->V; p++) nu[p] = NONE32;
    vec32 pages = {0, 0, 0};
    for (uint32_t g = 0; g < G; g++) {
        int rc = expand_command(o, seq[g], &pages);
        if (rc) { free(pages.v); free(seq); return rc; }
        for (size_t i = 0; i < pages.n; i++)
            if (g < nu[pages.v[i]]) nu[pages.v[i]] = g;
    }
    free(pages.v); free(seq);

    /* 4. The incoming task's timeslice, cut to the longest command prefix whose pages fit the pool. */
    uint32_t g_cut = g_end0;
    for (;;) {
        uint64_t distinct = 0;
        for (uint64_t p = 0; p < o->V; p++) if (nu[p] < g_cut) distinct++;
        if (distinct <= o->F) break;
        g_cut--;
    }
    if (g_end0 > 0 && g_cut == 0) return E_WSET;

    /* 5. Fetch list: wanted, not resident; in order of use. */
    size_t n_fetch = 0, n_cand = 0, n_free = 0;
    sortkey_t *fk = (sortkey_t *)malloc((o->V + 1) * sizeof(sortkey_t));
    sortkey_t *vk = (sortkey_t *)malloc((o->V + 1) * sizeof(sortkey_t));
    if (!fk || !vk) { free(fk); free(vk); return E_NOMEM; }
    for (uint64_t p = 0; p < o->V; p++) {
        int wanted = nu[p] < g_cut, resident = o->page_table[p] != NONE32;
        if (wanted && !resident) { fk[n_fetch].nu = nu[p]; fk[n_fetch].page = (uint32_t)p; n_fetch++; }
        if (!wanted && resident) { vk[n_cand].nu = nu[p]; vk[n_cand].page = (uint32_t)p; n_cand++; }
    }
    qsort(fk, n_fetch, sizeof(sortkey_t), cmp_fetch);

    /* 6-7. Evict only as many as the fetches need beyond the free frames; farthest next use first. */
    vec32 free_frames = {0, 0, 0};
    for (uint32_t f = 0; f < o->F; f++) if (o->frame_owner[f] == NONE32) { push32(&free_frames, f); n_free++; }
    size_t n_evict = n_fetch > n_free ? n_fetch - n_free : 0;
    qsort(vk, n_cand, sizeof(sortkey_t), cmp_victim);
    if (n_evict > n_cand) { free(fk); free(vk); free(free_frames.v); return E_INVAL; }

    /* 8. Frames: free ones lowest first, then the victims' frames in eviction order. */
    o->fetch_pages.n = o->fetch_frames.n = o->evict_pages.n = o->evict_frames.n = 0;
    for (size_t i = 0; i < n_evict; i++) {
        push32(&o->evict_pages, vk[i].page);
        push32(&o->evict_frames, o->page_table[vk[i].page]);
    }
    size_t used_free = n_fetch < n_free ? n_fetch : n_free;
    for (size_t i = 0; i < n_fetch; i++) {
        push32(&o->fetch_pages, fk[i].page);
        push32(&o->fetch_frames, i < used_free ? free_frames.v[i] : o->evict_frames.v[i - used_free]);
    }
    free(fk); free(vk); free(free_frames.v);
    o->n_fetch = (uint32_t)n_fetch; o->n_evict = (uint32_t)n_evict; o->n_free_used = (uint32_t)used_free;
    o->g_cut = g_cut; o->g_end0 = g_end0; o->G = G;
    o->plan_pending = 1;
    return E_OK;
}

/* out[0..6] = n_fetch, n_evict, n_free_used, g_cut, g_end0, G, covered_launches */
int orc_plan_counts(const orc_t *o, uint32_t *out) {
    if (!o->plan_pending) return E_STALE;
    out[0] = o->n_fetch; out[1] = o->n_evict; out[2] = o->n_free_used;
    out[3] = o->g_cut; out[4] = o->g_end0; out[5] = o->G; out[6] = o->g_cut;
    return E_OK;
}

int orc_plan_lists(const orc_t *o, uint32_t *evict_pages, uint32_t *evict_frames,
                   uint32_t *fetch_pages, uint32_t *fetch_frames) {
    if (!o->plan_pending) return E_STALE;
    memcpy(evict_pages, o->evict_pages.v, o->n_evict * sizeof(uint32_t));
    memcpy(evict_frames, o->evict_frames.v, o->n_evict * sizeof(uint32_t));
    memcpy(fetch_pages, o->fetch_pages.v, o->n_fetch * sizeof(uint32_t));
    memcpy(fetch_frames, o->fetch_frames.v, o->n_fetch * sizeof(uint32_t));
    return E_OK;
}

static uint64_t slot_of(const orc_t *o, uint32_t page) {
    return o->host_slot ? o->host_slot[page] : page;
}

/* Carry out the pending plan: victims out (unmap, copy to host), then targets in (copy, map). */
int orc_migrate(orc_t *o) {
    if (!o->plan_pending) return E_STALE;
    if (o->mig_done) return E_INVAL;                       /* a prefix has been carried out: finish it the same way */
    size_t P = (size_t)1 << o->page_shift;
    for (uint32_t i = 0; i < o->n_evict; i++) {
        uint32_t p = o->evict_pages.v[i], f = o->evict_frames.v[i];
        o->page_table[p] = NONE32;
        o->frame_owner[f] = NONE32;
        if (o->pool) memcpy(o->host + slot_of(o, p) * P, o->pool + (size_t)f * P, P);
    }
    for (uint32_t i = 0; i < o->n_fetch; i++) {
        uint32_t p = o->fetch_pages.v[i], f = o->fetch_frames.v[i];
        if (o->pool) memcpy(o->pool + (size_t)f * P, o->host + slot_of(o, p) * P, P);
        o->page_table[p] = f;
        o->frame_owner[f] = p;
    }
    o->plan_pending = 0;
    return E_OK;
}

/* Early execution (Sec. 6.3: pages migrate in predicted access order and a kernel starts as soon as the
 * pages it depends on are resident).  need[g], g < g_cut: how many leading entries of the fetch list must
 * have landed before the g-th covered command may start = fetches first used by a command <= g. */
int orc_ready_need(const orc_t *o, uint32_t *need) {
    if (!o->plan_pending) return E_STALE;
    for (uint32_t g = 0; g < o->g_cut; g++) {
        uint32_t n = 0;
        for (uint32_t i = 0; i < o->n_fetch; i++) if (o->nu[o->fetch_pages.v[i]] <= g) n++;
        need[g] = n;
    }
    return E_OK;
}

/* Carry out the pending plan up to and including fetch entry n - 1, entry by entry in list order: the
 * victim whose frame the entry reuses goes out first, then the target comes in.  Calls continue where the
 * last one stopped; the plan is done when n reaches n_fetch. */
int orc_migrate_prefix(orc_t *o, uint32_t n) {
    if (!o->plan_pending) return E_STALE;
    if (n > o->n_fetch || n < o->mig_done) return E_INVAL;
    size_t P = (size_t)1 << o->page_shift;
    for (uint32_t i = o->mig_done; i < n; i++) {
        uint32_t p = o->fetch_pages.v[i], f = o->fetch_frames.v[i];
        if (i >= o->n_free_used) {
            uint32_t v = o->evict_pages.v[i - o->n_free_used];
            o->page_table[v] = NONE32;
            o->frame_owner[f] = NONE32;
            if (o->pool) memcpy(o->host + slot_of(o, v) * P, o->pool + (size_t)f * P, P);
        }
        if (o->pool) memcpy(o->pool + (size_t)f * P, o->host + slot_of(o, p) * P, P);
        o->page_table[p] = f;
        o->frame_owner[f] = p;
    }
    o->mig_done = n;
    if (n == o->n_fetch) { o->plan_pending = 0; o->mig_done = 0; }
    return E_OK;
}

/* Demand-paging fallback (Sec. 5.2: a page the prediction missed is brought in by an ordinary page fault).
 * The running command touches `pages`; every one that is not resident faults: it takes the lowest free
 * frame, or else the frame of the resident page outside `pages` whose next use (as of the latest plan) is
 * farthest - never-used pages first, ties to the lowest page id - which is the head of the eviction order
 * the plan established (Sec. 6.2).  Bytes move as in a migration.  Returns the number of faults. */
int64_t orc_demand_touch(orc_t *o, const uint32_t *pages, uint32_t n) {
    if (o->plan_pending) return E_INVAL;                      /* between a plan and its migration nothing runs */
    size_t P = (size_t)1 << o->page_shift;
    int64_t faults = 0;
    uint8_t *in_use = (uint8_t *)calloc(o->V + 1, 1);
    if (!in_use) return E_NOMEM;
    for (uint32_t i = 0; i < n; i++) { if (pages[i] >= o->V) { free(in_use); return E_RANGE; } in_use[pages[i]] = 1; }
    for (uint32_t i = 0; i < n; i++) {
        uint32_t p = pages[i];
        if (o->page_table[p] != NONE32) continue;
        if (o->host_slot && o->host_slot[p] == NONE32) { free(in_use); return E_RANGE; }
        faults++;
        uint32_t f = NONE32;
        for (uint32_t k = 0; k < o->F && f == NONE32; k++) if (o->frame_owner[k] == NONE32) f = k;
        if (f == NONE32) {
            uint32_t victim = NONE32;
            for (uint64_t q = 0; q < o->V; q++) {
                if (o->page_table[q] == NONE32 || in_use[q]) continue;
                if (victim == NONE32 || o->nu[q] > o->nu[victim]) victim = (uint32_t)q;
            }
            if (victim == NONE32) { free(in_use); return E_WSET; }   /* the command alone does not fit */
            f = o->page_table[victim];
            o->page_table[victim] = NONE32;
            if (o->pool) memcpy(o->host + slot_of(o, victim) * P, o->pool + (size_t)f * P, P);
        }
        if (o->pool) memcpy(o->pool + (size_t)f * P, o->host + slot_of(o, p) * P, P);
        o->page_table[p] = f;
        o->frame_owner[f] = p;
        o->nu[p] = 0;                                         /* in use now */
    }
    free(in_use);
    return faults;
}

int orc_pagetable_query(const orc_t *o, const uint64_t *pages, uint32_t n, uint32_t *out) {
    for (uint32_t i = 0; i < n; i++) if (pages[i] >= o->V) return E_RANGE;
    for (uint32_t i = 0; i < n; i++) out[i] = o->page_table[pages[i]];
    return E_OK;
}

void orc_state(const orc_t *o, uint32_t *page_table, uint32_t *frame_owner) {
    memcpy(page_table, o->page_table, o->V * sizeof(uint32_t));
    memcpy(frame_owner, o->frame_owner, (size_t)o->F * sizeof(uint32_t));
}

/*
 * Demand paging with least-recently-used replacement (the driver behaviour the paper
 * compares against, Sec. 6.2 "Driver support": faults with full HBM evict from the list
 * head).  Textbook LRU over the reference string formed by the launches in execution
 * order, each launch referencing its pages in ascending id order.  Returns the number
 * of page faults (= pages fetched).
 */
int64_t orc_lru_faults(orc_t *o, const uint32_t *task, const uint64_t *index, uint64_t n_launches,
                       uint32_t capacity) {
    uint64_t V = o->V;
    uint32_t *prev = (uint32_t *)malloc(V * sizeof(uint32_t));
    uint32_t *next = (uint32_t *)malloc(V * sizeof(uint32_t));
    uint8_t *in = (uint8_t *)calloc(V, 1);
    if (!prev || !next || !in) return E_NOMEM;
    uint32_t head = NONE32, tail = NONE32;   /* head = least recently used */
    uint64_t resident = 0;
    int64_t faults = 0;
    vec32 pages = {0, 0, 0};
    for (uint64_t l = 0; l < n_launches; l++) {
        if (task[l] >= o->n_tasks || index[l] >= o->tasks[task[l]].n) { faults = E_INVAL; break; }
        int rc = expand_command(o, &o->tasks[task[l]].cmds[index[l]], &pages);
        if (rc) { faults = rc; break; }
        for (size_t i = 0; i < pages.n; i++) {
            uint32_t p = pages.v[i];
            if (in[p]) {                       /* hit: unlink */
                if (prev[p] != NONE32) next[prev[p]] = next[p]; else head = next[p];
                if (next[p] != NONE32) prev[next[p]] = prev[p]; else tail = prev[p];
            } else {
                faults++;
                if (resident == capacity) {    /* evict the least recently used page */
                    uint32_t v = head;
                    head = next[v];
                    if (head != NONE32) prev[head] = NONE32; else tail = NONE32;
                    in[v] = 0; resident--;
                }
                in[p] = 1; resident++;
            }
            prev[p] = tail; next[p] = NONE32;  /* append as most recently used */
            if (tail != NONE32) next[tail] = p; else head = p;
            tail = p;
        }
    }
    free(pages.v); free(prev); free(next); free(in);
    return faults;
}
