// C-ABI entry points of libmsched: context, template registry, per-task command queues,
// timeline flattening, and the calls that drive the planning and migration kernels.
#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstdlib>
#include <cstring>
#include <new>

#include "msched_internal.h"

using namespace msched;

namespace msched {
int g_last_hip = 0;   // last HIP error of any context (readable when no context exists, e.g. after a failed create)
}

namespace {

#define HIP_TRY(c, x)                                                \
    do {                                                             \
        hipError_t e_ = (x);                                         \
        if (e_ != hipSuccess) { (c)->last_hip = g_last_hip = (int)e_; return MSCHED_E_HIP; } \
    } while (0)

// Nothing may be thrown across the C boundary: the few container operations inside can only fail for memory.
template <class F> int guarded(F &&body) noexcept {
    try { return body(); }
    catch (const std::bad_alloc &) { return MSCHED_E_NOMEM; }
    catch (...) { return MSCHED_E_INVAL; }
}

// value = coeff * product(args[idx]), refusing arithmetic that leaves 64 bits (Sec. 5.2: extents
// are a linear coefficient times a product of launch arguments).
int checked_formula(uint64_t coeff, const uint8_t *idx, int n, const uint64_t *args, uint32_t n_args, uint64_t *out) {
    uint64_t v = coeff;
    for (int j = 0; j < n; ++j) {
        if (idx[j] >= n_args) return MSCHED_E_RANGE;
        if (__builtin_mul_overflow(v, args[idx[j]], &v)) return MSCHED_E_OVERFLOW;
    }
    *out = v;
    return MSCHED_OK;
}

int check_range(const msched_ctx *c, uint64_t addr, uint64_t len) {
    if (len == 0) return MSCHED_OK;
    uint64_t last;
    if (__builtin_add_overflow(addr, len - 1, &last)) return MSCHED_E_OVERFLOW;
    if ((last >> c->page_shift) >= c->V) return MSCHED_E_RANGE;
    return MSCHED_OK;
}

// Evaluate every rule once on the host so that nothing the kernels will touch can be out of bounds.
int validate_launch(const msched_ctx *c, const DevKernel &k, const uint64_t *args, uint32_t n_args) {
    for (uint32_t r = 0; r < k.n_rules; ++r) {
        const msched_rule &q = k.rules[r];
        if (q.kind == MSCHED_RULE_LIST) continue;
        if (q.base_arg >= n_args) return MSCHED_E_RANGE;
        const uint64_t base = args[q.base_arg];
        uint64_t size, stride, count;
        int rc;
        if ((rc = checked_formula(q.size_coeff, q.size_args, q.n_size_args, args, n_args, &size))) return rc;
        if (q.kind != MSCHED_RULE_STRIDED) {
            if ((rc = check_range(c, base, size))) return rc;
            continue;
        }
        if ((rc = checked_formula(q.stride_coeff, q.stride_args, q.n_stride_args, args, n_args, &stride))) return rc;
        if ((rc = checked_formula(q.count_coeff, q.count_args, q.n_count_args, args, n_args, &count))) return rc;
        if (size == 0 || count == 0) continue;
        uint64_t span, last_start;                       // the last chunk reaches farthest
        if (__builtin_mul_overflow(count - 1, stride, &span)) return MSCHED_E_OVERFLOW;
        if (__builtin_add_overflow(base, span, &last_start)) return MSCHED_E_OVERFLOW;
        if ((rc = check_range(c, last_start, size))) return rc;
    }
    return MSCHED_OK;
}

// A later command whose rule describes exactly the region an earlier queued command of its task already
// describes cannot lower any page's first use while that command is queued, so a plan leaves it out.
// Iterative workloads launch the same kernels over the same buffers again and again (the paper finds 77 % of
// accesses fixed-size, Sec. 5.2), which makes most rules of a timeline repeats.  The test is exact: regions
// are compared as full tuples (page range for fixed/linear rules, the four strided parameters, or the id-list
// address and length), never by hash alone.  `empty`: the rule describes nothing.
inline void region_signature(const msched_ctx *c, const msched_rule &q, const CmdRec &r, RegionSig &sig, bool &empty) {
    empty = false;
    if (q.kind == MSCHED_RULE_LIST) {
        sig = {4, (uint64_t)(uintptr_t)r.ids, r.n_ids, 0};
        empty = r.n_ids == 0;
        return;
    }
    auto eval = [&](uint64_t coeff, const uint8_t *idx, int n) {
        uint64_t v = coeff;
        for (int j = 0; j < n; ++j) v *= r.args[idx[j]];      // validated at enqueue: cannot overflow
        return v;
    };
    const uint64_t base = r.args[q.base_arg];
    const uint64_t size = q.kind == MSCHED_RULE_FIXED ? q.size_coeff : eval(q.size_coeff, q.size_args, q.n_size_args);
    if (q.kind != MSCHED_RULE_STRIDED) {
        if (size == 0) { empty = true; return; }
        sig = {1, base >> c->page_shift, (base + size - 1) >> c->page_shift, 0};
        return;
    }
    const uint64_t stride = eval(q.stride_coeff, q.stride_args, q.n_stride_args);
    const uint64_t count = eval(q.count_coeff, q.count_args, q.n_count_args);
    if (size == 0 || count == 0) { empty = true; return; }
    sig = {base, size, stride, count ^ (3ull << 62)};
}

constexpr size_t kMirrorArenaBytes = 4u << 20;
hipError_t mirror_alloc(msched_ctx *c, size_t bytes, void **out) {
    if (!c->mirror_arena) {
        if (hipMalloc((void **)&c->mirror_arena, kMirrorArenaBytes) != hipSuccess) { (void)hipGetLastError(); c->mirror_arena = nullptr; }
        c->mirror_arena_used = 0;
    }
    const size_t at = (c->mirror_arena_used + 255) & ~(size_t)255;
    if (c->mirror_arena && at + bytes <= kMirrorArenaBytes) {
        *out = c->mirror_arena + at;
        c->mirror_arena_used = at + bytes;
        return hipSuccess;
    }
    return hipMalloc(out, bytes);
}
void mirror_free(msched_ctx *c, void *p) {                   // pieces of the arena are given up with the arena
    const uint8_t *q = static_cast<const uint8_t *>(p);
    if (p && !(c->mirror_arena && q >= c->mirror_arena && q < c->mirror_arena + kMirrorArenaBytes)) (void)hipFree(p);
}

// Room for `count` more ranges in a task's ring: ranges of retired commands are dead, and when the live ones fill
// it, a ring of twice the size takes over (pinned memory and its mirror: rare, so the stream is drained first - a
// sweep of a plan whose second half still runs may be reading the mirror).
int range_room(msched_ctx *c, TaskQueue &t, uint64_t count) {
    const uint64_t live_from = t.ranges_live_from();
    if (t.rng_end + count - live_from <= t.rng_cap) return MSCHED_OK;
    uint64_t ncap = std::max<uint64_t>(4096, t.rng_cap);
    while (ncap < 2 * (t.rng_end + count - live_from)) ncap *= 2;
    if (ncap > (1ull << 30)) return MSCHED_E_NOMEM;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    RangeRec *nh = nullptr;
    HIP_TRY(c, hipHostMalloc((void **)&nh, ncap * sizeof(RangeRec), hipHostMallocDefault));
    for (uint64_t q = live_from; q < t.rng_end; ++q) nh[q & (ncap - 1)] = t.rng[q & (t.rng_cap - 1)];
    if (t.rng) (void)hipHostFree(t.rng);
    mirror_free(c, t.rng_dev);                   // the mirror, if there was one, is made anew (and filled) by the plan that next wants it
    t.rng = nh; t.rng_dev = nullptr; t.rng_cap = ncap;
    t.rng_uploaded = live_from;
    return MSCHED_OK;
}

// The page ranges a fixed / linear / strided rule describes for command i of a task (template expansion, Sec. 5.2),
// appended to the task's ring.  Returns 1 when the command would hold more than `cap` ranges, < 0 on failure.
inline int append_ranges(msched_ctx *c, TaskQueue &t, const msched_rule &q, const CmdRec &r, size_t i,
                         uint32_t back, uint64_t first, size_t cap) {
    auto eval = [&](uint64_t coeff, const uint8_t *idx, int cnt) {
        uint64_t v = coeff;
        for (int j = 0; j < cnt; ++j) v *= r.args[idx[j]];    // validated at enqueue: cannot overflow
        return v;
    };
    const uint32_t sh = c->page_shift;
    const uint64_t base = r.args[q.base_arg];
    uint64_t size = q.kind == MSCHED_RULE_FIXED ? q.size_coeff : eval(q.size_coeff, q.size_args, q.n_size_args);
    if (size == 0) return MSCHED_OK;
    uint64_t stride = 0, count = 1;
    if (q.kind == MSCHED_RULE_STRIDED) {
        stride = eval(q.stride_coeff, q.stride_args, q.n_stride_args);
        count = eval(q.count_coeff, q.count_args, q.n_count_args);
        if (count == 0) return MSCHED_OK;
        if (size >= stride || count == 1) { size = (count - 1) * stride + size; count = 1; }   // the chunks abut or overlap
    }
    if (count > cap - (t.rng_end - first)) return 1;
    const int rc = range_room(c, t, count);
    if (rc) return rc;
    for (uint64_t j = 0; j < count; ++j) {
        const uint64_t c0 = base + j * stride, at = t.rng_end++ & (t.rng_cap - 1);
        t.rng[at] = RangeRec{(uint32_t)(c0 >> sh), (uint32_t)(((c0 + size - 1) >> sh) + 1), back, (uint32_t)i};
    }
    return MSCHED_OK;
}

// Bring a task's range mirror up to date (one or two copies on the context's stream, straight from the pinned ring).
// The mirror itself is made when a plan first wants it: tasks whose plans always stage their tables never get one.
int upload_ranges(msched_ctx *c, TaskQueue &t) {
    if (t.rng_cap == 0) return MSCHED_OK;
    if (t.rng_dev == nullptr) {
        HIP_TRY(c, mirror_alloc(c, t.rng_cap * sizeof(RangeRec), (void **)&t.rng_dev));
        t.rng_uploaded = 0;
    }
    const uint64_t from = std::max(t.rng_uploaded, t.ranges_live_from());
    if (from < t.rng_end) {
        const uint64_t mask = t.rng_cap - 1, pos = from & mask, n = t.rng_end - from, n1 = std::min(n, t.rng_cap - pos);
        HIP_TRY(c, hipMemcpyAsync(t.rng_dev + pos, t.rng + pos, n1 * sizeof(RangeRec), hipMemcpyHostToDevice, c->stream));
        if (n > n1) HIP_TRY(c, hipMemcpyAsync(t.rng_dev, t.rng, (n - n1) * sizeof(RangeRec), hipMemcpyHostToDevice, c->stream));
    }
    t.rng_uploaded = t.rng_end;
    return MSCHED_OK;
}

// Is the command `back` places before command i of a task still queued (and with it in every timeline)?
inline bool repeats_queued(const msched_ctx *c, const TaskQueue &t, size_t i, uint32_t back) {
    return c->dedupe_regions && back != 0 && i - back >= t.cursor;
}

void free_ctx(msched_ctx *c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->stream);
    for (auto &t : c->tasks) if (t.recs) (void)hipHostFree(t.recs);
    for (auto &t : c->tasks) if (t.prep_buf) (void)hipFree(t.prep_buf);
    for (auto &t : c->tasks) { if (t.rng) (void)hipHostFree(t.rng); mirror_free(c, t.rng_dev); }
    if (c->mirror_arena) (void)hipFree(c->mirror_arena);
    if (c->list_src_host) (void)hipHostFree(c->list_src_host);
    if (c->list_prep_host) (void)hipHostFree(c->list_prep_host);
    if (c->list_src_stage) (void)hipFree(c->list_src_stage);
    if (c->bucket_mark) (void)hipFree(c->bucket_mark);
    if (c->list_ahead_host) (void)hipHostFree(c->list_ahead_host);
    if (c->ahead_ev) (void)hipEventDestroy(c->ahead_ev);
    void *dev[] = {c->page_table, c->frame_owner, c->nu, c->slot, c->evict_pages, c->evict_frames, c->fetch_pages,
                   c->fetch_frames, c->flags, c->matrix, c->partial, c->chunk_hint, c->offsets, c->hdr_dev, c->kernels_dev,
                   c->query_buf, c->cmd_dev, c->list_bucket_fill, c->list_pairs};
    for (void *p : dev) if (p) (void)hipFree(p);
    if (c->hdr_host) (void)hipHostFree(c->hdr_host);
    if (c->ranges_host) (void)hipHostFree(c->ranges_host);
    if (c->ranges_dev) (void)hipFree(c->ranges_dev);
    if (c->key16) (void)hipFree(c->key16);
    if (c->poll_stream) { (void)hipStreamSynchronize(c->poll_stream); (void)hipStreamDestroy(c->poll_stream); }
    for (void *p : {(void *)c->page_done, (void *)c->chunks_done, (void *)c->landed}) if (p) (void)hipFree(p);
    if (c->need_host) (void)hipHostFree(c->need_host);
    if (c->gate_host) (void)hipHostFree(c->gate_host);
    if (c->progress_host) (void)hipHostFree(c->progress_host);
    if (c->cmd_ptrs_host) (void)hipHostFree((void *)c->cmd_ptrs_host);
    for (auto &e : c->ev) if (e) (void)hipEventDestroy(e);
    delete c;
}

int env_u32(const char *name, uint32_t lo, uint32_t hi, uint32_t dflt) {
    const char *s = getenv(name);
    if (!s || !*s) return (int)dflt;
    long v = strtol(s, nullptr, 10);
    if (v < (long)lo || v > (long)hi) return (int)dflt;
    return (int)v;
}

}  // namespace

extern "C" {

int msched_create(const msched_config *cfg, msched_ctx **out) {
    if (!cfg || !out) return MSCHED_E_INVAL;
    if (cfg->page_shift < 6 || cfg->page_shift > 30 || cfg->n_frames == 0 || cfg->n_virtual_pages == 0 ||
        cfg->n_virtual_pages >= 0xFFFFFFFFull || !cfg->hbm_pool || !cfg->host_store ||
        ((uintptr_t)cfg->hbm_pool & 15) || ((uintptr_t)cfg->host_store & 15))
        return MSCHED_E_INVAL;
    if (!cfg->host_slot && cfg->n_host_slots < cfg->n_virtual_pages) return MSCHED_E_INVAL;
    if (cfg->host_slot) {
        // two pages that shared a slot would overwrite each other's backing bytes on eviction
        std::vector<uint64_t> taken;
        const int rc_map = guarded([&]() -> int { taken.assign((cfg->n_host_slots + 63) / 64, 0); return MSCHED_OK; });
        if (rc_map) return rc_map;
        for (uint64_t p = 0; p < cfg->n_virtual_pages; ++p) {
            const uint64_t s = cfg->host_slot[p];
            if (s == MSCHED_NO_SLOT) continue;
            if (s >= cfg->n_host_slots) return MSCHED_E_RANGE;
            if (taken[s >> 6] & (1ull << (s & 63))) return MSCHED_E_INVAL;
            taken[s >> 6] |= 1ull << (s & 63);
        }
    }
    msched_ctx *c = new (std::nothrow) msched_ctx();
    if (!c) return MSCHED_E_NOMEM;
    const int rc_tables = guarded([&]() -> int {
        c->runs.reserve(MSCHED_MAX_TIMELINE_ENTRIES);
        c->reserved.reserve(kMaxListSources);
        return MSCHED_OK;
    });
    if (rc_tables) { delete c; return rc_tables; }
    c->cfg = *cfg;
    c->cfg.host_slot = nullptr;
    c->stream = (hipStream_t)cfg->stream;
    c->V = cfg->n_virtual_pages; c->F = cfg->n_frames; c->page_shift = cfg->page_shift;
    c->migrate_chunk_shift = (uint32_t)env_u32("MSCHED_MIGRATE_CHUNK_SHIFT", 6, 24, 21);
    c->early_chunk_shift = (uint32_t)env_u32("MSCHED_EARLY_CHUNK_SHIFT", 12, 24, 16);
    c->migrate_ticket = (uint32_t)env_u32("MSCHED_MIGRATE_TICKET", 0, 1, 0);
    c->paint = (uint32_t)env_u32("MSCHED_PAINT", 0, 1, 1);
    c->resident_ranges = (uint32_t)env_u32("MSCHED_RESIDENT_RANGES", 0, 1, 1);
    c->migrate_max_blocks = (uint32_t)env_u32("MSCHED_MIGRATE_BLOCKS", 1, 1 << 20, 512);
    c->migrate_hints = (uint32_t)env_u32("MSCHED_MIGRATE_HINTS", 0, 3, 0);
    c->expand_split = (uint32_t)env_u32("MSCHED_EXPAND_SPLIT", 1, 64, 0);
    c->max_chunks = (uint32_t)env_u32("MSCHED_MAX_CHUNKS", 1, kMaxChunks, kMaxChunks);
    c->stage_threshold = (uint32_t)env_u32("MSCHED_STAGE_THRESHOLD", 0, 1 << 30, 2048);
    c->dedupe_regions = env_u32("MSCHED_DEDUPE_REGIONS", 0, 1, 1) != 0;
    c->list_prepared = (uint32_t)env_u32("MSCHED_LIST_PREPARED", 0, 1, 1);
    // One part measured as good as four on the planning-stress schedule (the kernel's time is the instructions a
    // thread spends on its 24 ids, whichever of them it keeps) at a quarter of the ring memory: parts stay a switch.
    c->prep_split_max = (uint32_t)env_u32("MSCHED_PREP_SPLIT", 1, kMaxPrepSplit, 1);
    c->list_cache_bytes = (uint64_t)env_u32("MSCHED_LIST_CACHE_MB", 1, 65536, 128) << 20;
    c->list_ahead = (uint32_t)env_u32("MSCHED_LIST_AHEAD", 0, 65536, 128);
    c->plan_spin = (uint32_t)env_u32("MSCHED_PLAN_SPIN", 0, 1, 1);
    c->fuse_lists = (uint32_t)env_u32("MSCHED_FUSE_LISTS", 0, 1, 1);
    c->order_emit = (uint32_t)env_u32("MSCHED_ORDER_EMIT", 0, 1, 1);
    c->force_multi_kernel = env_u32("MSCHED_FORCE_MULTI_KERNEL", 0, 1, 0) != 0;
    c->no_large_lds = env_u32("MSCHED_NO_LARGE_LDS", 0, 1, 0) != 0;
    c->list_binned_min_ids = (uint64_t)env_u32("MSCHED_LIST_BINNED_MIN_IDS", 0, 1 << 30, 262144);
    c->list_b0 = (uint32_t)env_u32("MSCHED_LIST_B0", 0, 4096, 4);
    c->list_b1 = std::max(c->list_b0, (uint32_t)env_u32("MSCHED_LIST_B1", 0, 4096, 32));

    c->epoch = (uint32_t)env_u32("MSCHED_INITIAL_EPOCH", 0, kMaxEpoch, 0);   // test hook: start near the wrap
    int rc = MSCHED_OK;
    auto fail = [&](hipError_t e) { c->last_hip = g_last_hip = (int)e; rc = MSCHED_E_HIP; };
    hipError_t e;
    if ((e = hipGetDevice(&c->device)) != hipSuccess) fail(e);
    // the static staging array of msched_pagetable_query_static: its address on this device, looked up once
    if (rc == MSCHED_OK && (e = query_scratch_init(nullptr)) != hipSuccess) fail(e);
#define ALLOC(ptr, bytes) if (rc == MSCHED_OK && (e = hipMalloc((void **)&(ptr), (bytes))) != hipSuccess) fail(e)
    // page table, next use and slots are read 16 bytes at a time: padded, so that the last lane may run past V
    ALLOC(c->page_table, c->V * 4 + 64);
    ALLOC(c->frame_owner, (size_t)c->F * 4);
    ALLOC(c->nu, c->V * 4 + 64);
    ALLOC(c->evict_pages, (size_t)c->F * 4);
    ALLOC(c->evict_frames, (size_t)c->F * 4);
    ALLOC(c->fetch_pages, (size_t)c->F * 4);
    ALLOC(c->fetch_frames, (size_t)c->F * 4);
    ALLOC(c->flags, 256);
    ALLOC(c->offsets, (size_t)2 * (MSCHED_MAX_TIMELINE_COMMANDS + 1) * 4);
    ALLOC(c->hdr_dev, sizeof(PlanHeader));
    ALLOC(c->chunk_hint, (size_t)3 * kMaxChunks * 4);
    if (rc == MSCHED_OK && (e = hipMemset(c->chunk_hint, 0, (size_t)3 * kMaxChunks * 4)) != hipSuccess) fail(e);
    // row-group sums of the count matrix: the counting sweep adds into them, k_offsets clears what it read
    ALLOC(c->partial, (size_t)kSumRows * 2 * (MSCHED_MAX_TIMELINE_COMMANDS + 1) * 4);
    if (rc == MSCHED_OK && (e = hipMemset(c->partial, 0, (size_t)kSumRows * 2 * (MSCHED_MAX_TIMELINE_COMMANDS + 1) * 4)) != hipSuccess) fail(e);
    ALLOC(c->cmd_dev, sizeof(CmdRec) * (MSCHED_MAX_TIMELINE_COMMANDS + 1));
    if (cfg->host_slot) {
        ALLOC(c->slot, c->V * 4);
        if (rc == MSCHED_OK && (e = hipMemcpy(c->slot, cfg->host_slot, c->V * 4, hipMemcpyHostToDevice)) != hipSuccess) fail(e);
    }
#undef ALLOC
    if (rc == MSCHED_OK && (e = hipHostMalloc((void **)&c->hdr_host, sizeof(PlanHeader), hipHostMallocDefault)) != hipSuccess) fail(e);
    if (rc == MSCHED_OK) memset(c->hdr_host, 0, sizeof(PlanHeader));            // no stamp yet
    if (rc == MSCHED_OK && (e = hipHostMalloc((void **)&c->cmd_ptrs_host,
                                              sizeof(void *) * (MSCHED_MAX_TIMELINE_COMMANDS + 1), hipHostMallocDefault)) != hipSuccess) fail(e);
    if (rc == MSCHED_OK && (e = hipHostGetDevicePointer((void **)&c->cmd_ptrs_dev, (void *)c->cmd_ptrs_host, 0)) != hipSuccess) fail(e);
    if (rc == MSCHED_OK && (e = hipHostGetDevicePointer(&c->host_dev, cfg->host_store, 0)) != hipSuccess) fail(e);
    if (rc == MSCHED_OK && (e = hipHostMalloc((void **)&c->ranges_host, sizeof(PageRange) * kMaxRanges, hipHostMallocDefault)) != hipSuccess) fail(e);
    if (rc == MSCHED_OK && (e = hipHostGetDevicePointer((void **)&c->ranges_host_dev, c->ranges_host, 0)) != hipSuccess) fail(e);
    if (rc == MSCHED_OK && (e = hipMalloc((void **)&c->ranges_dev, sizeof(PageRange) * kMaxRanges)) != hipSuccess) fail(e);
    if (rc == MSCHED_OK && (e = hipMalloc((void **)&c->key16, c->V * 2 + 64)) != hipSuccess) fail(e);
    if (rc == MSCHED_OK && c->page_shift > std::min(c->migrate_chunk_shift, c->early_chunk_shift)) {
        // pages larger than a work unit of the copy: their chunks are counted, the last one maps the page
        if ((e = hipMalloc((void **)&c->chunks_done, (size_t)c->F * 4)) != hipSuccess) fail(e);
        else if ((e = hipMemset(c->chunks_done, 0, (size_t)c->F * 4)) != hipSuccess) fail(e);
    }
    for (int i = 0; i < 10 && rc == MSCHED_OK; ++i)
        if ((e = hipEventCreate(&c->ev[i])) != hipSuccess) fail(e);

    if (rc == MSCHED_OK && (e = launch_init_tables(c)) != hipSuccess) fail(e);
    if (rc == MSCHED_OK && (e = launch_nu_reset(c)) != hipSuccess) fail(e);
    if (rc == MSCHED_OK && (e = hipMemsetAsync(c->flags, 0, 256, c->stream)) != hipSuccess) fail(e);
    if (rc == MSCHED_OK && (e = hipStreamSynchronize(c->stream)) != hipSuccess) fail(e);
    if (rc != MSCHED_OK) { free_ctx(c); return rc; }
    *out = c;
    return MSCHED_OK;
}

int msched_destroy(msched_ctx *ctx) {
    if (!ctx) return MSCHED_E_INVAL;
    free_ctx(ctx);
    return MSCHED_OK;
}

int msched_kernel_register(msched_ctx *c, const msched_rule *rules, uint32_t n_rules, uint32_t *kernel_id) {
    if (!c || !kernel_id || n_rules > MSCHED_MAX_RULES || (n_rules && !rules)) return MSCHED_E_INVAL;
    DevKernel k;
    memset(&k, 0, sizeof k);
    k.n_rules = n_rules;
    bool has_list = false;
    for (uint32_t r = 0; r < n_rules; ++r) {
        const msched_rule &q = rules[r];
        if (q.kind < MSCHED_RULE_FIXED || q.kind > MSCHED_RULE_LIST) return MSCHED_E_INVAL;
        if (q.n_size_args > MSCHED_MAX_PRODUCT_ARGS || q.n_stride_args > MSCHED_MAX_PRODUCT_ARGS ||
            q.n_count_args > MSCHED_MAX_PRODUCT_ARGS)
            return MSCHED_E_INVAL;
        if (q.kind == MSCHED_RULE_FIXED && q.n_size_args != 0) return MSCHED_E_INVAL;
        k.rules[r] = q;
        if (q.kind == MSCHED_RULE_LIST) has_list = true;
    }
    const int rc_room = guarded([&]() -> int {               // host tables first, so that nothing below can fail half-way
        c->kernels.reserve(c->kernels.size() + 1);
        c->kernel_has_list.reserve(c->kernel_has_list.size() + 1);
        return MSCHED_OK;
    });
    if (rc_room) return rc_room;
    // the table is small and changes rarely: keep a device copy in step with the host one
    if (c->kernels.size() + 1 > c->kernels_cap) {
        const size_t ncap = std::max<size_t>(64, c->kernels_cap * 2);
        DevKernel *nd = nullptr;
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        HIP_TRY(c, hipMalloc((void **)&nd, ncap * sizeof(DevKernel)));
        if (!c->kernels.empty()) {
            const hipError_t e = hipMemcpy(nd, c->kernels.data(), c->kernels.size() * sizeof(DevKernel), hipMemcpyHostToDevice);
            if (e != hipSuccess) { (void)hipFree(nd); HIP_TRY(c, e); }
        }
        if (c->kernels_dev) (void)hipFree(c->kernels_dev);
        c->kernels_dev = nd;
        c->kernels_cap = ncap;
    }
    HIP_TRY(c, hipMemcpy(c->kernels_dev + c->kernels.size(), &k, sizeof k, hipMemcpyHostToDevice));
    c->kernels.push_back(k);
    c->has_list_rule = c->has_list_rule || has_list;
    c->kernel_has_list.push_back(has_list ? 1 : 0);
    c->max_rules = std::max(c->max_rules, n_rules);
    *kernel_id = (uint32_t)(c->kernels.size() - 1);
    return MSCHED_OK;
}

int msched_task_create(msched_ctx *c, uint32_t *task_id) {
    if (!c || !task_id) return MSCHED_E_INVAL;
    return guarded([&]() -> int {
        c->pos.reserve(c->tasks.size() + 1);
        c->tasks.emplace_back();
        c->pos.resize(c->tasks.size());
        *task_id = (uint32_t)(c->tasks.size() - 1);
        return MSCHED_OK;
    });
}

int msched_launch_enqueue(msched_ctx *c, uint32_t task, uint32_t kernel_id, const uint64_t *args, uint32_t n_args,
                          uint32_t latency_ticks, const uint32_t *id_list, uint32_t n_ids) {
    if (!c || task >= c->tasks.size() || kernel_id >= c->kernels.size() || n_args > MSCHED_MAX_ARGS ||
        (n_args && !args) || (n_ids && !id_list))
        return MSCHED_E_INVAL;
    const int rc = validate_launch(c, c->kernels[kernel_id], args, n_args);
    if (rc) return rc;
    TaskQueue &t = c->tasks[task];
    if (t.n - t.base == t.cap) {
        // The record array is full: drop the retired records, and grow it if most of it is still live.  Kernels read
        // queue records only ahead of the cut of a plan (staging, expansion, id-list binning), and msched_plan returns
        // after the cut has stamped its header; what msched_migrate queues behind the copy (id-list preparation) reads
        // the caller's id arrays and a table of its own, never a record.  So nothing that is still queued or running
        // can hold an address into the array - and the stream is drained here all the same, so that this stays true
        // if a later kernel of a plan ever reads records: this happens once per `cap` launches, a wait costs nothing then.
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        const size_t live = t.n - t.cursor, off = t.cursor - t.base;
        const uint64_t keep_from = t.cap ? t.range_begin(t.cursor) : 0;      // the retired commands' ranges go too
        if (t.cap && live <= t.cap / 2) {
            // a queue in steady state (launches retire as fast as they arrive): the live records move to the front,
            // nothing is allocated
            if (live && off) {
                memmove(t.recs, t.recs + off, live * sizeof(CmdRec));
                auto front = [&](auto &v) { std::copy(v.begin() + off, v.begin() + off + live, v.begin()); };
                front(t.lat); front(t.n_ids); front(t.list_back); front(t.range_end); front(t.prep); front(t.ids); front(t.flag);
                std::copy(t.rule_back.begin() + off * MSCHED_MAX_RULES, t.rule_back.begin() + (off + live) * MSCHED_MAX_RULES, t.rule_back.begin());
            }
        } else {
            const size_t ncap = std::max<size_t>(256, live * 2);
            // the compact arrays first: if one of them cannot grow, nothing has changed yet
            std::vector<uint32_t> lat, n_ids, list_back, rule_back;
            std::vector<uint64_t> range_end, prep;
            std::vector<const uint32_t *> ids;
            std::vector<uint8_t> flag;
            const int rc_room = guarded([&]() -> int {
                lat.resize(ncap); n_ids.resize(ncap); list_back.resize(ncap); range_end.resize(ncap); prep.resize(ncap);
                ids.resize(ncap); flag.resize(ncap); rule_back.resize(ncap * MSCHED_MAX_RULES);
                return MSCHED_OK;
            });
            if (rc_room) return rc_room;
            CmdRec *nr = nullptr, *nd = nullptr;
            HIP_TRY(c, hipHostMalloc((void **)&nr, ncap * sizeof(CmdRec), hipHostMallocDefault));
            const hipError_t e = hipHostGetDevicePointer((void **)&nd, nr, 0);
            if (e != hipSuccess) { (void)hipHostFree(nr); HIP_TRY(c, e); }
            if (live) {
                memcpy(nr, t.recs + off, live * sizeof(CmdRec));
                std::copy_n(t.lat.begin() + off, live, lat.begin());
                std::copy_n(t.n_ids.begin() + off, live, n_ids.begin());
                std::copy_n(t.list_back.begin() + off, live, list_back.begin());
                std::copy_n(t.range_end.begin() + off, live, range_end.begin());
                std::copy_n(t.prep.begin() + off, live, prep.begin());
                std::copy_n(t.ids.begin() + off, live, ids.begin());
                std::copy_n(t.flag.begin() + off, live, flag.begin());
                std::copy_n(t.rule_back.begin() + off * MSCHED_MAX_RULES, live * MSCHED_MAX_RULES, rule_back.begin());
            }
            if (t.recs) (void)hipHostFree(t.recs);
            t.recs = nr; t.recs_dev = nd; t.cap = ncap;
            t.lat.swap(lat); t.n_ids.swap(n_ids); t.list_back.swap(list_back); t.range_end.swap(range_end);
            t.prep.swap(prep); t.ids.swap(ids); t.flag.swap(flag); t.rule_back.swap(rule_back);
        }
        t.ranges_base = keep_from;
        t.base = t.cursor;
    }
    return guarded([&]() -> int {
        const size_t i = t.n, li = i - t.base;
        CmdRec &r = t.recs[li];
        memset(&r, 0, sizeof r);
        r.kernel = kernel_id; r.n_args = n_args; r.latency = latency_ticks; r.n_ids = n_ids; r.ids = id_list;
        for (uint32_t a = 0; a < n_args; ++a) r.args[a] = args[a];
        // Template expansion (Sec. 5.2): the formulas are evaluated here, once, with the launch's arguments; a plan
        // only walks the page ranges.  A rule's region is also looked up among the regions earlier commands of the
        // task described, so that plans can leave repeats out without looking anything up themselves.
        const DevKernel &k = c->kernels[kernel_id];
        const uint64_t first = t.rng_end;
        uint8_t flag = 0;
        uint32_t list_back = 0;
        struct Unwind {                              // a failure half-way must not leave ranges for the next command to inherit
            TaskQueue &t; uint64_t end; bool armed = true;
            ~Unwind() { if (armed) t.rng_end = end; }
        } unwind{t, first};
        if (t.last_region.size() > 4096 && t.last_region.size() > 2 * t.pruned_at) {
            // regions only retired commands described can no longer make anything a repeat
            for (auto it = t.last_region.begin(); it != t.last_region.end();)
                it = it->second < t.cursor ? t.last_region.erase(it) : std::next(it);
            t.pruned_at = t.last_region.size();
        }
        uint32_t *rule_back = &t.rule_back[li * MSCHED_MAX_RULES];
        for (uint32_t q = 0; q < MSCHED_MAX_RULES; ++q) rule_back[q] = kRuleEmpty;
        for (uint32_t q = 0; q < k.n_rules; ++q) {
            RegionSig sig;
            bool empty;
            region_signature(c, k.rules[q], r, sig, empty);
            if (empty) continue;
            size_t &last = t.last_region.try_emplace(sig, (size_t)-1).first->second;
            const uint32_t back = (last != (size_t)-1 && i - last < 0xFFFFFFFEull) ? (uint32_t)(i - last) : 0u;
            last = i;
            rule_back[q] = back;
            if (k.rules[q].kind == MSCHED_RULE_LIST) {
                flag |= kCmdList;
                list_back = back;
            } else if (!(flag & kCmdNoPaint)) {
                const int rc_app = append_ranges(c, t, k.rules[q], r, i, back, first, kMaxRanges);
                if (rc_app < 0) return rc_app;
                if (rc_app == 1) {
                    flag |= kCmdNoPaint;           // too many chunks to keep: plans that hold this command expand it per page
                    t.rng_end = first;
                }
            }
        }
        t.lat[li] = latency_ticks; t.n_ids[li] = n_ids; t.ids[li] = id_list; t.prep[li] = 0;
        t.flag[li] = flag; t.list_back[li] = list_back;
        t.range_end[li] = t.rng_end;
        t.n++;
        unwind.armed = false;
        return MSCHED_OK;
    });
}

int msched_launch_retire(msched_ctx *c, uint32_t task, uint32_t n_launches) {
    if (!c || task >= c->tasks.size()) return MSCHED_E_INVAL;
    TaskQueue &t = c->tasks[task];
    if (t.cursor + n_launches > t.n) return MSCHED_E_RANGE;
    t.cursor += n_launches;
    return MSCHED_OK;
}

namespace {

// Room for `bytes` in a task's ring of prepared id lists.  Blocks are handed out roughly in program order and
// die with their command's retirement, so the ring's tail is the oldest block a queued command still owns.
bool ring_alloc(msched_ctx *c, TaskQueue &t, uint64_t bytes, uint64_t &off) {
    if (!t.prep_buf) {
        if (hipMalloc((void **)&t.prep_buf, c->list_cache_bytes) != hipSuccess) {
            (void)hipGetLastError();               // no memory for a ring: plans bin their lists from scratch from now on
            t.prep_buf = nullptr;
            c->list_prepared = 0;
            return false;
        }
        t.prep_size = c->list_cache_bytes;
    }
    if (bytes > t.prep_size) return false;
    uint64_t head = t.prep_head;
    const uint64_t pos = head % t.prep_size;
    if (pos + bytes > t.prep_size) head += t.prep_size - pos;        // a block never wraps: skip the ring's end
    if (head + bytes - t.prep_tail > t.prep_size) {
        t.prep_tail = t.prep_head;                                     // nothing live, unless a queued command says otherwise
        for (size_t i = t.cursor; i < t.n; ++i)                        // (mostly, not strictly, in program order: take the oldest)
            if (t.prep[i - t.base]) t.prep_tail = std::min(t.prep_tail, t.prep[i - t.base] - 1);
        if (head + bytes - t.prep_tail > t.prep_size) return false;
    }
    off = head;
    t.prep_head = head + bytes;
    return true;
}

// Give back the ring blocks a plan reserved for id lists it was going to prepare itself, newest first: the plan
// failed before its kernels were launched, so the blocks hold nothing.
void undo_reservations(msched_ctx *c) {
    for (auto it = c->reserved.rbegin(); it != c->reserved.rend(); ++it) {
        TaskQueue &t = c->tasks[it->task];
        t.prep[it->cmd - t.base] = 0;
        t.prep_head = it->head;
    }
    c->reserved.clear();
}

// The pieces of every live id list of the plan: prepared on first sight, reused by every later plan that still
// has the command in its timeline (a command is typically planned once per task of the round).
// Returns 0 and fills the two pinned tables, 1 when the pieces do not fit (the caller bins from scratch), or < 0.
// Blocks reserved here are listed in c->reserved until the plan's kernels are out.
int gather_list_sources(msched_ctx *c, PlanGeom &g) {
    // first use; each piece on its own so that a failure half-way neither leaks nor leaves a hole
    if (!c->list_src_host) HIP_TRY(c, hipHostMalloc((void **)&c->list_src_host, sizeof(ListSource) * kMaxListSources, hipHostMallocDefault));
    if (!c->list_src_dev) HIP_TRY(c, hipHostGetDevicePointer((void **)&c->list_src_dev, c->list_src_host, 0));
    if (!c->list_prep_host) HIP_TRY(c, hipHostMalloc((void **)&c->list_prep_host, sizeof(ListPrep) * kMaxListSources, hipHostMallocDefault));
    if (!c->list_prep_dev) HIP_TRY(c, hipHostGetDevicePointer((void **)&c->list_prep_dev, c->list_prep_host, 0));
    if (!c->list_src_stage) HIP_TRY(c, hipMalloc((void **)&c->list_src_stage, sizeof(ListSource) * kMaxListSources));
    if (!c->bucket_mark) {
        uint32_t *marks = nullptr;
        const size_t bytes = 4 * ((size_t)kMaxBuckets + kMaxChunks);     // behind the marks: the first sweep's chunk order
        HIP_TRY(c, hipMalloc((void **)&marks, bytes));
        const hipError_t e = hipMemset(marks, 0, bytes);
        if (e != hipSuccess) { (void)hipFree(marks); HIP_TRY(c, e); }
        c->bucket_mark = marks;
    }
    uint32_t n_src = 0, n_new = 0;
    c->reserved.clear();
    const uint64_t split = g.split, hdr_words = (uint64_t)prep_part_buckets(g.n_buckets, g.split) + 2;
    for (const PlanRun &run : c->runs) {
        TaskQueue &t = c->tasks[run.task];
        for (uint32_t j = 0; j < run.count; ++j) {
            const size_t i = run.first + j, li = i - t.base;
            if (!(t.flag[li] & kCmdList) || repeats_queued(c, t, i, t.list_back[li])) continue;
            const uint32_t n_ids = t.n_ids[li];
            const uint32_t pieces = (n_ids + kPrepBlock - 1) / kPrepBlock;
            if (n_src + pieces > kMaxListSources) { undo_reservations(c); return 1; }
            const bool is_new = t.prep[li] == 0;
            if (is_new) {
                const uint64_t bytes = (split * ((uint64_t)pieces * hdr_words + n_ids) * 4 + 15) & ~15ull;
                const uint64_t head = t.prep_head;
                uint64_t off;
                if (!ring_alloc(c, t, bytes, off)) { undo_reservations(c); return 1; }
                t.prep[li] = off + 1;
                c->reserved.push_back({run.task, i, head});
            }
            uint32_t *block = reinterpret_cast<uint32_t *>(t.prep_buf + (t.prep[li] - 1) % t.prep_size);
            for (uint32_t p = 0; p < pieces; ++p) {
                const uint32_t n = std::min<uint32_t>(kPrepBlock, n_ids - p * kPrepBlock);
                if (is_new) c->list_prep_host[n_new++] = {t.ids[li] + (size_t)p * kPrepBlock, block, n, {0, 0, 0}};
                c->list_src_host[n_src++] = {block, run.g0 + j, (uint32_t)(hdr_words + n)};
                block += split * (hdr_words + n);
            }
        }
    }
    g.n_list_sources = n_src;
    g.n_list_new = n_new;
    return 0;
}

}  // namespace

namespace {
int plan_body(msched_ctx *c, const msched_timeline_entry *tl, uint32_t n_entries, msched_plan_t *out);
}

int msched_plan(msched_ctx *c, const msched_timeline_entry *tl, uint32_t n_entries, msched_plan_t *out) {
    return guarded([&]() -> int { return plan_body(c, tl, n_entries, out); });
}

namespace {

// Bit r of a command's mask: rule r of its template has nothing to add to this plan - it describes nothing, or
// repeats a region of a command that is still queued in front of it.  Only the per-page and binning kernels, which
// read whole records, want this; the mask rides in the top byte of the record's address (addresses use 48 bits).
uint64_t skip_mask(const msched_ctx *c, const TaskQueue &t, size_t i) {
    const size_t li = i - t.base;
    const uint32_t n_rules = c->kernels[t.recs[li].kernel].n_rules;
    const uint32_t *back = &t.rule_back[li * MSCHED_MAX_RULES];
    uint64_t skip = 0;
    for (uint32_t r = 0; r < n_rules; ++r)
        if (back[r] == kRuleEmpty || repeats_queued(c, t, i, back[r])) skip |= 1ull << r;
    return skip;
}

int plan_body(msched_ctx *c, const msched_timeline_entry *tl, uint32_t n_entries, msched_plan_t *out) {
    if (!c || !out || (n_entries && !tl) || n_entries > MSCHED_MAX_TIMELINE_ENTRIES) return MSCHED_E_INVAL;
    for (uint32_t e = 0; e < n_entries; ++e) if (tl[e].task >= c->tasks.size()) return MSCHED_E_INVAL;
    c->pending_plan = 0;
    using clk = std::chrono::steady_clock;
    const clk::time_point t_start = clk::now();

    // Flatten the timeline into the order of future commands (Sec. 6.1: the timeline says which
    // task runs, for how long and in what order; Sec. 6.2: each queue holds command latencies).
    // A command belongs to the entry in which it starts.  G sizes every launch below, so this
    // short walk over the latencies is done here; an entry becomes one run of consecutive commands.
    for (size_t t = 0; t < c->tasks.size(); ++t) c->pos[t] = c->tasks[t].cursor;
    c->runs.clear();
    uint32_t G = 0, g_end0 = 0;
    for (uint32_t e = 0; e < n_entries; ++e) {
        const TaskQueue &t = c->tasks[tl[e].task];
        size_t &p = c->pos[tl[e].task];
        const size_t first = p;
        const uint32_t g0 = G;
        uint64_t elapsed = 0;
        while (p < t.n && elapsed < tl[e].timeslice) {
            if (G == MSCHED_MAX_TIMELINE_COMMANDS) return MSCHED_E_INVAL;
            elapsed += t.lat[p - t.base];
            ++p; ++G;
        }
        if (p > first) c->runs.push_back(PlanRun{tl[e].task, g0, (uint32_t)(p - first), first});
        if (e == 0) g_end0 = G;
    }
    // What the commands bring: id lists that are not repeats, and whether every command kept its page ranges
    // (msched_launch_enqueue worked them out).  Plans with a command that did not scatter next uses per page.
    bool painted = c->paint != 0, live_list = false;
    uint64_t total_ids = 0;
    for (const PlanRun &run : c->runs) {
        const TaskQueue &t = c->tasks[run.task];
        for (uint32_t j = 0; j < run.count; ++j) {
            const size_t i = run.first + j, li = i - t.base;
            const uint8_t flag = t.flag[li];
            if ((flag & kCmdList) && !repeats_queued(c, t, i, t.list_back[li])) { live_list = true; total_ids += t.n_ids[li]; }
            if (flag & kCmdNoPaint) painted = false;
        }
    }
    memset(out, 0, sizeof *out);
    out->g_end0 = g_end0;
    out->n_commands = G;
    out->evict_pages = c->evict_pages; out->evict_frames = c->evict_frames;
    out->fetch_pages = c->fetch_pages; out->fetch_frames = c->fetch_frames;
    PlanHeader h;
    memset(&h, 0, sizeof h);
    h.n_resident = c->n_resident; h.first_free = c->n_resident;
    if (G > 0) {
        PlanGeom g;
        plan_geometry(c, G, g);
        g.g_end0 = g_end0;
        // Range rules reach the sweeps as page ranges with their command's position; the sweeps paint them into LDS
        // tile by tile, and no per-page next use goes through memory.  Sweeps of many workgroups read the ranges
        // where they already are - the tasks' mirrors in device memory, a slice per run, repeats left out by the
        // reader - so that in steady state a plan sends nothing but its kernels' arguments.  Otherwise (one
        // workgroup, many runs, switched off) the ranges are listed here, and copied over if many workgroups read
        // them.  Plans with more ranges than the list holds scatter next uses into nu[], like id lists.
        g.resident = false;
        uint32_t n_ranges = 0;
        // (A plan whose id lists are staged copies its ranges in the same kernel, and a copied list is the cheaper
        // one to read: the mirrors are for plans that would otherwise stage nothing.)
        if (painted && c->resident_ranges && !live_list && !g.single &&
            c->runs.size() <= std::min<size_t>(kMaxRangeRuns, g.waves)) {
            RangeRuns &rr = c->range_runs;
            uint64_t total = 0;
            rr.n = 0;
            // Only what is in the mirrors already: ranges of launches queued since the last migration (or a task's
            // first plan) are listed and copied once more - cheaper on the plan's path than an upload - and the
            // migration that follows brings the mirrors up to date behind its copy.
            bool all_there = true;
            for (const PlanRun &run : c->runs) {
                TaskQueue &t = c->tasks[run.task];
                const uint64_t q0 = t.range_begin(run.first), q1 = t.range_end[run.first + run.count - 1 - t.base];
                if (q1 > q0 && (t.rng_dev == nullptr || t.rng_uploaded < q1)) { t.want_mirror = true; all_there = false; }
            }
            if (!all_there) total = (uint64_t)kMaxResidentRanges + 1;
            for (const PlanRun &run : c->runs) {               // run j of the table is run j of the timeline
                if (!all_there) break;
                TaskQueue &t = c->tasks[run.task];
                const uint64_t q0 = t.range_begin(run.first), q1 = t.range_end[run.first + run.count - 1 - t.base];
                total += q1 - q0;
                if (total > kMaxResidentRanges) break;
                RangeRun &r = rr.run[rr.n++];
                r = RangeRun{};
                r.ring = t.rng_dev; r.mask = (uint32_t)(t.rng_cap - 1); r.first = (uint32_t)q0; r.count = (uint32_t)(q1 - q0);
                if (r.count == 0) {                            // nothing to read, but the reader's load is unconditional: 16 readable bytes
                    r.ring = reinterpret_cast<const RangeRec *>(c->flags); r.mask = 0; r.first = 0;
                }
                r.cmd_first = (uint32_t)run.first; r.g0 = run.g0; r.cursor = (uint32_t)t.cursor; r.dedupe = c->dedupe_regions ? 1u : 0u;
            }
            if (total <= kMaxResidentRanges) {
                g.resident = true;
                n_ranges = (uint32_t)total;
            }
        }
        if (painted && !g.resident) {
            for (const PlanRun &run : c->runs) {
                const TaskQueue &t = c->tasks[run.task];
                for (uint32_t j = 0; j < run.count && painted; ++j) {
                    const size_t i = run.first + j, li = i - t.base;
                    const uint32_t gpos = run.g0 + j;
                    for (uint64_t q = t.range_begin(i), q1 = t.range_end[li]; q < q1; ++q) {
                        const RangeRec &rec = t.range_at(q);
                        if (repeats_queued(c, t, i, rec.back)) continue;
                        if (n_ranges == kMaxRanges) { painted = false; break; }
                        c->ranges_host[n_ranges++] = PageRange{rec.lo, rec.hi, gpos, 0};
                    }
                }
            }
        }
        g.painted = painted;
        g.n_ranges = painted ? n_ranges : 0;
        g.use_nu = !painted || live_list;
        g.live_list = live_list;
        const size_t need = (size_t)g.n_chunks * g.n_keys;
        if (need > c->matrix_cap) {
            HIP_TRY(c, hipStreamSynchronize(c->stream));
            if (c->matrix) HIP_TRY(c, hipFree(c->matrix));
            c->matrix = nullptr; c->matrix_cap = 0;
            HIP_TRY(c, hipMalloc((void **)&c->matrix, need * 4 * 2));     // counts, and behind them the chunk start positions
            c->matrix_cap = need;
        }
        // Id lists: how many ids does this plan carry (repeated lists excluded)?  Many -> bucket path.
        g.list_binned = false;
        g.list_prepared = false;
        g.n_list_sources = g.n_list_new = 0;
        g.n_buckets = (uint32_t)((c->V + (1u << kBucketShift) - 1) >> kBucketShift);
        g.split = prep_split(g.n_buckets, c->prep_split_max);
        c->reserved.clear();
        if (c->has_list_rule && g.n_buckets <= kMaxBuckets) {
            const bool many = live_list && total_ids >= c->list_binned_min_ids && total_ids < (1ull << 31);
            if (many && c->list_prepared) {
                const int rc_src = gather_list_sources(c, g);
                if (rc_src < 0) return rc_src;
                g.list_prepared = rc_src == 0;
            }
            c->last_plan_prepared = g.list_prepared;
            if (many && !g.list_prepared) {
                g.list_binned = true;
                // room per sub-segment (8 per bucket): four times the average, at least 256 pairs
                g.bucket_cap = (uint32_t)std::max<uint64_t>(256, 4 * total_ids / ((uint64_t)g.n_buckets * 8) + 1);
                const size_t pairs = (size_t)g.n_buckets * 8 * g.bucket_cap;
                if (!c->list_bucket_fill) HIP_TRY(c, hipMalloc((void **)&c->list_bucket_fill, 4 * kMaxBuckets * 8));
                if (pairs > c->list_cap) {
                    HIP_TRY(c, hipStreamSynchronize(c->stream));
                    if (c->list_pairs) HIP_TRY(c, hipFree(c->list_pairs));
                    c->list_pairs = nullptr; c->list_cap = 0;
                    HIP_TRY(c, hipMalloc((void **)&c->list_pairs, (pairs + pairs / 4) * 4));
                    c->list_cap = pairs + pairs / 4;
                }
            }
        }
        // From here to the launch, a failure must give the reserved ring blocks back: the records would otherwise
        // point at blocks that hold no list, and the next plan would merge whatever is in them.
        struct GiveBack {
            msched_ctx *c; bool armed = true;
            ~GiveBack() { if (armed) undo_reservations(c); }
        } give_back{c};
        // The kernels that read whole records (next uses scattered per page, id lists binned per plan or expanded
        // directly) find them through a table of record addresses, one per position; painted plans whose lists
        // are prepared need no record on the device.
        g.needs_records = !painted || (live_list && !g.list_prepared);
        if (g.needs_records) {
            for (const PlanRun &run : c->runs) {
                const TaskQueue &t = c->tasks[run.task];
                for (uint32_t j = 0; j < run.count; ++j) {
                    const size_t i = run.first + j;
                    c->cmd_ptrs_host[run.g0 + j] = reinterpret_cast<const CmdRec *>(
                        reinterpret_cast<uintptr_t>(t.recs_dev + (i - t.base)) | (skip_mask(c, t, i) << 56));
                }
            }
        }
        if (c->epoch == kMaxEpoch) {                 // the epoch field is about to wrap: start over
            HIP_TRY(c, launch_nu_reset(c));
            c->epoch = 0;
        }
        ++c->epoch;
        const clk::time_point t_prep = clk::now();
        if (++c->hdr_seq == 0) c->hdr_seq = 1;
        HIP_TRY(c, launch_plan(c, g));
        give_back.armed = false;                      // the preparation is queued: the blocks will hold their lists
        c->reserved.clear();
        const clk::time_point t_launch = clk::now();
        // The counts are all the caller waits for: the cut stamps the pinned header once they (and need[]) are
        // written, while the second sweep is still filling the lists, which only stream-ordered work reads.
        const volatile uint32_t *stamp = &c->hdr_host->seq;
        bool landed = false;
        if (c->plan_spin) {
            for (uint32_t spins = 0; !(landed = *stamp == c->hdr_seq); ++spins)
                if ((spins & 0xfff) == 0xfff && hipStreamQuery(c->stream) != hipErrorNotReady) break;   // finished or failed
            (void)hipGetLastError();                    // hipErrorNotReady from the queries is not an error
        }
        if (!landed) {
            HIP_TRY(c, hipStreamSynchronize(c->stream));
            if (*stamp != c->hdr_seq) { c->last_hip = g_last_hip = (int)hipErrorUnknown; return MSCHED_E_HIP; }
        }
        std::atomic_thread_fence(std::memory_order_acquire);
        h = *c->hdr_host;
        const clk::time_point t_done = clk::now();
        c->phase_ms[MSCHED_HOST_PREP] = std::chrono::duration<float, std::milli>(t_prep - t_start).count();
        c->phase_ms[MSCHED_HOST_LAUNCH] = std::chrono::duration<float, std::milli>(t_launch - t_prep).count();
        c->phase_ms[MSCHED_HOST_WAIT] = std::chrono::duration<float, std::milli>(t_done - t_launch).count();
        c->plan_timing_pending = c->profiling != 0;     // read from the events when somebody asks (that waits for the stream)
        if (h.status & kStatRange) return MSCHED_E_RANGE;
        if (h.status & kStatWset) return MSCHED_E_WSET_TOO_LARGE;
    }
    out->n_fetch = h.n_fetch; out->n_evict = h.n_evict; out->n_free_used = h.n_free_used;
    out->g_cut = h.g_cut; out->covered_launches = h.g_cut;
    out->plan_id = ++c->plan_seq;
    c->plan_early = c->early;
    c->early_tag = (uint32_t)out->plan_id ? (uint32_t)out->plan_id : 1u;
    c->pending_plan = out->plan_id;
    c->pending = h;
    return MSCHED_OK;
}

// Bin the id lists of commands queued behind the ones just planned, while the migration keeps the host link
// busy and most compute units idle: the next plan then finds them prepared.  Blocks are handed out in program
// order, so a task stops at the first command that does not fit its ring.
void prepare_ahead(msched_ctx *c) {
    if (!c->list_ahead || !c->list_prepared || !c->last_plan_prepared) return;
    const uint32_t n_buckets = (uint32_t)((c->V + (1u << kBucketShift) - 1) >> kBucketShift);
    // Look-ahead is an optimisation: whatever goes wrong here switches it off and leaves the lists to the plans.
    auto give_up = [&](hipError_t e) { c->last_hip = g_last_hip = (int)e; (void)hipGetLastError(); c->list_ahead = 0; };
    hipError_t e;
    if (!c->list_ahead_host &&
        (e = hipHostMalloc((void **)&c->list_ahead_host, sizeof(ListPrep) * kMaxListSources, hipHostMallocDefault)) != hipSuccess) {
        c->list_ahead_host = nullptr;
        return give_up(e);
    }
    if (!c->list_ahead_dev && (e = hipHostGetDevicePointer((void **)&c->list_ahead_dev, c->list_ahead_host, 0)) != hipSuccess)
        return give_up(e);
    if (!c->ahead_ev && (e = hipEventCreateWithFlags(&c->ahead_ev, hipEventDisableTiming)) != hipSuccess) {
        c->ahead_ev = nullptr;
        return give_up(e);
    }
    if (c->ahead_pending) {                                  // the table is free again once the last batch has been read
        if ((e = hipEventSynchronize(c->ahead_ev)) != hipSuccess) return give_up(e);
        c->ahead_pending = false;
    }
    const uint64_t split = prep_split(n_buckets, c->prep_split_max), hdr_words = (uint64_t)prep_part_buckets(n_buckets, (uint32_t)split) + 2;
    uint32_t n_new = 0;
    bool full = false;
    struct Fresh { uint32_t task; size_t li; };
    std::vector<Fresh> fresh;
    std::vector<size_t> scan0(c->tasks.size());
    auto forget = [&]() {                                      // nothing of this batch was (or will be) binned
        for (const Fresh &f : fresh) c->tasks[f.task].prep[f.li] = 0;
        for (size_t ti = 0; ti < c->tasks.size(); ++ti) c->tasks[ti].prep_scan = scan0[ti];
    };
    for (size_t ti = 0; ti < c->tasks.size(); ++ti) {
        TaskQueue &t = c->tasks[ti];
        scan0[ti] = t.prep_scan;
        size_t i = std::max(t.prep_scan, t.cursor);
        const size_t end = std::min(t.n, t.cursor + (size_t)c->list_ahead);
        for (; i < end && !full; ++i) {
            const size_t li = i - t.base;
            if (!(t.flag[li] & kCmdList) || t.prep[li]) continue;
            const uint32_t n_ids = t.n_ids[li];
            const uint32_t pieces = (n_ids + kPrepBlock - 1) / kPrepBlock;
            if (n_new + pieces > kMaxListSources) { full = true; break; }
            const uint64_t bytes = (split * ((uint64_t)pieces * hdr_words + n_ids) * 4 + 15) & ~15ull;
            uint64_t off;
            if (!ring_alloc(c, t, bytes, off)) break;        // no room now: the plan that needs it will see to it
            t.prep[li] = off + 1;
            fresh.push_back({(uint32_t)ti, li});
            uint32_t *block = reinterpret_cast<uint32_t *>(t.prep_buf + off % t.prep_size);
            for (uint32_t p = 0; p < pieces; ++p) {
                const uint32_t n = std::min<uint32_t>(kPrepBlock, n_ids - p * kPrepBlock);
                c->list_ahead_host[n_new++] = {t.ids[li] + (size_t)p * kPrepBlock, block, n, {0, 0, 0}};
                block += split * (hdr_words + n);
            }
        }
        t.prep_scan = i;
        if (full) break;
    }
    if (n_new == 0) return;
    const bool timed = c->profiling && hipEventRecord(c->ev[8], c->stream) == hipSuccess;
    if ((e = launch_list_prepare(c, c->list_ahead_dev, n_new, n_buckets, (uint32_t)split)) != hipSuccess ||
        (e = hipEventRecord(c->ahead_ev, c->stream)) != hipSuccess) {
        // nothing was binned: the records must not point at blocks that hold no list
        // (a launch that did go out before a failed record is waited for, so the table is not rewritten under it)
        (void)hipStreamSynchronize(c->stream);
        forget();
        return give_up(e);
    }
    c->ahead_pending = true;
    if (timed && hipEventRecord(c->ev[9], c->stream) == hipSuccess) c->prepare_timed = 1;
}

}  // namespace

int msched_migrate(msched_ctx *c, const msched_plan_t *plan) {
    if (!c || !plan) return MSCHED_E_INVAL;
    if (c->pending_plan == 0 || plan->plan_id != c->pending_plan) return MSCHED_E_STALE_PLAN;
    if (c->profiling) HIP_TRY(c, hipEventRecord(c->ev[5], c->stream));
    HIP_TRY(c, launch_migrate(c, c->pending));
    if (c->profiling) { HIP_TRY(c, hipEventRecord(c->ev[6], c->stream)); c->migrate_timed = 1; }
    c->n_resident += c->pending.n_free_used;
    c->pending_plan = 0;
    c->prepare_timed = 0;
    const int rc_prep = guarded([&]() -> int { prepare_ahead(c); return MSCHED_OK; });
    if (rc_prep) return rc_prep;
    // Ranges of launches queued since the last migration go to the tasks' mirrors now, behind the copy, so that the
    // next plans find them there.
    if (c->resident_ranges)
        for (TaskQueue &t : c->tasks)
            if (t.want_mirror) { const int rc_up = upload_ranges(c, t); if (rc_up) return rc_up; }
    return MSCHED_OK;
}

int msched_set_early_start(msched_ctx *c, int enable) {
    if (!c) return MSCHED_E_INVAL;
    if (enable && !c->early_ready) {
        // First use: bookkeeping of the in-order landing.  Each piece on its own, so that a failure half-way neither
        // leaks nor leaves a hole; early execution stays off until all of them exist.
        auto zeroed = [&](uint32_t **ptr, size_t bytes) -> hipError_t {
            if (*ptr) return hipSuccess;
            uint32_t *m = nullptr;
            hipError_t e = hipMalloc((void **)&m, bytes);
            if (e != hipSuccess) return e;
            if ((e = hipMemset(m, 0, bytes)) != hipSuccess) { (void)hipFree(m); return e; }
            *ptr = m;
            return hipSuccess;
        };
        HIP_TRY(c, zeroed(&c->page_done, (size_t)c->F * 4));
        HIP_TRY(c, zeroed(&c->chunks_done, (size_t)c->F * 4));
        HIP_TRY(c, zeroed(&c->landed, 256));
        if (!c->need_host)
            HIP_TRY(c, hipHostMalloc((void **)&c->need_host, (MSCHED_MAX_TIMELINE_COMMANDS + 1) * 4, hipHostMallocDefault));
        if (!c->progress_host) {
            HIP_TRY(c, hipHostMalloc((void **)&c->progress_host, 64, hipHostMallocDefault));
            *c->progress_host = 0;
        }
        if (!c->gate_host) {
            HIP_TRY(c, hipHostMalloc((void **)&c->gate_host, sizeof(GateRec) * (MSCHED_MAX_TIMELINE_COMMANDS + 1), hipHostMallocDefault));
            memset(c->gate_host, 0, sizeof(GateRec) * (MSCHED_MAX_TIMELINE_COMMANDS + 1));
        }
        if (!c->poll_stream) HIP_TRY(c, hipStreamCreateWithFlags(&c->poll_stream, hipStreamNonBlocking));
        HIP_TRY(c, launch_peek(c));                          // the first launch on a stream sets up its queue: not during a migration
        HIP_TRY(c, hipDeviceSynchronize());
        c->early_ready = true;
    }
    c->early = enable ? 1 : 0;
    return MSCHED_OK;
}

int msched_plan_ready_need(msched_ctx *c, const msched_plan_t *plan, uint32_t *need) {
    if (!c || !plan || (plan->covered_launches && !need)) return MSCHED_E_INVAL;
    if (plan->plan_id != c->plan_seq || !c->plan_early) return MSCHED_E_STALE_PLAN;
    if (plan->covered_launches)                                // written by the plan's kernels, which have finished
        memcpy(need, c->need_host, (size_t)plan->covered_launches * 4);
    return MSCHED_OK;
}

int msched_gate_enqueue(msched_ctx *c, const msched_plan_t *plan, uint32_t g, void *stream, uint32_t timeout_us) {
    if (!c || !plan) return MSCHED_E_INVAL;
    if (plan->plan_id != c->plan_seq || !c->plan_early || !c->early_ready) return MSCHED_E_STALE_PLAN;
    if (c->pending_plan != 0) return MSCHED_E_STALE_PLAN;       // not migrated yet: see the header
    if (g >= plan->covered_launches || (hipStream_t)stream == c->stream) return MSCHED_E_INVAL;   // on the context's own stream it would wait for itself
    const uint64_t ticks = (uint64_t)(timeout_us ? timeout_us : 2000000u) * 100u;                   // 100 MHz wall clock
    c->gate_host[g].status = 0;
    std::atomic_thread_fence(std::memory_order_release);
    HIP_TRY(c, launch_gate(c, g, c->need_host[g], ticks, (hipStream_t)stream));
    return MSCHED_OK;
}

int msched_gate_result(msched_ctx *c, uint32_t g, uint32_t *status, float *ready_ms) {
    if (!c || g > MSCHED_MAX_TIMELINE_COMMANDS) return MSCHED_E_INVAL;
    if (!c->gate_host) return MSCHED_E_STALE_PLAN;
    const uint32_t st = *(volatile uint32_t *)&c->gate_host[g].status;
    std::atomic_thread_fence(std::memory_order_acquire);
    if (status) *status = st;
    if (ready_ms) *ready_ms = st == 1 ? (float)((double)c->gate_host[g].ticks / 1e5) : 0.f;
    return MSCHED_OK;
}

int msched_progress(msched_ctx *c, uint32_t *landed) {
    if (!c || !landed) return MSCHED_E_INVAL;
    if (!c->early_ready) { *landed = 0; return MSCHED_OK; }
    HIP_TRY(c, launch_peek(c));
    HIP_TRY(c, hipStreamSynchronize(c->poll_stream));
    *landed = *c->progress_host;
    return MSCHED_OK;
}

int msched_pagetable_query(msched_ctx *c, const uint64_t *page_ids, uint32_t n, uint32_t *out) {
    if (!c || (n && (!page_ids || !out))) return MSCHED_E_INVAL;
    for (uint32_t i = 0; i < n; ++i) if (page_ids[i] >= c->V) return MSCHED_E_RANGE;
    if (n == 0) return MSCHED_OK;
    if ((size_t)n * 2 > c->query_cap) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        if (c->query_buf) HIP_TRY(c, hipFree(c->query_buf));
        c->query_buf = nullptr; c->query_cap = 0;
        HIP_TRY(c, hipMalloc((void **)&c->query_buf, (size_t)n * 2 * 4));
        c->query_cap = (size_t)n * 2;
    }
    return guarded([&]() -> int {
        std::vector<uint32_t> ids(n);
        for (uint32_t i = 0; i < n; ++i) ids[i] = (uint32_t)page_ids[i];
        HIP_TRY(c, hipMemcpyAsync(c->query_buf, ids.data(), (size_t)n * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, launch_query(c, c->query_buf, n, c->query_buf + n));
        HIP_TRY(c, hipMemcpyAsync(out, c->query_buf + n, (size_t)n * 4, hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        return MSCHED_OK;
    });
}

int msched_pagetable_query_static(msched_ctx *c, const uint64_t *page_ids, uint32_t n, uint32_t *out) {
    if (!c || (n && (!page_ids || !out))) return MSCHED_E_INVAL;
    if (n > MSCHED_QUERY_STATIC_MAX) return MSCHED_E_TOO_LARGE;
    for (uint32_t i = 0; i < n; ++i) if (page_ids[i] >= c->V) return MSCHED_E_RANGE;
    if (n == 0) return MSCHED_OK;
    HIP_TRY(c, query_static(c, page_ids, n, out));
    return MSCHED_OK;
}

int msched_plan_copy_lists(msched_ctx *c, const msched_plan_t *plan, uint32_t *evict_pages, uint32_t *evict_frames,
                           uint32_t *fetch_pages, uint32_t *fetch_frames) {
    if (!c || !plan) return MSCHED_E_INVAL;
    if (plan->plan_id != c->plan_seq) return MSCHED_E_STALE_PLAN;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    const size_t ne = (size_t)plan->n_evict * 4, nf = (size_t)plan->n_fetch * 4;
    if (evict_pages && ne) HIP_TRY(c, hipMemcpy(evict_pages, c->evict_pages, ne, hipMemcpyDeviceToHost));
    if (evict_frames && ne) HIP_TRY(c, hipMemcpy(evict_frames, c->evict_frames, ne, hipMemcpyDeviceToHost));
    if (fetch_pages && nf) HIP_TRY(c, hipMemcpy(fetch_pages, c->fetch_pages, nf, hipMemcpyDeviceToHost));
    if (fetch_frames && nf) HIP_TRY(c, hipMemcpy(fetch_frames, c->fetch_frames, nf, hipMemcpyDeviceToHost));
    return MSCHED_OK;
}

int msched_state_copy(msched_ctx *c, uint32_t *page_table, uint32_t *frame_owner) {
    if (!c) return MSCHED_E_INVAL;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (page_table) HIP_TRY(c, hipMemcpy(page_table, c->page_table, c->V * 4, hipMemcpyDeviceToHost));
    if (frame_owner) HIP_TRY(c, hipMemcpy(frame_owner, c->frame_owner, (size_t)c->F * 4, hipMemcpyDeviceToHost));
    return MSCHED_OK;
}

int msched_set_profiling(msched_ctx *c, int level) {
    if (!c || level < 0 || level > 2) return MSCHED_E_INVAL;
    c->profiling = level;
    for (float &m : c->phase_ms) m = 0.f;
    return MSCHED_OK;
}

int msched_get_phase_ms(msched_ctx *c, float *ms) {
    if (!c || !ms) return MSCHED_E_INVAL;
    if (c->plan_timing_pending) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        HIP_TRY(c, hipEventElapsedTime(&c->phase_ms[MSCHED_PHASE_PLAN], c->ev[0], c->ev[4]));
        if (c->profiling >= 2)
            for (int i = 0; i < 4; ++i) HIP_TRY(c, hipEventElapsedTime(&c->phase_ms[i], c->ev[i], c->ev[i + 1]));
        c->plan_timing_pending = false;
    }
    if (c->profiling && c->migrate_timed) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        HIP_TRY(c, hipEventElapsedTime(&c->phase_ms[MSCHED_PHASE_MIGRATE], c->ev[5], c->ev[6]));
        c->phase_ms[MSCHED_PHASE_PREPARE] = 0.f;
        if (c->prepare_timed) HIP_TRY(c, hipEventElapsedTime(&c->phase_ms[MSCHED_PHASE_PREPARE], c->ev[8], c->ev[9]));
    }
    for (int i = 0; i < MSCHED_N_PHASES; ++i) ms[i] = c->phase_ms[i];
    return MSCHED_OK;
}

const char *msched_strerror(int code) {
    switch (code) {
        case MSCHED_OK: return "ok";
        case MSCHED_E_INVAL: return "invalid argument";
        case MSCHED_E_RANGE: return "page, slot or argument index out of range";
        case MSCHED_E_OVERFLOW: return "template arithmetic overflows 64 bits";
        case MSCHED_E_WSET_TOO_LARGE: return "first command's working set exceeds the frame pool";
        case MSCHED_E_STALE_PLAN: return "plan is not the latest or was already carried out";
        case MSCHED_E_NOMEM: return "out of memory";
        case MSCHED_E_HIP: return "HIP call failed";
        case MSCHED_E_TOO_LARGE: return "request exceeds a fixed-size buffer of the library";
        default: return "unknown error";
    }
}

int msched_last_hip_error(msched_ctx *c) { return c ? c->last_hip : g_last_hip; }

}  // extern "C"
