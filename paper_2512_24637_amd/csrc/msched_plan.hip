// Planning kernels for gfx950: template expansion + next-use scatter, per-chunk class
// histograms over the page table, budget cut / victim threshold, and the ordered emission
// of the fetch and eviction lists.
//
// Method (paper: arXiv 2512.24637, Sec. 5.2 and Sec. 6.1-6.2): every page gets nu[p] = position
// of the first future command that touches it ("never" if the timeline does not).  The fetch
// list is the non-resident pages with nu < g_cut ordered by (nu, page id); the eviction list is
// the resident pages with nu >= g_cut ordered by (nu descending with "never" first, page id),
// truncated to what the fetches need.  Both orders are "class (a small integer) then page id",
// so the lists come out of one stable counting sort whose classes are the G+1 possible values of
// nu: a workgroup owns a contiguous chunk of the page table, counts its pages per class, a small
// kernel turns the chunk x class counts into output offsets, and a second sweep writes each page
// straight to its final position.  No comparison sort, no per-command bitmaps.
//
// nu[] is never reset: an entry holds (epoch << 12) | (4095 - g), the epoch grows by one per plan
// and the scatter is an atomic max, so entries of earlier plans read as "never" and the smallest
// g of the current plan wins.
#include <algorithm>

#include <cstdlib>
#include <cstring>

#include "msched_internal.h"

// In-kernel timers, a compile-time option (-DMSCHED_KERNEL_TIMERS; paper_2512_24637_amd/build.py build(timers=True)
// writes libmsched_timers.so beside the library): thread 0 of every workgroup of an instrumented kernel stores the
// 100 MHz wall clock at the kernel's phase boundaries, slot i of the workgroup's row of 16 in the kernel's table
// of 4096 rows, in a device buffer of 8 tables the caller hands over with msched_debug_set_ticks (exported by that
// build only; null switches the timers off).  Compiled out otherwise.
#ifdef MSCHED_KERNEL_TIMERS
static __device__ uint64_t *g_ticks = nullptr;
#define MSCHED_TICK(kernel, i)                                                                              \
    do {                                                                                                    \
        if (threadIdx.x == 0 && g_ticks != nullptr && blockIdx.x < 4096)                                    \
            g_ticks[((size_t)(kernel) * 4096 + blockIdx.x) * 16 + (i)] = wall_clock64();                    \
    } while (0)
extern "C" int msched_debug_set_ticks(uint64_t *buf) {
    return hipMemcpyToSymbol(HIP_SYMBOL(g_ticks), &buf, sizeof buf) == hipSuccess ? MSCHED_OK : MSCHED_E_HIP;
}
#else
#define MSCHED_TICK(kernel, i) do { } while (0)
#endif
enum { kTickPrepare = 0, kTickCount = 1, kTickCut = 2, kTickEmit = 3, kTickStage = 4 };

namespace msched {

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ uint64_t lanes_below() { return (1ull << lane_id()) - 1ull; }

// ------------------------------------------------------------------------------------------
// Stage the G command records of this plan from pinned host memory into device memory (one
// pass over the link instead of one round trip per expansion workgroup).  Short timelines skip this
// and let the few expansion workgroups read their record through the pinned table themselves.
// ------------------------------------------------------------------------------------------
// When the first sweep merges the id lists itself (k_count_lists), one more workgroup rides along and writes the
// order in which that sweep takes its chunks.
struct ChunkOrder {
    const uint32_t *bucket_mark;        // null: no order wanted
    uint32_t n_buckets, n_chunks, buckets_per_chunk;
    uint32_t first_rank;                // marks from this value on put a chunk first; smaller non-zero ones second
    uint32_t *order;                    // [n_chunks] chunks that hold a bucket with ids first, then the others
};
__device__ void chunk_order_block(const ChunkOrder &o);

__global__ __launch_bounds__(256) void k_stage(const CmdRec *const *__restrict__ cmd_ptrs, uint32_t G,
                                                CmdRec *__restrict__ cmd_dev, uint32_t *__restrict__ bucket_fill,
                                                uint32_t n_buckets, const PageRange *__restrict__ ranges_src,
                                                PageRange *__restrict__ ranges_dst, uint32_t n_ranges,
                                                const ListSource *__restrict__ list_src, ListSource *__restrict__ list_dst,
                                                uint32_t n_list_src, ChunkOrder co) {
    uint32_t n_blocks = gridDim.x;
    if (co.bucket_mark != nullptr) {                        // the last workgroup is the extra one
        if (blockIdx.x == --n_blocks) { chunk_order_block(co); return; }
    }
    const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    for (uint32_t i = t; i < n_list_src; i += n_blocks * blockDim.x)                      // and so does the table of list pieces
        reinterpret_cast<uint4 *>(list_dst)[i] = reinterpret_cast<const uint4 *>(list_src)[i];
    for (uint32_t b = t; b < n_buckets; b += n_blocks * blockDim.x) bucket_fill[b] = 0;   // binned id lists start empty
    for (uint32_t r = t; r < n_ranges; r += n_blocks * blockDim.x)                        // the range list rides along
        reinterpret_cast<uint4 *>(ranges_dst)[r] = reinterpret_cast<const uint4 *>(ranges_src)[r];
    const uint32_t g = t >> 3, part = t & 7;
    if (g >= G) return;
    const uint64_t tagged = reinterpret_cast<uint64_t>(cmd_ptrs[g]);
    const uint4 *src = reinterpret_cast<const uint4 *>(tagged & kPtrMask);
    uint4 v = src[part];
    if (part == 1) { v.z = (uint32_t)(tagged >> 56); v.w = 0; }       // CmdRec::reserved <- skip mask
    reinterpret_cast<uint4 *>(cmd_dev + g)[part] = v;
}

// ------------------------------------------------------------------------------------------
// Template expansion + next-use scatter (Sec. 5.2 templates; Sec. 6.2 access order).
// One workgroup per (command g, rule r, split s).  An entry only ever grows while this kernel
// runs, so a plain load that already shows a value >= ours lets the atomic be skipped.
// ------------------------------------------------------------------------------------------
struct ExpandArgs {
    const CmdRec *cmds;                 // staged records, or null: read through cmd_ptrs
    const CmdRec *const *cmd_ptrs; uint32_t G;
    const DevKernel *kernels;
    uint32_t *nu; const uint32_t *slot; uint32_t *flags;
    uint64_t V; uint32_t page_shift, n_split, epoch_base;   // epoch_base = epoch << kNuShift
};

__device__ __forceinline__ void touch(const ExpandArgs &a, uint32_t p, uint32_t enc) {
    if (a.slot != nullptr && a.slot[p] == kNone) { atomicOr(a.flags, kStatRange); return; }
    if (a.nu[p] < enc) atomicMax(&a.nu[p], enc);
}

// Items t0, t0 + step, ... < n of a page sequence, kBatch at a time: all page ids first, then all
// current entries, then the atomics (which return nothing and are not waited for), so a lane keeps
// kBatch independent memory round trips in flight instead of one dependent chain per page.
// With kDedupe (explicit id lists, where popular pages repeat many times inside one command) a small
// direct-mapped table in LDS remembers pages this workgroup has already handled: every workgroup
// writes one value only, so a repeat can be dropped before it reaches memory.  The table is a filter,
// not a set: a lost race or an evicted entry only costs a redundant atomic.
constexpr int kBatch = 8;
constexpr uint32_t kListSeenBits = 15;     // entries (log2) of the duplicate filter of k_expand_list
constexpr int kListThreads = 1024;
template <bool kDedupe, typename PageOf>
__device__ __forceinline__ void touch_many(const ExpandArgs &a, uint64_t t0, uint64_t step, uint64_t n, uint32_t enc,
                                           uint32_t *seen, uint32_t seen_bits, PageOf page_of) {
    for (uint64_t i0 = t0; i0 < n; i0 += step * kBatch) {
        uint32_t p[kBatch], cur[kBatch];
        bool ok[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const uint64_t i = i0 + (uint64_t)j * step;
            ok[j] = i < n;
            p[j] = ok[j] ? page_of(i) : 0u;
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            if (ok[j] && p[j] >= a.V) { atomicOr(a.flags, kStatRange); ok[j] = false; }
            if (kDedupe && ok[j]) {
                // an LDS exchange also settles duplicates among the lanes of one instruction
                const uint32_t h = (p[j] * 2654435761u) >> (32 - seen_bits);
                if (atomicExch(&seen[h], p[j]) == p[j]) ok[j] = false;
            }
        }
        if (a.slot != nullptr) {
#pragma unroll
            for (int j = 0; j < kBatch; ++j)
                if (ok[j] && a.slot[p[j]] == kNone) { atomicOr(a.flags, kStatRange); ok[j] = false; }
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j) cur[j] = ok[j] ? a.nu[p[j]] : 0xFFFFFFFFu;
#pragma unroll
        for (int j = 0; j < kBatch; ++j)
            if (cur[j] < enc) atomicMax(&a.nu[p[j]], enc);
    }
}

__device__ __forceinline__ uint64_t formula(const uint64_t *args, uint64_t coeff, const uint8_t *idx, int n) {
    uint64_t v = coeff;
    for (int j = 0; j < n; ++j) v *= args[idx[j]];
    return v;
}

// The command record of position g into LDS: from the staged copy, or through the pinned table
// (whose entries carry the skip mask in their top byte).
__device__ __forceinline__ void load_record(const ExpandArgs &a, uint32_t g, uint64_t *s_rec) {
    if (threadIdx.x < sizeof(CmdRec) / 8) {
        if (a.cmds) {
            s_rec[threadIdx.x] = reinterpret_cast<const uint64_t *>(a.cmds + g)[threadIdx.x];
        } else {
            const uint64_t tagged = reinterpret_cast<uint64_t>(a.cmd_ptrs[g]);
            const uint64_t v = reinterpret_cast<const uint64_t *>(tagged & kPtrMask)[threadIdx.x];
            s_rec[threadIdx.x] = (threadIdx.x == 3) ? (tagged >> 56) : v;     // word 3 = CmdRec::reserved
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(256) void k_expand(ExpandArgs a) {
    const uint32_t g = blockIdx.x, r = blockIdx.y;
    __shared__ uint64_t s_rec[sizeof(CmdRec) / 8];
    load_record(a, g, s_rec);
    const CmdRec *rec = reinterpret_cast<const CmdRec *>(s_rec);
    const DevKernel &k = a.kernels[rec->kernel];
    if (r >= k.n_rules || ((rec->reserved >> r) & 1)) return;
    const msched_rule q = k.rules[r];
    const uint32_t sh = a.page_shift;
    const uint32_t enc = a.epoch_base | (kNuMask - g);
    const uint64_t t0 = blockIdx.z * (uint64_t)blockDim.x + threadIdx.x;
    const uint64_t step = a.n_split * (uint64_t)blockDim.x;

    if (q.kind == MSCHED_RULE_LIST) return;                 // id lists are expanded by k_expand_list
    uint64_t base = rec->args[q.base_arg];
    uint64_t size = (q.kind == MSCHED_RULE_FIXED) ? q.size_coeff
                                                  : formula(rec->args, q.size_coeff, q.size_args, q.n_size_args);
    if (size == 0) return;
    if (q.kind == MSCHED_RULE_STRIDED) {
        const uint64_t stride = formula(rec->args, q.stride_coeff, q.stride_args, q.n_stride_args);
        const uint64_t count = formula(rec->args, q.count_coeff, q.count_args, q.n_count_args);
        if (count == 0) return;
        if (size >= stride || count == 1) {
            size = (count - 1) * stride + size;             // the chunks abut or overlap: one range
        } else {
            const uint64_t max_pages = ((size - 1) >> sh) + 2;
            if (max_pages <= 8) {                           // many small chunks: a thread per chunk
                for (uint64_t j = t0; j < count; j += step) {
                    const uint64_t c0 = base + j * stride;
                    const uint64_t p0 = c0 >> sh, p1 = (c0 + size - 1) >> sh;
                    for (uint64_t p = p0; p <= p1; ++p) touch(a, (uint32_t)p, enc);
                }
            } else {                                        // few large chunks: threads across pages
                for (uint64_t j = 0; j < count; ++j) {
                    const uint64_t c0 = base + j * stride;
                    const uint64_t p0 = c0 >> sh, n = ((c0 + size - 1) >> sh) - p0 + 1;
                    touch_many<false>(a, t0, step, n, enc, nullptr, 0, [p0](uint64_t i) { return (uint32_t)(p0 + i); });
                }
            }
            return;
        }
    }
    const uint64_t p0 = base >> sh, n = ((base + size - 1) >> sh) - p0 + 1;
    touch_many<false>(a, t0, step, n, enc, nullptr, 0, [p0](uint64_t i) { return (uint32_t)(p0 + i); });
}

// Explicit page-id lists (sparse gathers).  One 1024-thread workgroup per command: popular pages repeat
// many times inside one list, and every repeat that reaches memory costs a random cache-line access, so
// the workgroup first drops repeats in a 32 Ki-entry direct-mapped table in LDS (gfx950 has 160 KiB per
// workgroup); what is left goes through the same check-then-atomic as the ranges.
__global__ __launch_bounds__(kListThreads) void k_expand_list(ExpandArgs a, uint32_t g0, uint32_t n_split,
                                                              uint32_t seen_bits) {
    const uint32_t g = g0 + blockIdx.x / n_split, split = blockIdx.x % n_split;
    __shared__ uint64_t s_rec[sizeof(CmdRec) / 8];
    __shared__ uint32_t seen[1u << kListSeenBits];
    load_record(a, g, s_rec);
    const CmdRec *rec = reinterpret_cast<const CmdRec *>(s_rec);
    const uint32_t n = rec->n_ids;
    if (n == 0) return;
    const DevKernel &k = a.kernels[rec->kernel];
    bool has_list = false;
    for (uint32_t r = 0; r < k.n_rules; ++r)
        has_list |= k.rules[r].kind == MSCHED_RULE_LIST && !((rec->reserved >> r) & 1);
    if (!has_list) return;
    for (uint32_t i = threadIdx.x; i < (1u << seen_bits); i += blockDim.x) seen[i] = kNone;
    __syncthreads();
    const uint32_t *ids = rec->ids;
    const uint32_t enc = a.epoch_base | (kNuMask - g);
    touch_many<true>(a, (uint64_t)split * blockDim.x + threadIdx.x, (uint64_t)n_split * blockDim.x, n, enc, seen, seen_bits,
                     [ids](uint64_t i) { return ids[i]; });
}

// ------------------------------------------------------------------------------------------
// Large id lists, binned.  Scattered single-lane atomics are the slowest thing this GPU does to
// memory (about 27 G/s measured, against 250 G/s for atomics on consecutive addresses and 100-200 G/s
// for scattered loads and stores), so when a plan carries many ids they do not touch nu[] one by one:
//   k_list_bin      per command, 24 Ki ids at a time: drop repeats in LDS, keep the survivors in LDS,
//                   count them per bucket of 8 Ki consecutive pages, reserve room in each bucket's
//                   segment with one global atomic per non-empty bucket, write (page in bucket, g) pairs
//   k_list_reduce   per bucket: max-reduce its pairs in a 32 KiB LDS table and merge the table into its
//                   own slice of nu[] with plain, dense loads and stores (nothing else writes nu[] while
//                   the list kernels run: the range expansion is launched after them on the same stream)
// A bucket's segment has room for four times the average; pairs that do not fit fall back to the
// check-then-atomic of the direct path, so any distribution is handled, a uniform one is handled fast.
// ------------------------------------------------------------------------------------------
__device__ uint32_t block_exclusive_scan(uint32_t *a, uint32_t n, uint32_t *wave_sums);
__device__ __forceinline__ uint32_t chunk_of_block(uint32_t block, uint32_t n_chunks);

constexpr uint32_t kBucketPages = 1u << kBucketShift;
constexpr uint32_t kBinSeenBits = 13;                       // duplicate filter: 8 Ki entries, 32 KiB
constexpr uint32_t kBinBlock = 24576;                       // ids handled per pass of k_list_bin (survivors: 96 KiB of LDS)

// Every bucket's segment is split into kBinLanes sub-segments with a fill counter each, and command g
// appends to sub-segment g % kBinLanes: hundreds of workgroups reserving room through one counter per
// bucket would queue up behind each other at that address.
constexpr uint32_t kBinLanes = 8;

struct ListArgs {
    ExpandArgs e;
    uint32_t *bucket_fill;          // [n_buckets][kBinLanes] pairs offered to each sub-segment (may exceed its room)
    uint32_t *pairs;                // [n_buckets][kBinLanes][sub_cap]: (page & (kBucketPages - 1)) | (g << kBucketShift)
    uint32_t n_buckets, sub_cap;
};

__global__ __launch_bounds__(kListThreads) void k_list_bin(ListArgs a, uint32_t n_split) {
    const uint32_t g = blockIdx.x / n_split, split = blockIdx.x % n_split;
    __shared__ uint64_t s_rec[sizeof(CmdRec) / 8];
    __shared__ uint32_t n_kept;
    extern __shared__ uint32_t bin_lds[];                   // 128 KiB + 4 per bucket (measured faster than smaller passes)
    uint32_t *seen = bin_lds;                               // [1 << kBinSeenBits]
    uint32_t *kept = seen + (1u << kBinSeenBits);           // [kBinBlock]
    uint32_t *cnt = kept + kBinBlock;                       // [n_buckets] survivors of this pass, then running write offset
    load_record(a.e, g, s_rec);
    const CmdRec *rec = reinterpret_cast<const CmdRec *>(s_rec);
    const DevKernel &k = a.e.kernels[rec->kernel];
    bool has_list = false;
    for (uint32_t r = 0; r < k.n_rules; ++r)
        has_list |= k.rules[r].kind == MSCHED_RULE_LIST && !((rec->reserved >> r) & 1);
    const uint32_t n_all = has_list ? rec->n_ids : 0;
    const uint32_t share = (n_all + n_split - 1) / n_split;             // this workgroup's part of the list
    const uint32_t first = min(n_all, split * share), n = min(n_all, first + share) - first;
    if (n == 0) return;
    for (uint32_t i = threadIdx.x; i < (1u << kBinSeenBits); i += blockDim.x) seen[i] = kNone;
    const uint32_t *ids = rec->ids + first;
    const uint32_t enc = a.e.epoch_base | (kNuMask - g);
    const int lane = lane_id();
    const uint64_t below = lanes_below();
    for (uint32_t block0 = 0; block0 < n; block0 += kBinBlock) {
        const uint32_t block_n = min(kBinBlock, n - block0);
        for (uint32_t b = threadIdx.x; b < a.n_buckets; b += blockDim.x) cnt[b] = 0;
        if (threadIdx.x == 0) n_kept = 0;
        __syncthreads();
        // 1. survivors of the duplicate filter go to LDS; count them per bucket
        for (uint32_t base = 0; base < block_n; base += blockDim.x * kBatch) {
            uint32_t p[kBatch];
            bool ok[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const uint32_t i = base + j * blockDim.x + threadIdx.x;
                ok[j] = i < block_n;
                p[j] = ok[j] ? ids[block0 + i] : 0u;
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                if (ok[j] && p[j] >= a.e.V) { atomicOr(a.e.flags, kStatRange); ok[j] = false; }
                if (ok[j] && a.e.slot != nullptr && a.e.slot[p[j]] == kNone) { atomicOr(a.e.flags, kStatRange); ok[j] = false; }
                if (ok[j]) {
                    const uint32_t h = (p[j] * 2654435761u) >> (32 - kBinSeenBits);
                    if (atomicExch(&seen[h], p[j]) == p[j]) ok[j] = false;
                }
                const uint64_t keep = __ballot(ok[j]);       // one LDS add per wavefront reserves the slots
                if (keep) {
                    uint32_t start = 0;
                    const int leader = __ffsll((long long)keep) - 1;
                    if (lane == leader) start = atomicAdd(&n_kept, (uint32_t)__popcll(keep));
                    start = __builtin_amdgcn_readlane(start, leader);
                    if (ok[j]) {
                        kept[start + __popcll(keep & below)] = p[j];
                        atomicAdd(&cnt[p[j] >> kBucketShift], 1u);
                    }
                }
            }
        }
        __syncthreads();
        // 2. one global atomic per non-empty bucket reserves this pass's room in its sub-segment
        const uint32_t sub = g % kBinLanes;
        for (uint32_t b = threadIdx.x; b < a.n_buckets; b += blockDim.x) {
            const uint32_t c = cnt[b];
            cnt[b] = c ? atomicAdd(&a.bucket_fill[b * kBinLanes + sub], c) : 0u;
        }
        __syncthreads();
        // 3. pairs out; what does not fit goes the direct way
        const uint32_t m = n_kept;
        for (uint32_t i = threadIdx.x; i < m; i += blockDim.x) {
            const uint32_t p = kept[i], b = p >> kBucketShift;
            const uint32_t pos = atomicAdd(&cnt[b], 1u);
            if (pos < a.sub_cap)
                a.pairs[((size_t)b * kBinLanes + sub) * a.sub_cap + pos] = (p & (kBucketPages - 1)) | (g << kBucketShift);
            else if (a.e.nu[p] < enc)
                atomicMax(&a.e.nu[p], enc);
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(kListThreads) void k_list_reduce(ListArgs a) {
    const uint32_t b = blockIdx.x;
    __shared__ uint32_t tab[kBucketPages];
    uint32_t fill[kBinLanes], any = 0;
#pragma unroll
    for (uint32_t l = 0; l < kBinLanes; ++l) { fill[l] = min(a.bucket_fill[b * kBinLanes + l], a.sub_cap); any |= fill[l]; }
    if (any == 0) return;
    for (uint32_t i = threadIdx.x; i < kBucketPages; i += blockDim.x) tab[i] = 0;
    __syncthreads();
    for (uint32_t l = 0; l < kBinLanes; ++l) {
        const uint32_t *seg = a.pairs + ((size_t)b * kBinLanes + l) * a.sub_cap;
        const uint32_t n = fill[l];
        for (uint32_t base = 0; base < n; base += blockDim.x * 4) {     // four loads in flight per lane
            uint32_t pr[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t i = base + j * blockDim.x + threadIdx.x;
                pr[j] = i < n ? seg[i] : kNone;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (pr[j] != kNone) atomicMax(&tab[pr[j] & (kBucketPages - 1)], kNuMask - (pr[j] >> kBucketShift));   // never 0
        }
    }
    __syncthreads();
    const uint64_t p0 = (uint64_t)b << kBucketShift;
    const uint64_t p1 = min(a.e.V, p0 + kBucketPages);
    for (uint64_t p = p0 + threadIdx.x; p < p1; p += blockDim.x) {
        const uint32_t v = tab[p - p0];
        const uint32_t cur = a.e.nu[p];
        const uint32_t enc = a.e.epoch_base | v;
        if (v && cur < enc) a.e.nu[p] = enc;                 // this workgroup is the only writer of its slice
    }
}

// ------------------------------------------------------------------------------------------
// Prepared id lists.  Binning a command's ids by bucket does not depend on the plan, only merging them under
// the command's position g does, and a queued command is planned again at every context switch until it has
// run.  So the first plan that sees a command bins its list once, into a block of its own (no shared
// cursors, no global atomics), and every plan merges the blocks of the commands in its timeline:
//   k_list_prepare  per new piece (up to 24 Ki ids): drop repeats in LDS, count per bucket, exclusive scan,
//                   write the bucket starts and the ids grouped by bucket
//   k_list_merge    per bucket: gather that bucket's ids from every piece of the plan, max-reduce them under
//                   their commands' g in a 32 KiB LDS table, merge the table into the bucket's slice of nu[]
//   k_count_lists   large tables, whose sweep tiles are exactly one bucket: the first sweep gathers the bucket's
//                   ids itself, into its LDS tile, and nu[] is neither written nor read (count_body)
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kListThreads) void k_list_prepare(const ListPrep *__restrict__ prep, uint32_t n_buckets,
                                                               uint32_t split, uint64_t V, const uint32_t *__restrict__ slot,
                                                               uint32_t *__restrict__ bucket_mark) {
    extern __shared__ uint32_t bin_lds[];
    uint32_t *seen = bin_lds;                               // [1 << kBinSeenBits]
    uint32_t *cnt = seen + (1u << kBinSeenBits);            // [buckets of the part + 1] counts, then starts, then write cursors
    __shared__ uint32_t bad;
    __shared__ uint32_t wave_sums[kListThreads / kWave];
    // A piece is prepared by prep_split workgroups, neighbours in dispatch order: each reads all its ids (the
    // second to fourth reader find them in the L2) and keeps those of its own range of buckets, a part of the work
    // in LDS and of the output each.  One workgroup per piece left most of the chip idle: a context switch brings a
    // few dozen new commands.
    const uint32_t per_part = prep_part_buckets(n_buckets, split);
    const uint32_t part = blockIdx.x % split;
    const ListPrep pr = prep[blockIdx.x / split];
    const uint32_t n = min(pr.n, kPrepBlock);
    // part q takes the buckets q, q + split, q + 2 split, ...: a gather's pages sit in one region of the page table,
    // and consecutive ranges of buckets would leave all of them to one part
    const uint32_t nb = part < n_buckets ? (n_buckets - part + split - 1) / split : 0;   // buckets of this part
    MSCHED_TICK(kTickPrepare, 0);
    for (uint32_t i = threadIdx.x; i < (1u << kBinSeenBits); i += blockDim.x) seen[i] = kNone;
    for (uint32_t b = threadIdx.x; b <= per_part; b += blockDim.x) cnt[b] = 0;
    if (threadIdx.x == 0) bad = 0;
    __syncthreads();
    MSCHED_TICK(kTickPrepare, 1);
    // A piece is at most kPrepBlock = 24 x 1024 ids, 24 per thread.  The work on them is done in passes over all of
    // a thread's ids, so that the round trips of one pass (memory, or an LDS operation whose result is needed)
    // overlap instead of queueing up id by id: all loads; look-ups and exchanges with the table of repeats, four
    // ids at a time; counts per bucket.  What a thread keeps stays in its registers (24 ids and a mask) until the
    // bucket starts are known and it writes them out: no copy of the survivors in LDS (96 KiB less of it).
    constexpr int kPerThread = kPrepBlock / kListThreads;
    static_assert(kPerThread * kListThreads == (int)kPrepBlock, "a thread's share of a piece");
    uint32_t p[kPerThread];
    uint32_t ok = 0;                                      // bit j: id j of this thread is (still) to be kept
    {
#pragma unroll
        for (int j = 0; j < kPerThread; ++j) {
            const uint32_t i = j * blockDim.x + threadIdx.x;
            p[j] = i < n ? pr.ids[i] : 0u;
            if (i < n) ok |= 1u << j;
        }
#pragma unroll
        for (int j = 0; j < kPerThread; ++j) {
            if (!((ok >> j) & 1u)) continue;
            if (p[j] >= V) { if (part == 0) bad = 1; ok &= ~(1u << j); continue; }
            if ((p[j] >> kBucketShift) % split != part) ok &= ~(1u << j);   // another part's
        }
        if (slot != nullptr) {                               // eight look-ups in flight (unconditional, at a clamped page: a load
            constexpr int kSlotsAhead = 8;                   // under a condition waits inside its branch, one round trip per id)
            static_assert(kPerThread % kSlotsAhead == 0, "whole batches");
#pragma unroll
            for (int j0 = 0; j0 < kPerThread; j0 += kSlotsAhead) {
                uint32_t sl[kSlotsAhead];
#pragma unroll
                for (int u = 0; u < kSlotsAhead; ++u) sl[u] = slot[min((uint64_t)p[j0 + u], V - 1)];
#pragma unroll
                for (int u = 0; u < kSlotsAhead; ++u)
                    if (((ok >> (j0 + u)) & 1u) && sl[u] == kNone) { bad = 1; ok &= ~(1u << (j0 + u)); }
            }
        }
        MSCHED_TICK(kTickPrepare, 2);
        // Repeats are dropped through a table of pairs of entries: an id goes into the first entry of its
        // pair and moves what was there into the second.  Two popular ids that share a pair then both stay
        // visible - with one entry each would throw the other out every time, and a gather's most popular
        // pages would reach the merge once per repeat (twice the ids in the heaviest buckets, measured).
        // An id is only ever dropped on finding itself, and only a thread that keeps an id (or found it there)
        // puts it into the table, so whatever threads race here, one copy survives.
        // Both entries are first looked at with plain reads (lanes reading one address are served together), and
        // only an id that finds itself in neither goes on to the exchange: a gather's hottest page is a tenth of
        // all ids, and that many exchanges on one LDS address, which are served one by one, took longer than
        // everything else in this kernel together.  Ids go through in groups of kGroup, so that from the second
        // group on the popular ones are already there to be found.
        constexpr int kGroup = 4;
        static_assert(kPerThread % kGroup == 0, "whole groups");
#pragma unroll
        for (int j0 = 0; j0 < kPerThread; j0 += kGroup) {
            uint32_t first[kGroup], second[kGroup];
#pragma unroll
            for (int u = 0; u < kGroup; ++u) {
                const int j = j0 + u;
                const uint32_t h = (p[j] * 2654435761u) >> (32 - kBinSeenBits);
                first[u] = ((ok >> j) & 1u) ? seen[h] : kNone;
                second[u] = ((ok >> j) & 1u) ? seen[h ^ 1u] : kNone;
            }
#pragma unroll
            for (int u = 0; u < kGroup; ++u) {
                const int j = j0 + u;
                if (!((ok >> j) & 1u)) continue;
                if (first[u] == p[j] || second[u] == p[j]) { ok &= ~(1u << j); first[u] = kNone; continue; }
                first[u] = atomicExch(&seen[(p[j] * 2654435761u) >> (32 - kBinSeenBits)], p[j]);   // what was in the first entry
            }
#pragma unroll
            for (int u = 0; u < kGroup; ++u) {
                const int j = j0 + u;
                if (!((ok >> j) & 1u)) continue;
                if (first[u] == p[j]) ok &= ~(1u << j);
                else if (first[u] != kNone) seen[((p[j] * 2654435761u) >> (32 - kBinSeenBits)) ^ 1u] = first[u];
            }
        }
        MSCHED_TICK(kTickPrepare, 3);
#pragma unroll
        for (int j = 0; j < kPerThread; ++j)
            if ((ok >> j) & 1u) atomicAdd(&cnt[(p[j] >> kBucketShift) / split], 1u);
        MSCHED_TICK(kTickPrepare, 5);
    }
    __syncthreads();
    MSCHED_TICK(kTickPrepare, 6);
    // Buckets that ever received an id stay marked for the life of the context: the merge looks at no other.
    // (Marks are never taken back, so a bucket whose commands have all retired costs a look, not a wrong result.)
    for (uint32_t b = threadIdx.x; b < nb; b += blockDim.x)
        if (cnt[b] && !bucket_mark[part + b * split]) bucket_mark[part + b * split] = 1;
    MSCHED_TICK(kTickPrepare, 7);
    block_exclusive_scan(cnt, per_part + 1, wave_sums);    // cnt[b] = start of the part's bucket b, cnt[per_part] = total
    MSCHED_TICK(kTickPrepare, 8);
    uint32_t *block = pr.block + (size_t)part * prep_part_words(n_buckets, split, pr.n);
    if (threadIdx.x == 0) block[0] = bad;
    for (uint32_t b = threadIdx.x; b <= per_part; b += blockDim.x) block[1 + b] = cnt[b];
    __syncthreads();
    MSCHED_TICK(kTickPrepare, 9);
    uint32_t *out = block + per_part + 2;
    constexpr int kAhead = 4;                                 // positions asked for before the first is used
#pragma unroll
    for (int j0 = 0; j0 < kPerThread; j0 += kAhead) {
        uint32_t at[kAhead];
#pragma unroll
        for (int u = 0; u < kAhead; ++u)
            at[u] = ((ok >> (j0 + u)) & 1u) ? atomicAdd(&cnt[(p[j0 + u] >> kBucketShift) / split], 1u) : 0u;   // the starts double as write cursors
#pragma unroll
        for (int u = 0; u < kAhead; ++u)
            if ((ok >> (j0 + u)) & 1u) out[at[u]] = p[j0 + u];
    }
    MSCHED_TICK(kTickPrepare, 10);
}

// The ids of bucket b in one prepared piece: where they start and how many they are.
__device__ __forceinline__ const uint32_t *piece_segment(const ListSource &S, uint32_t b, uint32_t split, uint32_t per_part, uint32_t &len) {
    const uint32_t q = b % split, j = b / split;
    const uint32_t *part = S.block + (size_t)q * S.part_words;
    const uint32_t lo = part[1 + j], hi = part[2 + j];
    len = hi - lo;
    return part + per_part + 2 + lo;
}
// Did any part of the piece see an id that cannot be planned?
__device__ __forceinline__ bool piece_bad(const ListSource &S, uint32_t split) {
    bool bad = false;
    for (uint32_t q = 0; q < split; ++q) bad |= S.block[(size_t)q * S.part_words] != 0;
    return bad;
}

struct MergeArgs {
    const ListSource *src; uint32_t n_src, n_buckets, split;
    uint32_t *nu; uint32_t *flags; uint64_t V; uint32_t epoch_base;
    const uint32_t *bucket_mark;        // [n_buckets] has any prepared piece of this context ever put an id here?
};

// A workgroup per bucket.  The bucket's ids sit in one short segment per piece (tens of ids when a plan holds
// hundreds of pieces), so the pieces are dealt to the wavefronts, kMergePieces at a time: what a piece needs
// (segment address, length, next-use code) is the same for all lanes and is read once per piece, the lanes load
// the segments' ids side by side, and an id costs one load and one LDS atomic.  Whatever a segment holds beyond
// kMergeHead ids (a few long lists instead of many short ones) is shared out over the whole workgroup afterwards.
// (Measured and dropped: the per-piece values in scalar registers, a second workgroup for buckets with many ids,
// the marked buckets listed first in dispatch order - each slower than this on the planning-stress structure.)
constexpr int kMergePieces = 8;                     // segments in flight per wavefront
constexpr uint32_t kMergeHead = 4 * kWave;          // ids of a segment its wavefront takes itself

// The segments of one bucket, staged in LDS: for piece s its first id, its length and the value `code[s]` that goes
// into the bucket's table.  `put(id, code)` is the LDS atomic of the caller (the largest code or the smallest
// command wins, depending on what the table holds).
// kWidth: lanes that share a segment.  With 64 a wave-wide load takes a row of 64 ids from one segment; with 32 (16)
// it takes a row of 32 (16) ids from each of two (four) segments, which suits the short segments of plans with
// hundreds of pieces: a tile's merge is a chain of load round trips, and the fewer lanes a load leaves idle, the
// fewer round trips it takes.
template <int kPieces, int kRowsPerPass, int kWidth, class Put>
__device__ __forceinline__ void merge_segments(const uint32_t *const *first, const uint32_t *len, const uint32_t *code,
                                               uint32_t n_src, bool any_long, Put put) {
    static_assert(kWidth == 64 || kWidth == 32 || kWidth == 16, "lanes per segment");
    constexpr int kPerLoad = kWave / kWidth;                 // segments a wave-wide load reads from
    constexpr int kPerPass = kPieces * kPerLoad;             // segments a wavefront takes per pass
    const uint32_t lane = (uint32_t)lane_id(), wave = threadIdx.x / kWave, waves = blockDim.x / kWave;
    const uint32_t sub = lane / kWidth, off = lane % kWidth;
    for (uint32_t s0 = wave * kPerPass; s0 < n_src; s0 += waves * kPerPass) {
        const uint32_t *ptr[kPieces];
        uint32_t n[kPieces], e[kPieces];
#pragma unroll
        for (int j = 0; j < kPieces; ++j) {             // the same for the kWidth lanes of a group
            const uint32_t want = s0 + j * kPerLoad + sub;
            const uint32_t s = min(want, n_src - 1);
            n[j] = (want < n_src) ? min(len[s], kMergeHead) : 0u;
            e[j] = code[s];
            ptr[j] = first[s];
        }
        uint32_t n_max = 0;
#pragma unroll
        for (int j = 0; j < kPieces; ++j) n_max = max(n_max, n[j]);
        if (kPerLoad > 1) {                                  // the longest segment of any group decides the passes
#pragma unroll
            for (int d = kWidth; d < kWave; d <<= 1) n_max = max(n_max, (uint32_t)__shfl_xor((int)n_max, d, kWave));
        }
        // kRowsPerPass rows of kWidth ids from each of the segments per pass: every load of a pass is issued before its first atomic
        for (uint32_t r0 = 0; r0 < n_max; r0 += kRowsPerPass * kWidth) {
            uint32_t id[kRowsPerPass][kPieces];
#pragma unroll
            for (int q = 0; q < kRowsPerPass; ++q)
#pragma unroll
                for (int j = 0; j < kPieces; ++j)
                    id[q][j] = r0 + q * kWidth + off < n[j] ? ptr[j][r0 + q * kWidth + off] : kNone;
#pragma unroll
            for (int q = 0; q < kRowsPerPass; ++q)
#pragma unroll
                for (int j = 0; j < kPieces; ++j)
                    if (id[q][j] != kNone) put(id[q][j], e[j]);
        }
    }
    if (any_long) {
        for (uint32_t s = 0; s < n_src; ++s) {
            const uint32_t n = len[s];
            if (n <= kMergeHead) continue;
            const uint32_t *ptr = first[s];
            const uint32_t c = code[s];
            constexpr int kInFlight = 4;
            for (uint32_t i0 = kMergeHead + threadIdx.x; i0 < n; i0 += blockDim.x * kInFlight) {
                uint32_t id[kInFlight];
#pragma unroll
                for (int j = 0; j < kInFlight; ++j) id[j] = i0 + j * blockDim.x < n ? ptr[i0 + j * blockDim.x] : kNone;
#pragma unroll
                for (int j = 0; j < kInFlight; ++j)
                    if (id[j] != kNone) put(id[j], c);
            }
        }
    }
}

__global__ __launch_bounds__(kListThreads) void k_list_merge(MergeArgs a) {
    // buckets with ids tend to be neighbours (one table): the strided map spreads them over the dispatch order
    // and with it over the compute units
    const uint32_t b = chunk_of_block(blockIdx.x, gridDim.x);
    if (b != 0 && !a.bucket_mark[b]) return;                // bucket 0 always runs: it also reports unplannable ids
    __shared__ uint32_t tab[kBucketPages];
    extern __shared__ uint64_t merge_lds[];
    const uint32_t **first = reinterpret_cast<const uint32_t **>(merge_lds);   // [n_src] this bucket's first id in piece s
    uint32_t *len = reinterpret_cast<uint32_t *>(first + a.n_src);             // [n_src] ids of this bucket in piece s
    uint32_t *enc = len + a.n_src;                                              // [n_src] next-use code of the piece's command
    uint32_t longest = 0;
    const uint32_t split = a.split, per_part = prep_part_buckets(a.n_buckets, split);
    for (uint32_t s = threadIdx.x; s < a.n_src; s += blockDim.x) {
        const ListSource S = a.src[s];
        uint32_t n;
        first[s] = piece_segment(S, b, split, per_part, n);
        len[s] = n;
        enc[s] = kNuMask - S.g;
        longest = max(longest, n);
        if (b == 0 && piece_bad(S, split)) atomicOr(a.flags, kStatRange);   // the piece held an id that cannot be planned
    }
    for (uint32_t i = threadIdx.x; i < kBucketPages; i += blockDim.x) tab[i] = 0;
    const int any_ids = __syncthreads_or(longest != 0);
    const int any_long = __syncthreads_or(longest > kMergeHead);
    if (!any_ids) return;
    merge_segments<kMergePieces, 2, kWave>(first, len, enc, a.n_src, any_long != 0,
                   [&](uint32_t id, uint32_t code) { atomicMax(&tab[id & (kBucketPages - 1)], code); });   // never 0
    __syncthreads();
    const uint64_t p0 = (uint64_t)b << kBucketShift;
    const uint64_t p1 = min(a.V, p0 + kBucketPages);
    for (uint64_t p = p0 + threadIdx.x; p < p1; p += blockDim.x) {
        const uint32_t v = tab[p - p0];
        if (v) a.nu[p] = a.epoch_base | v;                   // this workgroup is the only writer of its slice
    }
}

// ------------------------------------------------------------------------------------------
// Class of a page: key in [0, K) = not resident with nu = key; key in [K, 2K) = resident with
// nu = key - K; K = G + 1 and class G stands for "never used in the timeline".  Pages that are
// neither resident nor used take part in nothing (key kNone).
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t classify(uint32_t frame, uint32_t enc, uint32_t epoch, uint32_t G, uint32_t painted) {
    const bool resident = frame != kNone;
    const uint32_t c = min(painted, ((enc >> kNuShift) == epoch) ? (kNuMask - (enc & kNuMask)) : G);
    if (!resident && c == G) return kNone;
    return resident ? (G + 1 + c) : c;
}

// Workgroups are dispatched in blockIdx order; chunks whose pages carry many different classes
// (sparse gathers) cost more than uniform ones and tend to be neighbours in the page table.  Striding
// the block -> chunk map spreads them over the whole launch instead of leaving them for its tail.
__device__ __forceinline__ uint32_t chunk_of_block(uint32_t block, uint32_t n_chunks) {
    constexpr uint32_t kStride = 61;                       // prime; the map is a bijection when it does not divide n
    // (On a 1280-chunk sweep strides 3, 7, 13, 61, 257, 509 and 641 are within 1 % of each other; 31, 101 and 1021
    // are 9 % slower: some strides line the heavy chunks up on few compute units.)
    if (n_chunks % kStride == 0) return block;
    return (uint32_t)(((uint64_t)block * kStride) % n_chunks);
}

struct SweepGeom {
    uint64_t V;
    uint32_t chunk_pages;     // pages per workgroup
    uint32_t steps;           // 64-page steps per wavefront per tile (<= kMaxSteps)
    uint32_t rounds;          // tiles per chunk; a tile is waves * steps * 64 consecutive pages
    uint32_t G, epoch;
    // next uses that come from range rules: a list of page ranges painted into LDS tile by tile
    const PageRange *ranges;
    uint32_t n_ranges;        // 0: nothing to paint
    uint32_t use_nu;          // 0: nu[] holds nothing for this plan and is not read
    const uint32_t *bucket_mark;   // non-null: nu[] holds something of this plan only in buckets marked here (all its
                                   // id lists came through prepared pieces); the sweep skips nu[] elsewhere
    const uint32_t *slot;     // page -> backing slot (or null): a wanted page without one is an error
    uint32_t *flags;
    uint16_t *key16;          // [V] class key of every page, written by the first sweep for the second
    uint32_t g_end0;          // commands of the first timeline entry: only their pages can be fetched
    uint32_t *emit_hint;      // [n_chunks] or null: what the first sweep saw in a chunk that the second may have to list
    uint32_t *paint_hint;     // [n_chunks] or null: plans left for which the chunk's tiles are painted in LDS without trying the queue first
                              // (2: a page that may be fetched, 1: a resident page the first entry does not use)
};
constexpr uint16_t kNoKey16 = 0xffff;                  // keys are below 2 * (MSCHED_MAX_TIMELINE_COMMANDS + 1) = 6144

// ------------------------------------------------------------------------------------------
// Painting.  A tile's next uses from range rules = for every page the smallest g among the ranges that
// cover it.  Each workgroup scans the plan's range list (a few KB, L2-resident), and
//   * a range that covers the whole tile only lowers one word, the tile's floor;
//   * a range that covers part of it is painted with LDS atomic minima: a few pages at once by the thread that
//     tested it, many pages queued and painted by all threads together.
// Nothing per page goes through memory: that is what the scatter path (k_expand) spends its time on.
// ------------------------------------------------------------------------------------------
// Where the painted tile starts in the first sweep's LDS: behind the histogram, on a 16-byte boundary.
__host__ __device__ inline uint32_t count_paint_offset(uint32_t n_keys) { return (n_keys + 3u) & ~3u; }
constexpr uint32_t kPaintQueue = 64;                      // partial ranges queued per batch; a tile meets a handful (LDS decides how
                                                          // many sweep workgroups a compute unit holds)
constexpr uint32_t kPaintSerial = 32;                     // ranges up to this many pages are painted by one thread
constexpr uint32_t kPaintHintPlans = 16;                  // plans a chunk paints in LDS straight away after its queue has overflowed
constexpr uint32_t kPaintByAll = 256;                     // queued ranges up to this many pages are painted by one wavefront, longer ones by all threads

struct PaintLds {
    uint32_t n_queued, floor;
    uint32_t lo[kPaintQueue], hi[kPaintQueue], g[kPaintQueue];
};

// The plan's ranges are tested in passes of kRangesPerThread per thread.  They come from the plan's own list; or,
// in the sweep for plans that brought none (kRuns), from the tasks' range mirrors: a wavefront serves one run of the
// timeline for the whole launch and takes rows of 64 of its entries, a lane working out its entry's position in the
// plan.  A range that repeats a region of a command still queued in front of its own is left out.
struct WaveRun {                      // what a wavefront knows of its run (the same in all lanes)
    const RangeRec *ring;
    uint32_t mask, first, count, cmd_first, g0, cursor, dedupe;
    uint32_t rank, waves;             // this wavefront among the `waves` that share the run
    uint32_t passes;
};
__device__ __forceinline__ WaveRun wave_run(const RangeRuns *runs) {
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    const RangeRun &run = runs->run[wave];                    // this wavefront's line of the table: one scalar load, tied to nothing
    WaveRun w;
    w.ring = run.ring;
    w.mask = run.mask; w.first = run.first; w.count = run.count; w.cmd_first = run.cmd_first;
    w.g0 = run.g0; w.cursor = run.cursor; w.dedupe = run.dedupe;
    w.rank = run.share & 0xffffu; w.waves = run.share >> 16;
    w.passes = run.passes;
    return w;
}
template <bool kRuns>
__device__ __forceinline__ bool pass_left(const SweepGeom &sg, const WaveRun &w, uint32_t pass) {   // the same answer in every thread
    if (!kRuns) return pass * blockDim.x * kRangesPerThread < sg.n_ranges;
    return pass < w.passes;
}
// body(R) for every range this thread is to test in pass `pass`.  From a list: range (pass * 4 + j) * blockDim + thread.
// From the mirrors: the wavefront's rows (pass * 4 + j) * waves + rank of its run, two loads in flight, both
// unconditional at an index clamped into the run (under a condition a load is compiled as a branch with the wait for
// it inside, and the two take a round trip each instead of one together; more at a time cost the sweep a workgroup
// per compute unit in registers).
constexpr uint32_t kRangesInFlight = 2;
static_assert(kRangesPerThread % kRangesInFlight == 0, "whole batches");
template <bool kRuns, class Body>
__device__ __forceinline__ void for_pass_ranges(const SweepGeom &sg, const WaveRun &w, uint32_t pass, Body body) {
    if (!kRuns) {
#pragma unroll
        for (uint32_t j = 0; j < kRangesPerThread; ++j) {
            const uint32_t r = (pass * kRangesPerThread + j) * blockDim.x + threadIdx.x;
            if (r >= sg.n_ranges) continue;
            body(sg.ranges[r]);
        }
        return;
    }
#pragma unroll
    for (uint32_t u0 = 0; u0 < kRangesPerThread; u0 += kRangesInFlight) {
        // nothing left for this wavefront (the same answer in all its lanes): no loads at all
        if (((pass * kRangesPerThread + u0) * w.waves + w.rank) * kRangeRow >= w.count) break;
        uint4 v[kRangesInFlight];
        bool live[kRangesInFlight];
#pragma unroll
        for (uint32_t u = 0; u < kRangesInFlight; ++u) {
            const uint32_t k = ((pass * kRangesPerThread + u0 + u) * w.waves + w.rank) * kRangeRow + (uint32_t)lane_id();
            live[u] = k < w.count;
            v[u] = reinterpret_cast<const uint4 *>(w.ring)[(w.first + min(k, w.count - 1)) & w.mask];
        }
#pragma unroll
        for (uint32_t u = 0; u < kRangesInFlight; ++u) {                         // RangeRec {lo, hi, back, cmd}
            if (w.dedupe && v[u].z != 0 && (int32_t)(v[u].w - v[u].z - w.cursor) >= 0) live[u] = false;
            if (live[u]) body(PageRange{v[u].x, v[u].y, w.g0 + (v[u].w - w.cmd_first), 0u});
        }
    }
}
static_assert(kRangeRow == (uint32_t)kWave, "a row of range entries is read by one wavefront");
static_assert(sizeof(RangeRec) == 16, "range entries are read as one 16-byte word");

template <bool kRuns>
__device__ __forceinline__ void paint_tile(const SweepGeom &sg, const WaveRun &runs, uint64_t t0, uint64_t t1, uint32_t *paint, PaintLds &q) {
    const uint32_t n = (t1 > t0) ? (uint32_t)(t1 - t0) : 0;
    for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) paint[i] = sg.G;
    if (threadIdx.x == 0) { q.n_queued = 0; q.floor = sg.G; }
    __syncthreads();
    for (uint32_t pass = 0; pass_left<kRuns>(sg, runs, pass); ++pass) {   // a thread tests kRangesPerThread ranges per pass (a pass costs three barriers)
        for_pass_ranges<kRuns>(sg, runs, pass, [&](const PageRange &R) {
            const uint64_t lo = max((uint64_t)R.lo, t0), hi = min((uint64_t)R.hi, t1);
            if (lo >= hi) return;
            if (lo == t0 && hi == t1) {
                atomicMin(&q.floor, R.g);
            } else if (hi - lo <= kPaintSerial) {             // a few pages: painted here and now, by the thread that found them
                for (uint32_t i = (uint32_t)(lo - t0); i < (uint32_t)(hi - t0); ++i) atomicMin(&paint[i], R.g);
            } else {                                          // many pages: queued (the lanes that are here together share one reservation)
                const uint64_t here = __ballot(true);
                const int leader = __ffsll((long long)here) - 1;
                uint32_t at = 0;
                if (lane_id() == leader) at = atomicAdd(&q.n_queued, (uint32_t)__popcll(here));
                at = __shfl(at, leader, kWave) + (uint32_t)__popcll(here & lanes_below());
                if (at < kPaintQueue) {
                    q.lo[at] = (uint32_t)(lo - t0); q.hi[at] = (uint32_t)(hi - t0); q.g[at] = R.g;
                } else {                                      // queue full: paint it here after all
                    for (uint32_t i = (uint32_t)(lo - t0); i < (uint32_t)(hi - t0); ++i) atomicMin(&paint[i], R.g);
                }
            }
        });
        __syncthreads();
        // the queue: a long range is painted by all threads together, the others by a wavefront each (a tile of many
        // ranges of some dozens of pages - the tiny schedule's one tile meets 40 - would otherwise walk them one by one).
        // Every wavefront reads the whole queue at once, an entry per lane, and hands the entries round from there: read
        // one by one from LDS, 40 entries were 3 us of round trips.
        static_assert(kPaintQueue <= (uint32_t)kWave, "an entry of the queue per lane");
        const uint32_t nq = min(q.n_queued, kPaintQueue);
        const uint32_t l = (uint32_t)lane_id();
        const uint32_t my_lo = l < nq ? q.lo[l] : 0u, my_hi = l < nq ? q.hi[l] : 0u, my_g = l < nq ? q.g[l] : 0u;
        for (uint64_t far = __ballot(my_hi - my_lo > kPaintByAll); far; far &= far - 1) {
            const int e = __ffsll((long long)far) - 1;
            const uint32_t lo = __shfl(my_lo, e, kWave), hi = __shfl(my_hi, e, kWave), g = __shfl(my_g, e, kWave);
            for (uint32_t i = lo + threadIdx.x; i < hi; i += blockDim.x) atomicMin(&paint[i], g);
        }
        for (uint32_t e = threadIdx.x / kWave; e < nq; e += blockDim.x / kWave) {
            const uint32_t lo = __shfl(my_lo, (int)e, kWave), hi = __shfl(my_hi, (int)e, kWave), g = __shfl(my_g, (int)e, kWave);
            if (hi - lo <= kPaintByAll)
                for (uint32_t i = lo + l; i < hi; i += kWave) atomicMin(&paint[i], g);
        }
        __syncthreads();
        if (threadIdx.x == 0) q.n_queued = 0;
        __syncthreads();
    }
}

// The cheap case of painting: a tile that only a few ranges reach into part of (dense ranges are long, a tile
// typically meets the end of one and the start of another).  The ranges are only tested and queued here, two
// barriers; every lane then applies the queue to its own pages in registers (sweep_tile), and nothing is painted
// in LDS.  Returns how many ranges were offered to the queue, the same number to every thread: above
// kPaintInRegisters the caller paints the tile in LDS instead (after a barrier of its own: paint_tile resets the
// queue).
// (Applying a queued range costs every lane about 30 instructions per eight pages: up to 32 ranges that is cheaper
// than painting the tile in LDS - three barriers and a pass over the tile - beyond it is not.  Measured with 8, 16, 32
// and 64: 32 is best on the tiny, the training and the decode schedule.)
#ifndef MSCHED_PAINT_IN_REGISTERS
#define MSCHED_PAINT_IN_REGISTERS 32
#endif
constexpr uint32_t kPaintInRegisters = MSCHED_PAINT_IN_REGISTERS;
// The queue is empty on entry (count_body resets it ahead of a barrier it needs anyway).
template <bool kRuns>
__device__ __forceinline__ uint32_t queue_ranges(const SweepGeom &sg, const WaveRun &runs, uint64_t t0, uint64_t t1, PaintLds &q) {
    for (uint32_t pass = 0; pass_left<kRuns>(sg, runs, pass); ++pass)
        for_pass_ranges<kRuns>(sg, runs, pass, [&](const PageRange &R) {
            const uint64_t lo = max((uint64_t)R.lo, t0), hi = min((uint64_t)R.hi, t1);
            if (lo >= hi) return;
            if (lo == t0 && hi == t1) {
                atomicMin(&q.floor, R.g);
            } else {
                const uint32_t at = atomicAdd(&q.n_queued, 1u);
                if (at < kPaintInRegisters) { q.lo[at] = (uint32_t)(lo - t0); q.hi[at] = (uint32_t)(hi - t0); q.g[at] = R.g; }
            }
        });
    __syncthreads();
    return q.n_queued;
}
static_assert(kPaintInRegisters <= kPaintQueue, "the queue holds what is applied from registers");

// A batch of a tile: kCountBatch x 64 consecutive pages of the wavefront's slice, lane l taking the kCountBatch
// consecutive pages from kCountBatch * l on.  Counting needs no page order, and eight consecutive pages make every
// access a 16-byte one: two loads each for page table and next use, two LDS reads for the painted tile, one
// store for the classes.  Eight pages at a time also keep the first sweep at half the registers of a whole
// 16-step slice, which doubles the workgroups a compute unit holds.
constexpr int kCountBatch = 8;
enum { kPaintNone = 0, kPaintLds = 1, kPaintQueued = 2 };   // where a tile's next uses from ranges are
struct Eight { uint4 lo, hi; };
__device__ __forceinline__ uint32_t eight_at(const Eight &e, int j) {
    const uint4 &h = j < 4 ? e.lo : e.hi;
    switch (j & 3) { case 0: return h.x; case 1: return h.y; case 2: return h.z; default: return h.w; }
}

// Count the batch's pages per key into one LDS histogram.  Runs of pages usually share a key (dense
// ranges, long stretches of resident pages nobody will use), so the first lane's key is settled for
// all its lanes with one add; whatever other keys the step holds go through per-lane LDS atomics.
__device__ __forceinline__ void count_batch(uint32_t *hist, const uint32_t (&key)[kCountBatch]) {
    const int lane = lane_id();
#pragma unroll
    for (int s = 0; s < kCountBatch; ++s) {
        const bool valid = key[s] != kNone;
        const uint64_t any = __ballot(valid);
        if (any) {
            const int leader = __ffsll((long long)any) - 1;
            const uint32_t k = __builtin_amdgcn_readlane(key[s], leader);
            const uint64_t same = __ballot(valid && key[s] == k);
            if (lane == leader) atomicAdd(&hist[k], (uint32_t)__popcll(same));
            if (valid && key[s] != k) atomicAdd(&hist[key[s]], 1u);
        }
    }
}

// Rank each page among the earlier pages of the same key inside this wavefront's slice (page
// order), counting into the wavefront's own LDS histogram.  Lanes with equal keys are grouped by
// ballot, so a step costs one pass per distinct key present, not one per page, and the loop itself
// touches no memory; one LDS atomic per distinct key then reserves the group's slots.
// On return key[s] holds (rank << 16) | key for a ranked page (ranks stay below the 1024 pages of a slice, keys below
// 2^16) and kNone for a page that takes no part: half the registers of two arrays.
__device__ __forceinline__ void rank_tile(const SweepGeom &sg, uint32_t *hist, uint32_t (&key)[kMaxSteps]) {
    const int lane = lane_id();
    const uint64_t below = lanes_below();
#pragma unroll
    for (int s = 0; s < kMaxSteps; ++s) {
        if ((uint32_t)s < sg.steps) {
            const bool valid = key[s] != kNone;
            int my_leader = lane;
            uint32_t my_rank = 0, group = 0;
            uint64_t todo = __ballot(valid);
            while (todo) {
                const int leader = __ffsll((long long)todo) - 1;
                const uint32_t k = __builtin_amdgcn_readlane(key[s], leader);
                const uint64_t same = __ballot(valid && key[s] == k);
                if (valid && key[s] == k) {
                    my_leader = leader;
                    my_rank = __popcll(same & below);
                    group = __popcll(same);
                }
                todo &= ~same;
            }
            uint32_t before = 0;
            if (valid && lane == my_leader) before = atomicAdd(&hist[key[s]], group);
            before = __shfl(before, my_leader, kWave);
            if (valid) key[s] |= (before + my_rank) << 16;
        }
    }
}

// First sweep: pages per key in one chunk -> one matrix row.  Counting needs no order, so all
// wavefronts of the workgroup add into one LDS histogram.
//
// kLists: the plan's id lists arrive as prepared pieces and a tile is exactly one bucket.  Then the workgroup merges
// its bucket's segments straight into the painted tile (the smallest command wins there, for ranges and lists
// alike) and nu[] is neither written nor read: the separate merge launch, 4 bytes written and 4 read per page of a
// bucket with ids, and one kernel boundary fall away.
struct TileLists {
    const ListSource *src; uint32_t n_src, n_buckets, split;
    const uint32_t *bucket_mark;        // [n_buckets] does any prepared piece hold an id of this bucket?
    const uint32_t *order;              // [n_chunks] the chunk of each workgroup (chunk_order_block)
};
// Shape of the merge inside the sweep, as build-time constants so that variants can be measured side by side:
// kFusedPieces loads in flight per wavefront and pass, each a row of kFusedWidth ids from each of 64 / kFusedWidth
// segments (a segment of one bucket and piece is a few dozen ids).  On the planning-stress schedule a tile's merge
// takes 10.8 us with rows of 64 ids, 9.6 with 32, 9.3 with 16; 8, 10 or 12 loads in flight instead of 6 are equal or
// slower, and so are two rows per segment and pass.
#ifndef MSCHED_FUSED_PIECES
#define MSCHED_FUSED_PIECES 6
#endif
#ifndef MSCHED_FUSED_WIDTH
#define MSCHED_FUSED_WIDTH 32
#endif
constexpr int kFusedPieces = MSCHED_FUSED_PIECES;
constexpr int kFusedWidth = MSCHED_FUSED_WIDTH;
constexpr int kFusedRows = 1;

template <bool kLists, bool kRuns = false>
__device__ __forceinline__ void count_body(const uint32_t *__restrict__ page_table, const uint32_t *__restrict__ nu,
                                           const SweepGeom &sg, uint32_t chunk, uint32_t *lds, uint32_t *row,
                                           uint32_t *group_row, uint32_t *slice_row, const TileLists *tl = nullptr,
                                           const RangeRuns *range_runs = nullptr) {
    const uint32_t n_keys = 2 * (sg.G + 1);
    const uint32_t waves = blockDim.x / kWave, wave = threadIdx.x / kWave;
    __shared__ PaintLds s_paint;
    MSCHED_TICK(kTickCount, 0);
    // asked for first, so that it is there when the tile's ranges are tested; read again behind every tile's sweep
    // (kept across that loop it would cost it a dozen registers)
    WaveRun runs{};
    if (kRuns) runs = wave_run(range_runs);
    for (uint32_t i = threadIdx.x; i < n_keys; i += blockDim.x) lds[i] = 0;
    if (threadIdx.x == 0) { s_paint.n_queued = 0; s_paint.floor = sg.G; }     // queue_ranges expects it empty
    if (threadIdx.x == 0 && sg.emit_hint != nullptr) sg.emit_hint[chunk] = 0;   // raised below, behind barriers
    // A chunk whose tiles met more partial ranges than are applied from registers is likely to meet as many in the next
    // plans (the timeline slides by a timeslice): it then paints them in LDS at once, instead of testing every range
    // twice - once to find out, once to paint.  A hint, not state: both ways give the same next uses, and it runs out
    // after kPaintHintPlans plans, when the queue is tried again.
    const uint32_t paint_hint = (sg.paint_hint != nullptr && sg.n_ranges) ? sg.paint_hint[chunk] : 0u;
    bool overflowed = false;
    __syncthreads();
    MSCHED_TICK(kTickCount, 1);
    const uint64_t p_begin = (uint64_t)chunk * sg.chunk_pages;
    const uint64_t p_end = min(sg.V, p_begin + sg.chunk_pages);
    const uint64_t tile_pages = (uint64_t)waves * sg.steps * kWave;
    uint32_t *paint = lds + count_paint_offset(n_keys);   // [tile_pages] when there are ranges to paint, 16-byte aligned
    const uint32_t lane = (uint32_t)lane_id();
    const uint4 none4 = {kNone, kNone, kNone, kNone}, zero4 = {0u, 0u, 0u, 0u};
    for (uint32_t round = 0; round < sg.rounds; ++round) {
        const uint64_t tile_begin = p_begin + round * tile_pages;
        const uint64_t tile_end = min(p_end, tile_begin + tile_pages);
        const uint64_t wave_begin = tile_begin + (uint64_t)wave * sg.steps * kWave;
        // The tile's pages, a batch at a time: classes from page table, nu[] (tile_nu) and the ranges (painted in
        // LDS, or still in the queue and applied here), written for the second sweep and counted.
        auto sweep_tile = [&](int tile_paint, bool tile_nu) {
            for (uint32_t s0 = 0; s0 < sg.steps; s0 += kCountBatch) {
                const uint32_t batch_pages = min((uint32_t)kCountBatch, sg.steps - s0) * kWave;
                const uint64_t first = wave_begin + (uint64_t)s0 * kWave + lane * kCountBatch;   // this lane's eight pages
                const bool live = lane * kCountBatch < batch_pages && first < p_end;
                // the arrays are padded, so a lane whose eight pages straddle the end of the table may load all eight
                Eight fr{none4, none4}, enc{zero4, zero4}, pt{zero4, zero4};
                if (live) {
                    const uint4 *src = reinterpret_cast<const uint4 *>(page_table + first);
                    fr = Eight{src[0], src[1]};
                    if (tile_nu) { const uint4 *e = reinterpret_cast<const uint4 *>(nu + first); enc = Eight{e[0], e[1]}; }
                    if (tile_paint == kPaintLds) { const uint4 *q = reinterpret_cast<const uint4 *>(paint + (first - tile_begin)); pt = Eight{q[0], q[1]}; }
                }
                uint32_t from_ranges[kCountBatch];
#pragma unroll
                for (int j = 0; j < kCountBatch; ++j) from_ranges[j] = tile_paint == kPaintLds ? eight_at(pt, j) : sg.G;
                if (tile_paint == kPaintQueued) {
                    // every lane applies every queued range to its eight pages: lane w fetches range w from LDS once,
                    // and the loop takes it from that lane's registers (a dependent LDS read per range and lane made
                    // a tile with dozens of short ranges spend most of its time here)
                    const uint32_t nq = __builtin_amdgcn_readfirstlane(s_paint.n_queued), at = (uint32_t)(first - tile_begin);   // uniform: a scalar loop
                    static_assert(kPaintInRegisters <= (uint32_t)kWave, "one queued range per lane");
                    const uint32_t q_lo = lane < nq ? s_paint.lo[lane] : 0u;
                    const uint32_t q_n = lane < nq ? s_paint.hi[lane] - q_lo : 0u;
                    const uint32_t q_g = lane < nq ? s_paint.g[lane] : 0u;
                    for (uint32_t w = 0; w < nq; ++w) {
                        const uint32_t lo = __builtin_amdgcn_readlane(q_lo, w), n = __builtin_amdgcn_readlane(q_n, w),
                                       g = __builtin_amdgcn_readlane(q_g, w);
#pragma unroll
                        for (int j = 0; j < kCountBatch; ++j)
                            if (at + j - lo < n) from_ranges[j] = min(from_ranges[j], g);
                    }
                }
                uint32_t key[kCountBatch];
#pragma unroll
                for (int j = 0; j < kCountBatch; ++j) {
                    const bool in = live && first + j < p_end;
                    const uint32_t painted = (in && tile_paint != kPaintNone) ? min(s_paint.floor, from_ranges[j]) : sg.G;
                    key[j] = in ? classify(eight_at(fr, j), eight_at(enc, j), sg.epoch, sg.G, painted) : kNone;
                }
                if (sg.slot != nullptr && sg.n_ranges) {      // a page a range wants must have a backing slot
#pragma unroll
                    for (int j = 0; j < kCountBatch; ++j)
                        if (key[j] < sg.G && sg.slot[first + j] == kNone) atomicOr(sg.flags, kStatRange);
                }
                // the second sweep reads the classes from here, 2 bytes a page
                if (live) {
                    uint32_t w[kCountBatch / 2];
#pragma unroll
                    for (int j = 0; j < kCountBatch; j += 2) {
                        const uint32_t a = key[j] == kNone ? (uint32_t)kNoKey16 : key[j];
                        const uint32_t b = key[j + 1] == kNone ? (uint32_t)kNoKey16 : key[j + 1];
                        w[j / 2] = a | (b << 16);
                    }
                    if (first + kCountBatch <= p_end) {
                        *reinterpret_cast<uint4 *>(sg.key16 + first) = uint4{w[0], w[1], w[2], w[3]};
                    } else {
#pragma unroll
                        for (int j = 0; j < kCountBatch; ++j)
                            if (first + j < p_end) sg.key16[first + j] = (uint16_t)(w[j / 2] >> (16 * (j & 1)));
                    }
                }
                count_batch(lds, key);
            }
        };
        // ranges of a tile without id lists: queued and applied from registers when they are few
        auto paint_ranges = [&]() -> int {
            if (!sg.n_ranges) return kPaintNone;
            // (a tile that is the whole table meets every range: with more ranges than can be applied from registers
            // there is no point in queueing them first)
            const bool all_partial = tile_begin == 0 && tile_end == sg.V && sg.n_ranges > kPaintInRegisters;
            if (!all_partial && paint_hint == 0) {
                if (queue_ranges<kRuns>(sg, runs, tile_begin, tile_end, s_paint) <= kPaintInRegisters) return kPaintQueued;
                overflowed = true;
            }
            __syncthreads();                                  // everybody has read the count
            paint_tile<kRuns>(sg, runs, tile_begin, tile_end, paint, s_paint);
            return kPaintLds;
        };
        if (kLists) {
            if (tile_begin < p_end) {
                const uint32_t b = (uint32_t)(tile_begin >> kBucketShift);      // the tile is this bucket
                if (b == 0) {                                 // its workgroup also reports ids that cannot be planned
                    for (uint32_t s = threadIdx.x; s < tl->n_src; s += blockDim.x)
                        if (piece_bad(tl->src[s], tl->split)) atomicOr(sg.flags, kStatRange);
                }
                // (Measured and dropped: asking for the page-table entries and the segment descriptions before
                // painting, so that their round trips overlap it - 5 us slower per plan.)
                if (!tl->bucket_mark[b]) {
                    const int how = paint_ranges();
                    MSCHED_TICK(kTickCount, 2);
                    sweep_tile(how, false);
                    MSCHED_TICK(kTickCount, 5);
                } else {
                    paint_tile<kRuns>(sg, runs, tile_begin, tile_end, paint, s_paint);
                    MSCHED_TICK(kTickCount, 2);
                    const uint32_t **first = reinterpret_cast<const uint32_t **>(paint + tile_pages);   // [kStagePieces]
                    uint32_t *len = reinterpret_cast<uint32_t *>(first + kStagePieces);
                    uint32_t *cmd = len + kStagePieces;
                    for (uint32_t s_base = 0; s_base < tl->n_src; s_base += kStagePieces) {
                        const uint32_t n_here = min(kStagePieces, tl->n_src - s_base);
                        uint32_t longest = 0;
                        for (uint32_t s = threadIdx.x; s < n_here; s += blockDim.x) {
                            const ListSource S = tl->src[s_base + s];
                            uint32_t n;
                            first[s] = piece_segment(S, b, tl->split, prep_part_buckets(tl->n_buckets, tl->split), n);
                            len[s] = n;
                            cmd[s] = S.g;
                            longest = max(longest, n);
                        }
                        const int any_long = __syncthreads_or(longest > kMergeHead);     // also the barrier behind the descriptions
                        MSCHED_TICK(kTickCount, 3);
                        merge_segments<kFusedPieces, kFusedRows, kFusedWidth>(first, len, cmd, n_here, any_long != 0,
                                       [&](uint32_t id, uint32_t g) { atomicMin(&paint[id & (kBucketPages - 1)], g); });
                        __syncthreads();                   // the next pieces overwrite the descriptions; the tile is read below
                    }
                    MSCHED_TICK(kTickCount, 4);
                    sweep_tile(kPaintLds, false);
                    MSCHED_TICK(kTickCount, 5);
                }
            }
        } else {
            const int tile_paint = paint_ranges();
            MSCHED_TICK(kTickCount, 2);
            // does any id list of this plan reach into this tile?  (the same answer for every thread)
            bool tile_nu = sg.use_nu != 0;
            if (tile_nu && sg.bucket_mark != nullptr && tile_begin < p_end) {
                uint32_t any = 0;
                for (uint64_t bk = tile_begin >> kBucketShift; bk <= ((tile_end - 1) >> kBucketShift); ++bk) any |= sg.bucket_mark[bk];
                tile_nu = any != 0;
            }
            sweep_tile(tile_paint, tile_nu);
            MSCHED_TICK(kTickCount, 5);
        }
        if (round + 1 < sg.rounds && (sg.n_ranges || kLists)) {
            if (kRuns) runs = wave_run(range_runs);
            __syncthreads();                              // the next tile repaints, and queues its ranges afresh
            if (threadIdx.x == 0) { s_paint.n_queued = 0; s_paint.floor = sg.G; }
            __syncthreads();
        }
    }
    __syncthreads();
    if (threadIdx.x == 0 && sg.paint_hint != nullptr && (overflowed || paint_hint != 0))
        sg.paint_hint[chunk] = overflowed ? kPaintHintPlans : paint_hint - 1;
    uint32_t hint = 0;
    for (uint32_t k = threadIdx.x; k < n_keys; k += blockDim.x) {
        const uint32_t v = lds[k];
        row[k] = v;
        if (group_row != nullptr && v) {                                // column sums by row group and by slice of it,
            atomicAdd(&group_row[k], v);                                // few keys are non-zero
            atomicAdd(&slice_row[k], v);
        }
        // first: a page that may be fetched, or a resident one whose next use lies in the last quarter of the timeline
        // (victims are taken from the far end); second: any other resident page the first entry does not use
        if (v) hint = max(hint, (k < sg.g_end0 || k >= 2 * sg.G + 1 - sg.G / 4) ? 2u : (k >= sg.G + 1 + sg.g_end0 ? 1u : 0u));
    }
    // Most chunks of a large table give the second sweep nothing to list, and those that do take it several times
    // longer: it starts with them (chunk_order_block in the cut kernel).  One atomic per wavefront that saw something.
    if (sg.emit_hint != nullptr) {
        const bool two = __ballot(hint == 2u) != 0, one = __ballot(hint == 1u) != 0;
        if (lane_id() == 0 && (two || one)) atomicMax(&sg.emit_hint[chunk], two ? 2u : 1u);
    }
    MSCHED_TICK(kTickCount, 6);
}

// Where a chunk's counts are added up for the column prefixes: the sums of its row group, and behind the
// kRowGroups rows of those the sums of its slice of the group (offsets_body).
__device__ __forceinline__ void sum_rows(uint32_t *partial, uint32_t chunk, uint32_t n_chunks, uint32_t n_keys,
                                         uint32_t *&group_row, uint32_t *&slice_row) {
    group_row = slice_row = nullptr;
    if (partial == nullptr) return;
    const uint32_t rows = (n_chunks + kRowGroups - 1) / kRowGroups;      // chunks per row group
    const uint32_t rows_sub = (rows + kOffsetSplit - 1) / kOffsetSplit;  // chunks per slice
    const uint32_t rg = chunk / rows, sub = (chunk - rg * rows) / rows_sub;
    group_row = partial + (size_t)rg * n_keys;
    slice_row = partial + (size_t)(kRowGroups + rg * kOffsetSplit + sub) * n_keys;
}

__global__ __launch_bounds__(kWave * kMaxWaves) void k_count(const uint32_t *__restrict__ page_table,
                                                              const uint32_t *__restrict__ nu, SweepGeom sg,
                                                              uint32_t *__restrict__ matrix,
                                                              uint32_t *__restrict__ partial) {
    extern __shared__ uint32_t lds[];
    const uint32_t chunk = chunk_of_block(blockIdx.x, gridDim.x), n_keys = 2 * (sg.G + 1);
    uint32_t *group_row, *slice_row;
    sum_rows(partial, chunk, gridDim.x, n_keys, group_row, slice_row);
    count_body<false>(page_table, nu, sg, chunk, lds, matrix + (size_t)chunk * n_keys, group_row, slice_row);
}

// The same sweep for plans that brought no range list: the ranges are read from the tasks' mirrors, run by run.
__global__ __launch_bounds__(kWave * kMaxWaves) void k_count_runs(const uint32_t *__restrict__ page_table,
                                                                   const uint32_t *__restrict__ nu, SweepGeom sg,
                                                                   uint32_t *__restrict__ matrix,
                                                                   uint32_t *__restrict__ partial, const RangeRuns rr) {
    extern __shared__ uint32_t lds[];
    const uint32_t chunk = chunk_of_block(blockIdx.x, gridDim.x), n_keys = 2 * (sg.G + 1);
    uint32_t *group_row, *slice_row;
    sum_rows(partial, chunk, gridDim.x, n_keys, group_row, slice_row);
    count_body<false, true>(page_table, nu, sg, chunk, lds, matrix + (size_t)chunk * n_keys, group_row, slice_row, nullptr, &rr);
}

// The first sweep with the id lists merged in (see count_body).  With 44 KiB of LDS a compute unit holds three
// of these workgroups, a tile with ids next to two without.  (Measured on the planning-stress structure: 1024
// threads with half the steps each, two workgroups per compute unit, 0.6 us slower per plan; 128 or 192 segments
// described at a time, which fits a fourth workgroup, 1.8 and 2.5 us slower.)
static_assert(kMaxWaves * kMaxSteps * kWave == (int)kBucketPages, "a full-size tile is one bucket");
constexpr int kFusedThreads = kWave * kMaxWaves;
// Registers: three of these workgroups (24 wavefronts, 6 per SIMD) share a compute unit, its LDS allows no more, so
// the kernel may use the 85 registers 6 wavefronts per SIMD leave each (at the 64 of 8 per SIMD it spilled).
#ifndef MSCHED_FUSED_MIN_WAVES
#define MSCHED_FUSED_MIN_WAVES 6
#endif
__global__ __launch_bounds__(kFusedThreads, MSCHED_FUSED_MIN_WAVES) void k_count_lists(const uint32_t *__restrict__ page_table, SweepGeom sg,
                                                              TileLists tl, uint32_t *__restrict__ matrix,
                                                              uint32_t *__restrict__ partial) {
    extern __shared__ uint32_t lds[];
    const uint32_t chunk = tl.order[blockIdx.x], n_keys = 2 * (sg.G + 1);
    uint32_t *group_row, *slice_row;
    sum_rows(partial, chunk, gridDim.x, n_keys, group_row, slice_row);
    count_body<true>(page_table, nullptr, sg, chunk, lds, matrix + (size_t)chunk * n_keys, group_row, slice_row, &tl);
}

// In-place exclusive scan of a[0..n) in LDS by the whole block (a multiple of 64 threads, at most
// 1024); returns the total to all threads.
__device__ uint32_t block_exclusive_scan(uint32_t *a, uint32_t n, uint32_t *wave_sums) {
    const uint32_t tid = threadIdx.x, nthreads = blockDim.x;
    const uint32_t per = (n + nthreads - 1) / nthreads;
    const uint32_t i0 = min(n, tid * per), i1 = min(n, i0 + per);
    uint32_t local = 0;
    for (uint32_t i = i0; i < i1; ++i) local += a[i];
    uint32_t incl = local;                                   // inclusive scan across the wavefront
    const int lane = lane_id();
    for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    const uint32_t wave = tid / kWave;
    __syncthreads();
    if (lane == kWave - 1) wave_sums[wave] = incl;
    __syncthreads();
    uint32_t wave_base = 0, total = 0;
    for (uint32_t w = 0; w < nthreads / kWave; ++w) {
        const uint32_t s = wave_sums[w];
        if (w < wave) wave_base += s;
        total += s;
    }
    uint32_t run = wave_base + incl - local;
    for (uint32_t i = i0; i < i1; ++i) { const uint32_t v = a[i]; a[i] = run; run += v; }
    __syncthreads();
    return total;
}

// Chunks whose buckets hold ids cost the first sweep several times what the others cost (they merge their
// segments first): dispatched first, the others fill in around them instead of waiting for the last of them.
// One workgroup of 256 threads; the marks are sticky, so an order made from marks a later preparation adds to
// is still a permutation - only less good.
__device__ void chunk_order_block(const ChunkOrder &o) {
    __shared__ uint32_t s_cnt[1024], s_wave[16];
    const uint32_t per = (o.n_chunks + blockDim.x - 1) / blockDim.x;      // at most kMaxChunks / 256 = 8
    const uint32_t c0 = min(o.n_chunks, threadIdx.x * per), c1 = min(o.n_chunks, c0 + per);
    uint32_t first = 0, second = 0;                                        // my chunks of the first and of the second rank
    for (uint32_t c = c0; c < c1; ++c) {
        uint32_t rank = 0;                                                 // the largest mark among the chunk's buckets
        const uint32_t b1 = min(o.n_buckets, (c + 1) * o.buckets_per_chunk);
        for (uint32_t b = c * o.buckets_per_chunk; b < b1; ++b) rank = max(rank, o.bucket_mark[b]);
        if (rank >= o.first_rank) first |= 1u << (c - c0);
        else if (rank != 0) second |= 1u << (c - c0);
    }
    s_cnt[threadIdx.x] = __popc(first);
    __syncthreads();
    const uint32_t n_first = block_exclusive_scan(s_cnt, blockDim.x, s_wave);
    uint32_t before_first = s_cnt[threadIdx.x];                            // chunks of the first rank below c
    __syncthreads();
    s_cnt[threadIdx.x] = __popc(second);
    __syncthreads();
    const uint32_t n_second = block_exclusive_scan(s_cnt, blockDim.x, s_wave);
    uint32_t before_second = s_cnt[threadIdx.x];
    for (uint32_t c = c0; c < c1; ++c) {
        if ((first >> (c - c0)) & 1u) o.order[before_first++] = c;
        else if ((second >> (c - c0)) & 1u) o.order[n_first + before_second++] = c;
        else o.order[n_first + n_second + (c - before_first - before_second)] = c;
    }
}
static_assert(kMaxChunks <= 256 * 32, "a thread of chunk_order_block keeps its chunks' marks in one word");

// Budget cut, counts, victim threshold (implicit in the offsets) and per-class output offsets.
//   D(k) = pages with nu < k; g_cut = largest k <= g_end0 with D(k) <= F            (cut)
//   fetch offsets: classes 0..g_cut-1 of non-resident pages, ascending
//   victim offsets: resident classes G (never used), G-1, ..., g_cut, in that order
// `groups` holds n_groups rows of per-key counts (row-group sums, or the matrix itself when it has
// few rows); they are replaced by their exclusive prefix over the rows.  One workgroup.
struct CutArgs {
    uint32_t *groups; uint32_t n_groups, G, g_end0, F;
    uint32_t *flags, *offsets;
    PlanHeader *hdr_dev, *hdr_host;
    uint32_t seq;                      // stamp for the host copy of the header
    uint32_t *need_host, *landed;      // early execution (both null when it is off)
    uint32_t in_place;                 // replace `groups` by their exclusive prefix over the rows (they are the matrix itself)
    uint32_t counts_in_lds;            // one workgroup does everything: the per-key totals are already in lds[0 .. n_keys)
};

// Exclusive scan of n values by ONE wavefront, no barrier: lane l owns the segment [l * per, (l + 1) * per) of
// the sequence value(0..n), sums it, the lane sums are scanned with shuffles, then put(i, exclusive prefix,
// value) is called for the lane's elements in order.  Returns the total to every lane.
template <class Value, class Put>
__device__ __forceinline__ uint32_t wave_exclusive_scan(uint32_t n, Value value, Put put) {
    const uint32_t lane = (uint32_t)lane_id();
    const uint32_t per = (n + kWave - 1) / kWave;
    const uint32_t i0 = min(n, lane * per), i1 = min(n, i0 + per);
    uint32_t local = 0;
    for (uint32_t i = i0; i < i1; ++i) local += value(i);
    uint32_t incl = local;
    for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t up = __shfl_up(incl, d, kWave);
        if ((int)lane >= d) incl += up;
    }
    const uint32_t total = __shfl(incl, kWave - 1, kWave);
    uint32_t run = incl - local;
    for (uint32_t i = i0; i < i1; ++i) { const uint32_t v = value(i); put(i, run, v); run += v; }
    return total;
}

// off_lds / hdr_lds (the single-workgroup kernel): the offsets and the header are also left in LDS, where the second
// sweep of the same workgroup finds them without a trip to memory.
__device__ void cut_body(const CutArgs &a, uint32_t *lds, uint32_t *off_lds = nullptr, PlanHeader *hdr_lds = nullptr) {
    const uint32_t G = a.G, K = G + 1, n_keys = 2 * K, g_end0 = a.g_end0, nthreads = blockDim.x;
    uint32_t *tot = lds;                 // [n_keys]
    __shared__ uint32_t s_cut, s_res, s_fetch;
    const uint32_t tid = threadIdx.x, wave = tid / kWave;
    if (tid == 0) { s_cut = 0; s_res = 0; s_fetch = 0; }
    // what the kernels before raised (every one of them is complete, or - in the single-workgroup kernel - behind a
    // barrier); asked for here so that the round trip is over by the time the header is written
    const uint32_t status_seen = tid == 0 ? __hip_atomic_load(a.flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
    MSCHED_TICK(kTickCut, 0);
    for (uint32_t key = tid; key < n_keys && !a.counts_in_lds; key += nthreads) {
        uint32_t v[kRowGroups];
#pragma unroll
        for (uint32_t rg = 0; rg < kRowGroups; ++rg) v[rg] = (rg < a.n_groups) ? a.groups[rg * n_keys + key] : 0;
        uint32_t run = 0;
#pragma unroll
        for (uint32_t rg = 0; rg < kRowGroups; ++rg) {
            if (rg < a.n_groups && a.in_place) a.groups[rg * n_keys + key] = run;
            run += v[rg];
        }
        tot[key] = run;
    }
    if (a.counts_in_lds)                                     // the one row's exclusive prefix over the rows: all zero
        for (uint32_t key = tid; key < n_keys; key += nthreads) a.groups[key] = 0;
    __syncthreads();
    MSCHED_TICK(kTickCut, 1);
    // The three scans below are short (K = G + 1 values): each is done by one wavefront without a barrier, the
    // cut by the first, resident pages counted by the others meanwhile; then fetch and victim offsets side by side.
    if (wave == 0) {
        // D(k) = pages first used before command k; the cut keeps the longest prefix of the first entry that fits
        uint32_t fit = 0;
        wave_exclusive_scan(g_end0, [&](uint32_t c) { return tot[c] + tot[K + c]; },
                            [&](uint32_t, uint32_t before, uint32_t v) { fit += (before + v <= a.F) ? 1u : 0u; });
        for (int d = kWave / 2; d > 0; d >>= 1) fit += __shfl_xor(fit, d, kWave);
        if (tid == 0) s_cut = fit;                          // D is monotone: the count of fitting k is the largest one
    }
    if (wave != 0 || nthreads == kWave) {
        uint32_t res = 0;
        const uint32_t first = nthreads == kWave ? tid : tid - kWave, step = nthreads == kWave ? kWave : nthreads - kWave;
        for (uint32_t c = first; c < K; c += step) res += tot[K + c];
        for (int d = kWave / 2; d > 0; d >>= 1) res += __shfl_xor(res, d, kWave);
        if (res && (tid % kWave) == 0) atomicAdd(&s_res, res);          // one add per wavefront, not per thread
    }
    __syncthreads();
    MSCHED_TICK(kTickCut, 2);
    const uint32_t g_cut = s_cut, n_res = s_res;
    const uint32_t last_wave = nthreads / kWave - 1;
    if (wave == 0) {
        // fetch offsets: classes 0 .. g_cut - 1 of the pages that are not resident, in order of use
        const uint32_t n_fetch = wave_exclusive_scan(K, [&](uint32_t c) { return c < g_cut ? tot[c] : 0u; },
                                                     [&](uint32_t c, uint32_t before, uint32_t v) {
                                                         const uint32_t at = (c < g_cut) ? before : kSkip;
                                                         a.offsets[c] = at;
                                                         if (off_lds) off_lds[c] = at;
                                                         // early execution: command c may start once the fetches of classes 0..c have landed
                                                         if (a.need_host && c < g_cut) a.need_host[c] = before + v;
                                                     });
        if (a.need_host) {                                  // need[] is in host memory: acknowledged ahead of the header's stamp
            __builtin_amdgcn_s_waitcnt(0);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        }
        if (tid == 0) s_fetch = n_fetch;
    }
    if (wave == last_wave) {
        // victim offsets, farthest next use first: resident classes G (never used), G - 1, ..., g_cut
        wave_exclusive_scan(K, [&](uint32_t j) { return (G - j >= g_cut) ? tot[K + (G - j)] : 0u; },
                            [&](uint32_t j, uint32_t before, uint32_t) {
                                const uint32_t at = (G - j >= g_cut) ? before : kSkip;
                                a.offsets[K + (G - j)] = at;
                                if (off_lds) off_lds[K + (G - j)] = at;
                            });
        if (a.landed && (tid % kWave) == 0) {   // entries landed, work units handed out, start of the migration kernel
            a.landed[0] = 0; a.landed[1] = 0; a.landed[2] = 0; a.landed[3] = 0;
        }
    }
    __syncthreads();
    MSCHED_TICK(kTickCut, 3);
    if (tid == 0) {
        uint32_t n_fetch = s_fetch;
        uint32_t status = status_seen;
        a.flags[0] = 0;                                     // clean for the next plan's expansion
        a.flags[1] = 0;                                     // work-unit counter of the migration that follows
        if (g_end0 > 0 && g_cut == 0) status |= kStatWset;
        if (status) n_fetch = 0;
        const uint32_t n_free = a.F - n_res;
        PlanHeader h;
        h.n_fetch = n_fetch;
        h.n_free_used = min(n_free, n_fetch);
        h.n_evict = n_fetch - h.n_free_used;
        h.g_cut = g_cut; h.n_resident = n_res; h.status = status; h.first_free = n_res; h.seq = 0;
        if (hdr_lds) *hdr_lds = h;
        *a.hdr_dev = h;
        // The host waits for the stamp, not for the end of the kernel: the counts (and need[]) go first, the stamp
        // once they have been acknowledged, so that whoever sees the stamp sees them.  The header and need[] lie in
        // pinned host memory, which no cache of the device holds: what orders the stores is the wait for their
        // acknowledgement, written out here (s_waitcnt 0; the workgroup-scope fence keeps the compiler from moving
        // stores across it).  A system-scope release would add a write-back of the L2 in front of the same wait -
        // 0.7 us after a sweep that has just written every page's class.
        *a.hdr_host = h;
        __builtin_amdgcn_s_waitcnt(0);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __hip_atomic_store(&a.hdr_host->seq, a.seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    MSCHED_TICK(kTickCut, 4);
}

__global__ __launch_bounds__(1024) void k_cut(CutArgs a) {
    extern __shared__ uint32_t lds[];
    cut_body(a, lds);
}

// starts[w][key] = pages of that key in chunks before w (exclusive prefix down each column of the count matrix),
// one thread per (key, row group, slice of the group): it starts from the sums of the row groups before its own
// and of the slices before its own in its group - the first sweep added both up - and walks its rows.
__device__ __forceinline__ void offsets_body(const uint32_t *__restrict__ matrix, uint32_t *__restrict__ starts,
                                             uint32_t n_chunks, uint32_t n_keys,
                                             const uint32_t *__restrict__ partial, uint32_t item, uint32_t g_end0) {
    // item = (key, row group, slice of the group): a compute unit fetches a few tens of GB/s at most, so the
    // matrix is spread over kOffsetSplit times as many workgroups as there are row groups x keys / block size.
    // (16 row groups of 8 slices measured best on a 1280-chunk sweep: 32 x 4 is 2 % slower, 64 groups 13 %.)
    const uint32_t key = item % n_keys, part = item / n_keys;
    const uint32_t rg = part / kOffsetSplit, sub = part % kOffsetSplit;
    if (rg >= kRowGroups) return;
    // pages that are not resident and first used after the incoming task's entry are never fetched, whatever the
    // cut turns out to be (g_cut <= g_end0): their columns get no offset and their start positions are never read
    if (key < n_keys / 2 && key >= g_end0) return;
    const uint32_t rows = (n_chunks + kRowGroups - 1) / kRowGroups;
    const uint32_t rows_sub = (rows + kOffsetSplit - 1) / kOffsetSplit;
    const uint32_t g0 = rg * rows, g1 = min(n_chunks, g0 + rows);       // the row group
    const uint32_t w0 = min(g1, g0 + sub * rows_sub), w1 = min(g1, w0 + rows_sub);
    // every load of the thread is asked for before the first is used: the sums in front of the slice, then its rows
    uint32_t front[kRowGroups + kOffsetSplit];
#pragma unroll
    for (uint32_t j = 0; j < kRowGroups; ++j) front[j] = j < rg ? partial[(size_t)j * n_keys + key] : 0u;
#pragma unroll
    for (uint32_t j = 0; j < kOffsetSplit; ++j)
        front[kRowGroups + j] = j < sub ? partial[(size_t)(kRowGroups + rg * kOffsetSplit + j) * n_keys + key] : 0u;
    constexpr uint32_t kRows = 16;
    uint32_t v[kRows];
#pragma unroll
    for (uint32_t j = 0; j < kRows; ++j) v[j] = (w0 + j < w1) ? matrix[(size_t)(w0 + j) * n_keys + key] : 0u;
    uint32_t run = 0;
#pragma unroll
    for (uint32_t j = 0; j < kRowGroups + kOffsetSplit; ++j) run += front[j];
    for (uint32_t w = w0; w < w1; w += kRows) {
        if (w != w0) {
#pragma unroll
            for (uint32_t j = 0; j < kRows; ++j) v[j] = (w + j < w1) ? matrix[(size_t)(w + j) * n_keys + key] : 0u;
        }
#pragma unroll
        for (uint32_t j = 0; j < kRows; ++j) {
            if (w + j < w1) starts[(size_t)(w + j) * n_keys + key] = run;
            run += v[j];
        }
    }
}

// The cut (one workgroup, three short scans) and the column prefixes (wide) need the same input,
// the per-key sums of the row groups, and nothing from each other: one launch, block 0 cuts.
__global__ __launch_bounds__(1024) void k_cut_offsets(CutArgs a, const uint32_t *__restrict__ matrix,
                                                        uint32_t *__restrict__ starts, uint32_t n_chunks, uint32_t n_keys,
                                                        ChunkOrder co) {
    extern __shared__ uint32_t lds[];
    if (blockIdx.x == 0) { cut_body(a, lds); return; }
    if (co.bucket_mark != nullptr && blockIdx.x == gridDim.x - 1) { chunk_order_block(co); return; }   // the extra workgroup
    offsets_body(matrix, starts, n_chunks, n_keys, a.groups, (blockIdx.x - 1) * blockDim.x + threadIdx.x, a.g_end0);
}

// Second sweep over one chunk: every listed page goes to its final position =
//   class offset + pages of the key in earlier chunks + in earlier tiles and wavefronts of this
//   chunk + rank inside the wavefront's slice.
struct EmitArgs {
    const uint32_t *page_table, *nu, *matrix, *offsets;
    const uint32_t *counts;           // the chunks' page counts per key, or null when only their start positions survive
    const PlanHeader *hdr;
    uint32_t *fetch_pages, *evict_pages, *evict_frames, *fetch_frames;
};

// LDS words emit_body needs: a histogram per wavefront, the running positions, and a 2 KiB staging line per wavefront.
__host__ __device__ inline size_t emit_lds_words(uint32_t waves, uint32_t n_keys) {
    return (((size_t)(waves + 1) * n_keys + 3) & ~(size_t)3) + (size_t)waves * (kMaxSteps * kWave / 2);   // staging lines 16-byte aligned
}

// The classes of a wavefront's slice (up to 1024 pages, 2 bytes each) are two 16-byte loads per lane; the lanes
// then exchange them through LDS, because lane l ranks pages l, 64 + l, ... (page order inside a step), not
// 16 l .. 16 l + 15.
constexpr uint32_t kLanePages = kMaxSteps * kWave / kWave;                    // consecutive pages a lane requests
static_assert(kLanePages == 16, "two uint4 of 16-bit classes per lane cover the slice");
struct SliceClasses { uint4 lo, hi; };
__device__ __forceinline__ SliceClasses request_slice(const SweepGeom &sg, uint32_t chunk, uint32_t round) {
    const uint32_t waves = blockDim.x / kWave, wave = threadIdx.x / kWave, lane = (uint32_t)lane_id();
    const uint64_t p_begin = (uint64_t)chunk * sg.chunk_pages;
    const uint64_t p_end = min(sg.V, p_begin + sg.chunk_pages);
    const uint64_t tile_pages = (uint64_t)waves * sg.steps * kWave;
    const uint4 none4 = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};     // kNoKey16 in every half
    const uint64_t first = p_begin + round * tile_pages + (uint64_t)wave * sg.steps * kWave + lane * kLanePages;
    // pages past the chunk's end are masked when the classes are read back; the array is padded past V
    if (lane * kLanePages >= sg.steps * kWave || first >= p_end) return SliceClasses{none4, none4};
    const uint4 *src = reinterpret_cast<const uint4 *>(sg.key16 + first);
    return SliceClasses{src[0], src[1]};
}

// kSingle (the single-workgroup kernel): the cut of the same workgroup has left the header in *hdr_lds and the
// offsets where the running positions go, and the first slice's classes (written by this workgroup's own first
// sweep) were asked for before the cut: nothing is read from memory before the pages are ranked.
template <bool kSingle = false>
__device__ __forceinline__ void emit_body(const EmitArgs &a, const SweepGeom &sg, uint32_t chunk, uint32_t *lds,
                                          const PlanHeader *hdr_lds = nullptr, const SliceClasses *first_slice = nullptr) {
    const uint32_t K = sg.G + 1, n_keys = 2 * K;
    const uint32_t waves = blockDim.x / kWave, wave = threadIdx.x / kWave;
    const int lane = lane_id();
    const uint64_t p_begin = (uint64_t)chunk * sg.chunk_pages;
    const uint64_t p_end = min(sg.V, p_begin + sg.chunk_pages);
    const uint64_t tile_pages = (uint64_t)waves * sg.steps * kWave;
    MSCHED_TICK(kTickEmit, 0);
    SliceClasses raw{};
    if (kSingle) raw = *first_slice;
    const PlanHeader *hdr = kSingle ? hdr_lds : a.hdr;
    const uint32_t n_fetch = hdr->n_fetch, n_evict = hdr->n_evict;
    const uint32_t n_free_used = hdr->n_free_used, first_free = hdr->first_free;
    if (n_fetch == 0) return;                             // same for every thread of the block
    uint32_t *base = lds + waves * n_keys;               // [n_keys] running output position per key
    uint32_t *hist = lds + wave * n_keys;
    uint16_t *stage = reinterpret_cast<uint16_t *>(lds + (((size_t)(waves + 1) * n_keys + 3) & ~(size_t)3)) + wave * (kMaxSteps * kWave);
    const uint32_t *row = a.matrix + (size_t)chunk * n_keys;
    // Most chunks of a large table hold no page that ends up in a list (a plan moves a few per cent of the pages):
    // the chunk's counts tell, before any page is looked at, whether some key with room left in its list occurs here.
    const uint32_t *cnt_row = a.counts ? a.counts + (size_t)chunk * n_keys : nullptr;
    bool live = cnt_row == nullptr;
    // The per-key tables first, two keys per thread in flight.  The slice's classes are asked for only once the
    // chunk is known to have work: three chunks in four of a large table have none, and loads come back in the
    // order they were issued, so a request for classes (memory) in front would hold up the tables (cache hits)
    // for nothing (measured: classes first 70.4 us per plan, between tables and their use 69.7, here 68.4).
    if (!kSingle) {
    constexpr int kKeysAhead = 2;
    uint32_t off_a[kKeysAhead], row_a[kKeysAhead], cnt_a[kKeysAhead];
#pragma unroll
    for (int j = 0; j < kKeysAhead; ++j) {
        // unconditional loads at a clamped key (under a condition each is compiled as a branch with its own wait
        // inside: six round trips in a row instead of one); the values of a key beyond the last are not used
        const uint32_t k = min(threadIdx.x + j * blockDim.x, n_keys - 1);
        off_a[j] = a.offsets[k];
        row_a[j] = row[k];
        cnt_a[j] = (cnt_row != nullptr ? cnt_row : row)[k];
    }
#pragma unroll
    for (int j = 0; j < kKeysAhead; ++j) {
        const uint32_t k = threadIdx.x + j * blockDim.x;
        if (k < n_keys) {
            const uint32_t at = (off_a[j] == kSkip) ? kSkip : off_a[j] + row_a[j];
            base[k] = at;
            if (cnt_row != nullptr && at < (k < K ? n_fetch : n_evict) && cnt_a[j] != 0) live = true;
        }
    }
    for (uint32_t k = threadIdx.x + kKeysAhead * blockDim.x; k < n_keys; k += blockDim.x) {
        const uint32_t off = a.offsets[k];
        const uint32_t at = (off == kSkip) ? kSkip : off + row[k];
        base[k] = at;
        if (cnt_row != nullptr && at < (k < K ? n_fetch : n_evict) && cnt_row[k] != 0) live = true;
    }
    MSCHED_TICK(kTickEmit, 1);
    if (!__syncthreads_or(live)) return;
    raw = request_slice(sg, chunk, 0);
    }
    for (uint32_t round = 0; round < sg.rounds; ++round) {
        if (round) raw = request_slice(sg, chunk, round);
        for (uint32_t i = threadIdx.x; i < waves * n_keys; i += blockDim.x) lds[i] = 0;
        reinterpret_cast<uint4 *>(stage + lane * kLanePages)[0] = raw.lo;      // read back by this wavefront only
        reinterpret_cast<uint4 *>(stage + lane * kLanePages)[1] = raw.hi;
        __syncthreads();
        const uint64_t tile_begin = p_begin + round * tile_pages;
        const uint64_t wave_begin = tile_begin + (uint64_t)wave * sg.steps * kWave;
        uint32_t key[kMaxSteps];
#pragma unroll
        for (int s = 0; s < kMaxSteps; ++s) {
            const uint64_t p = wave_begin + (uint64_t)s * kWave + lane;
            const uint16_t k16 = ((uint32_t)s < sg.steps && p < p_end) ? stage[s * kWave + lane] : kNoKey16;
            key[s] = k16 == kNoKey16 ? kNone : (uint32_t)k16;
        }
        // a key none of whose pages in this chunk can land inside its list is dropped here
#pragma unroll
        for (int s = 0; s < kMaxSteps; ++s)
            if (key[s] != kNone && base[key[s]] >= (key[s] < K ? n_fetch : n_evict)) key[s] = kNone;
        MSCHED_TICK(kTickEmit, 2);
        rank_tile(sg, hist, key);
        __syncthreads();
        MSCHED_TICK(kTickEmit, 3);
        // per key: each wavefront's start position in this tile; carry the running position on
        for (uint32_t k = threadIdx.x; k < n_keys; k += blockDim.x) {
            uint32_t run = base[k];
            for (uint32_t w = 0; w < waves; ++w) {
                const uint32_t t = lds[w * n_keys + k];
                lds[w * n_keys + k] = run;
                run += t;
            }
            base[k] = run;
        }
        __syncthreads();
        MSCHED_TICK(kTickEmit, 4);
#pragma unroll
        for (int s = 0; s < kMaxSteps; ++s) {
            if ((uint32_t)s < sg.steps && key[s] != kNone) {
                const uint32_t k = key[s] & 0xFFFFu;
                const uint32_t where = hist[k] + (key[s] >> 16);
                const uint32_t p = (uint32_t)(wave_begin + (uint64_t)s * kWave + lane);
                // Frames (Sec. 6.3: target i is populated into the space reclaimed from victim i): the first fetches
                // take the free frames, lowest first - frames are handed out in ascending order and only ever reused
                // through an eviction, so the free ones are [first_free, F) - and fetch n_free_used + j takes the
                // frame of victim j, which the workgroup that emits that victim writes into both lists.
                if (k < K) {
                    if (where < n_fetch) {
                        a.fetch_pages[where] = p;
                        if (where < n_free_used) a.fetch_frames[where] = first_free + where;
                    }
                } else if (where < n_evict) {
                    const uint32_t frame = a.page_table[p];
                    a.evict_pages[where] = p;
                    a.evict_frames[where] = frame;
                    a.fetch_frames[n_free_used + where] = frame;
                }
            }
        }
        __syncthreads();
        MSCHED_TICK(kTickEmit, 5);
    }
}

__global__ __launch_bounds__(kWave * kMaxWaves, 6) void k_emit(EmitArgs a, SweepGeom sg, uint32_t *__restrict__ partial,
                                                                uint32_t n_partial, const uint32_t *__restrict__ order) {
    extern __shared__ uint32_t lds[];
    // the row-group sums have been read by the cut: the next plan's first sweep adds into them again
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n_partial; i += gridDim.x * blockDim.x) partial[i] = 0;
    emit_body(a, sg, order != nullptr ? order[blockIdx.x] : chunk_of_block(blockIdx.x, gridDim.x), lds);
}

// Page tables small enough for one workgroup: count, cut, emit and frame assignment in one launch
// (planning such a table is bound by launch latency, not by bandwidth).
// A short range list rides in the kernel's arguments: the workgroup then reads it from the argument segment
// instead of from the pinned host memory the plan wrote it to - two passes over the list, each a round trip over
// the host link (9 of the 22 us of this kernel on the tiny round-robin schedule).
constexpr uint32_t kInlineRanges = 160;
struct InlineRanges { PageRange r[kInlineRanges]; };
__global__ __launch_bounds__(kWave * kMaxWaves) void k_tail(SweepGeom sg, CutArgs ca, EmitArgs ea, const InlineRanges inl) {
    extern __shared__ uint32_t lds[];
    __shared__ PageRange s_inl[kInlineRanges];
    if (sg.ranges == nullptr) {                           // the ranges came with the arguments: into LDS (count_body's first barrier comes before their use)
        for (uint32_t i = threadIdx.x; i < sg.n_ranges; i += blockDim.x) s_inl[i] = inl.r[i];
        sg.ranges = s_inl;
    }
    __shared__ PlanHeader s_hdr;
    count_body<false>(ea.page_table, ea.nu, sg, 0, lds, ca.groups, nullptr, nullptr);
    __syncthreads();
    const SliceClasses first_slice = request_slice(sg, 0, 0);   // the sweep has written them; on their way during the cut
    ca.counts_in_lds = 1;                                 // the only chunk's counts are where the sweep left them
    cut_body(ca, lds, lds + (blockDim.x / kWave) * 2 * (sg.G + 1), &s_hdr);   // the offsets: where emit_body keeps its running positions
    __syncthreads();
    emit_body<true>(ea, sg, 0, lds, &s_hdr, &first_slice);
}

__global__ __launch_bounds__(256) void k_zero(uint32_t *dst, uint64_t n) {
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < n; i += gridDim.x * (uint64_t)blockDim.x)
        dst[i] = 0;
}

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) return e_; } while (0)

hipError_t launch_nu_reset(msched_ctx *c) {
    (void)hipGetLastError();
    const uint32_t blocks = (uint32_t)std::max<uint64_t>(1, std::min<uint64_t>(4096, (c->V + 255) / 256));
    k_zero<<<blocks, 256, 0, c->stream>>>(c->nu, c->V);
    return hipGetLastError();
}

void plan_geometry(const msched_ctx *c, uint32_t G, PlanGeom &g) {
    g.G = G;
    g.n_keys = 2 * (G + 1);
    // (waves + 1) arrays of n_keys counters must fit in 48 KiB of LDS
    const uint32_t fit = (48u * 1024u) / (g.n_keys * 4u);
    g.waves = std::max<uint32_t>(1, std::min<uint32_t>(kMaxWaves, fit > 1 ? fit - 1 : 1));
    const uint64_t wave_pages = (uint64_t)g.waves * kWave;
    if (c->V <= kSingleChunkPages && !c->force_multi_kernel) {
        // one workgroup sweeps the whole table: count, cut, emit and frames fuse into one launch
        const uint64_t sub_steps = (c->V + wave_pages - 1) / wave_pages;
        g.steps = (uint32_t)std::min<uint64_t>(kMaxSteps, std::max<uint64_t>(1, sub_steps));
        g.rounds = (uint32_t)((sub_steps + g.steps - 1) / g.steps);
        g.chunk_pages = g.rounds * g.waves * g.steps * kWave;
        g.n_chunks = 1;
        g.single = true;
        return;
    }
    g.single = false;
    uint64_t per_chunk = (c->V + c->max_chunks - 1) / c->max_chunks;
    // Tables that still give every compute unit three workgroups of full-size tiles take those: fewer, longer
    // workgroups spend less of the sweep in its fixed per-workgroup parts (measured on 10 Mi pages: 1280
    // chunks of 8 Ki pages against 2048 of 5 Ki, 128 us against 139 us per plan).
    const uint64_t full_tile = wave_pages * kMaxSteps;
    if (per_chunk < full_tile && c->V / full_tile >= 768) per_chunk = full_tile;
    const uint64_t sub_steps = (per_chunk + wave_pages - 1) / wave_pages;
    if (sub_steps <= kMaxSteps) {
        g.steps = (uint32_t)std::max<uint64_t>(4, sub_steps);
        g.rounds = 1;
    } else {
        g.steps = kMaxSteps;
        g.rounds = (uint32_t)((sub_steps + kMaxSteps - 1) / kMaxSteps);
    }
    g.chunk_pages = g.rounds * g.waves * g.steps * kWave;
    g.n_chunks = (uint32_t)((c->V + g.chunk_pages - 1) / g.chunk_pages);
}

__global__ __launch_bounds__(256) void k_copy_ranges(const PageRange *__restrict__ src, PageRange *__restrict__ dst, uint32_t n) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) reinterpret_cast<uint4 *>(dst)[i] = reinterpret_cast<const uint4 *>(src)[i];
}

// The sweeps may ask for more dynamic LDS than the 64 KiB a kernel gets by default (counters + a painted tile).
hipError_t allow_large_lds() {
    static bool done[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= 64) return e == hipSuccess ? hipErrorInvalidDevice : e;
    if (done[dev]) return hipSuccess;
    const int bytes = 128 * 1024;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_count), hipFuncAttributeMaxDynamicSharedMemorySize, bytes)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_count_runs), hipFuncAttributeMaxDynamicSharedMemorySize, bytes)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_emit), hipFuncAttributeMaxDynamicSharedMemorySize, bytes)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_tail), hipFuncAttributeMaxDynamicSharedMemorySize, bytes)) != hipSuccess) return e;
    done[dev] = true;
    return hipSuccess;
}

hipError_t launch_list_prepare(msched_ctx *c, const ListPrep *table_dev, uint32_t n, uint32_t n_buckets, uint32_t split) {
    if (n == 0) return hipSuccess;
    (void)hipGetLastError();
    const size_t prep_lds = 4 * ((size_t)(1u << kBinSeenBits) + prep_part_buckets(n_buckets, split) + 1);
    k_list_prepare<<<n * split, kListThreads, prep_lds, c->stream>>>(table_dev, n_buckets, split, c->V, c->slot, c->bucket_mark);
    return hipGetLastError();
}

hipError_t launch_plan(msched_ctx *c, const PlanGeom &g) {
    (void)hipGetLastError();   // launches below are checked through the sticky error: start clean
    hipStream_t st = c->stream;
    const bool prof = c->profiling >= 2;
    // prepared id lists, painted ranges and full-size tiles (one bucket each): the first sweep merges the lists itself
    const bool fuse_lists = c->fuse_lists && c->has_list_rule && g.painted && g.list_prepared && g.n_list_sources &&
                            !g.single && g.waves == (uint32_t)kMaxWaves && g.steps == (uint32_t)kMaxSteps;
    if (c->profiling) CK(hipEventRecord(c->ev[0], st));
    {
        ExpandArgs a;
        a.cmd_ptrs = c->cmd_ptrs_dev; a.G = g.G; a.kernels = c->kernels_dev;
        a.nu = c->nu; a.slot = c->slot; a.flags = c->flags; a.V = c->V; a.page_shift = c->page_shift;
        a.n_split = c->expand_split ? c->expand_split : ((c->V > (1u << 20)) ? 8 : 1);
        a.epoch_base = c->epoch << kNuShift;
        // Records travel only when some kernel of this plan reads them (needs_records): a few expansion workgroups
        // read their record over the link themselves, many - and the id-list kernels - find a staged copy.  Painted
        // plans whose lists are prepared send only the two small tables (ranges, list pieces).
        const bool stage_records = g.needs_records &&
                                   ((uint64_t)g.G * c->max_rules * a.n_split > c->stage_threshold || g.live_list);
        const bool stage = stage_records || g.list_prepared || g.list_binned;
        a.cmds = stage_records ? c->cmd_dev : nullptr;
        const bool copy_ranges = g.n_ranges && !g.single && !g.resident;   // resident: the sweep reads the tasks' mirrors
        const uint32_t n_records = stage_records ? g.G : 0u;
        ChunkOrder co{nullptr, 0, 0, 0, 0, nullptr};
        if (fuse_lists) co = ChunkOrder{c->bucket_mark, g.n_buckets, g.n_chunks, g.rounds, 1, c->bucket_mark + kMaxBuckets};
        if (stage)
            k_stage<<<(std::max<uint32_t>(std::max(n_records * 8, (copy_ranges ? g.n_ranges : 0u) + g.n_list_sources), 1u) + 255) / 256 + (co.bucket_mark ? 1 : 0), 256, 0, st>>>(
                c->cmd_ptrs_dev, n_records, c->cmd_dev, c->list_bucket_fill, g.list_binned ? g.n_buckets * 8 : 0,
                c->ranges_host_dev, c->ranges_dev, copy_ranges ? g.n_ranges : 0, c->list_src_dev, c->list_src_stage,
                g.list_prepared ? g.n_list_sources : 0, co);
        else if (copy_ranges)
            k_copy_ranges<<<(g.n_ranges + 255) / 256, 256, 0, st>>>(c->ranges_host_dev, c->ranges_dev, g.n_ranges);
        // Id lists go first in three stream-ordered batches of growing size: the smallest g wins a page,
        // so once the first few commands have written the popular pages, the check in front of the
        // atomic turns every later touch of them into a plain (cached) load.
        if (g.list_prepared) {
            if (g.n_list_new) CK(launch_list_prepare(c, c->list_prep_dev, g.n_list_new, g.n_buckets, g.split));
            MergeArgs ma;
            ma.src = c->list_src_stage; ma.n_src = g.n_list_sources; ma.n_buckets = g.n_buckets; ma.split = g.split;
            ma.nu = c->nu; ma.flags = c->flags; ma.V = c->V; ma.epoch_base = a.epoch_base; ma.bucket_mark = c->bucket_mark;
            if (g.n_list_sources && !fuse_lists)
                k_list_merge<<<g.n_buckets, kListThreads, (size_t)g.n_list_sources * 16, st>>>(ma);
        } else if (g.list_binned) {
            ListArgs la;
            la.e = a; la.bucket_fill = c->list_bucket_fill; la.pairs = c->list_pairs;
            la.n_buckets = g.n_buckets; la.sub_cap = g.bucket_cap;
            const size_t bin_lds = 4 * ((size_t)(1u << kBinSeenBits) + kBinBlock + g.n_buckets);
            k_list_bin<<<g.G, kListThreads, bin_lds, st>>>(la, 1);
            k_list_reduce<<<g.n_buckets, kListThreads, 0, st>>>(la);
        } else if (g.live_list) {
            const uint32_t b0 = std::min<uint32_t>(g.G, c->list_b0), b1 = std::min<uint32_t>(g.G, c->list_b1);
            if (b0) k_expand_list<<<b0 * 16, kListThreads, 0, st>>>(a, 0, 16, kListSeenBits - 3);
            if (b1 > b0) k_expand_list<<<(b1 - b0) * 4, kListThreads, 0, st>>>(a, b0, 4, kListSeenBits - 2);
            if (g.G > b1) k_expand_list<<<g.G - b1, kListThreads, 0, st>>>(a, b1, 1, kListSeenBits);
        }
        // the ranges go after the lists: k_list_reduce merges into nu[] without atomics
        if (!g.painted) k_expand<<<dim3(g.G, c->max_rules, a.n_split), 256, 0, st>>>(a);
    }
    SweepGeom sg;
    sg.V = c->V; sg.chunk_pages = g.chunk_pages; sg.steps = g.steps; sg.rounds = g.rounds; sg.G = g.G;
    sg.epoch = c->epoch;
    sg.n_ranges = g.n_ranges; sg.use_nu = g.use_nu ? 1u : 0u;
    sg.bucket_mark = (g.painted && g.list_prepared) ? c->bucket_mark : nullptr;   // nothing but prepared lists wrote nu[] for this plan
    sg.slot = c->slot; sg.flags = c->flags; sg.key16 = c->key16;
    // the second sweep's order: only where the cut kernel has its wide part to carry the extra workgroup
    const bool order_emit = c->order_emit && !g.single && g.n_chunks > kRowGroups;
    sg.g_end0 = g.g_end0; sg.emit_hint = order_emit ? c->chunk_hint : nullptr;
    sg.paint_hint = g.single ? nullptr : c->chunk_hint + 2 * kMaxChunks;
    // one workgroup reads the range list where the host wrote it; many read a device copy, or the tasks' mirrors
    sg.ranges = g.single ? c->ranges_host_dev : g.resident ? nullptr : c->ranges_dev;
    const bool from_mirrors = g.resident && g.n_ranges;
    RangeRuns by_wave;                                       // the launch's copy of the table, a line per wavefront
    by_wave.n = 0;
    if (from_mirrors) {
        const RangeRuns &r = c->range_runs;
        const uint32_t W = g.waves;                          // r.n <= W <= kMaxRangeRuns
        uint32_t passes = 0;                                 // passes that cover the longest run with the wavefronts it gets
        for (uint32_t j = 0; j < r.n; ++j) {
            const uint32_t waves_j = (W - j + r.n - 1) / r.n, rows = (r.run[j].count + kRangeRow - 1) / kRangeRow;
            passes = std::max(passes, (rows + kRangesPerThread * waves_j - 1) / (kRangesPerThread * waves_j));
        }
        by_wave.n = r.n;
        for (uint32_t w = 0; w < W; ++w) {
            const uint32_t j = w % r.n;
            by_wave.run[w] = r.run[j];
            by_wave.run[w].share = (w / r.n) | ((W - j + r.n - 1) / r.n) << 16;
            by_wave.run[w].passes = passes;
        }
    }
    if (prof) CK(hipEventRecord(c->ev[1], st));
    const uint32_t threads = g.waves * kWave;
    const size_t paint_lds = g.n_ranges ? (size_t)g.waves * g.steps * kWave * 4 : 0;
    if (!c->no_large_lds) CK(allow_large_lds());
    const bool few_rows = g.n_chunks <= kRowGroups;          // the matrix rows are the row groups
    CutArgs ca;
    ca.groups = few_rows ? c->matrix : c->partial; ca.n_groups = few_rows ? g.n_chunks : kRowGroups;
    ca.G = g.G; ca.g_end0 = g.g_end0; ca.F = c->F; ca.flags = c->flags; ca.offsets = c->offsets;
    ca.hdr_dev = c->hdr_dev; ca.hdr_host = c->hdr_host; ca.seq = c->hdr_seq;
    ca.need_host = c->early ? c->need_host : nullptr; ca.landed = c->early ? c->landed : nullptr;
    ca.in_place = few_rows ? 1u : 0u;
    ca.counts_in_lds = 0;
    EmitArgs ea;
    ea.page_table = c->page_table; ea.nu = c->nu; ea.matrix = few_rows ? c->matrix : c->matrix + c->matrix_cap;   // chunk start positions
    ea.counts = few_rows ? nullptr : c->matrix;
    ea.offsets = c->offsets; ea.hdr = c->hdr_dev;
    ea.fetch_pages = c->fetch_pages; ea.evict_pages = c->evict_pages; ea.evict_frames = c->evict_frames;
    ea.fetch_frames = c->fetch_frames;
    const size_t cut_lds = (size_t)(g.n_keys + g.G + 1) * 4, emit_lds = emit_lds_words(g.waves, g.n_keys) * 4;
    if (g.single) {
        InlineRanges inl{};                                  // copied into the launch's argument buffer (entries beyond n_ranges are never read)
        if (g.n_ranges && g.n_ranges <= kInlineRanges) {
            memcpy(inl.r, c->ranges_host, sizeof(PageRange) * g.n_ranges);
            sg.ranges = nullptr;                             // the kernel points it at its argument
        }
        k_tail<<<1, threads, std::max(cut_lds, emit_lds + paint_lds + 16), st>>>(sg, ca, ea, inl);
        if (c->profiling) CK(hipEventRecord(c->ev[4], st));
        return hipGetLastError();
    }
    if (fuse_lists) {
        SweepGeom sc = sg;
        sc.steps = g.steps * g.waves / (kFusedThreads / kWave);       // the same tile, whatever the workgroup's width
        TileLists tl;
        tl.src = c->list_src_stage; tl.n_src = g.n_list_sources;
        tl.n_buckets = g.n_buckets; tl.split = g.split; tl.bucket_mark = c->bucket_mark;
        tl.order = c->bucket_mark + kMaxBuckets;
        const size_t lds = ((size_t)count_paint_offset(g.n_keys) + kBucketPages) * 4 + (size_t)kStagePieces * 16;
        k_count_lists<<<g.n_chunks, kFusedThreads, lds, st>>>(c->page_table, sc, tl, c->matrix, few_rows ? nullptr : c->partial);
    } else {
        const size_t count_lds = (size_t)count_paint_offset(g.n_keys) * 4 + paint_lds;
        if (from_mirrors)
            k_count_runs<<<g.n_chunks, threads, count_lds, st>>>(c->page_table, c->nu, sg, c->matrix, few_rows ? nullptr : c->partial, by_wave);
        else
            k_count<<<g.n_chunks, threads, count_lds, st>>>(c->page_table, c->nu, sg, c->matrix, few_rows ? nullptr : c->partial);
    }
    if (prof) CK(hipEventRecord(c->ev[2], st));
    const uint32_t cut_threads = std::min<uint32_t>(1024, std::max<uint32_t>(256, (g.n_keys + 63) / 64 * 64));   // a key per thread
    if (few_rows) {
        k_cut<<<1, cut_threads, cut_lds, st>>>(ca);
    } else {
        const uint32_t items = g.n_keys * kRowGroups * kOffsetSplit;
        ChunkOrder eo{nullptr, 0, 0, 0, 0, nullptr};
        if (order_emit) eo = ChunkOrder{c->chunk_hint, g.n_chunks, g.n_chunks, 1, 2, c->chunk_hint + kMaxChunks};
        k_cut_offsets<<<1 + (items + cut_threads - 1) / cut_threads + (order_emit ? 1 : 0), cut_threads, cut_lds, st>>>(
            ca, c->matrix, c->matrix + c->matrix_cap, g.n_chunks, g.n_keys, eo);
    }
    if (prof) CK(hipEventRecord(c->ev[3], st));
    k_emit<<<g.n_chunks, threads, emit_lds, st>>>(ea, sg, c->partial, few_rows ? 0 : kSumRows * g.n_keys,
                                                  order_emit ? c->chunk_hint + kMaxChunks : nullptr);
    if (c->profiling) CK(hipEventRecord(c->ev[4], st));
    return hipGetLastError();
}

}  // namespace msched
