// Planning kernels for gfx950: template expansion + next-use scatter, per-chunk class
// histograms over the page table, budget cut / victim threshold, and the ordered emission
// of the fetch and eviction lists.
//
// Method (paper: arXiv 2512.24637, Sec. 5.2 and Sec. 6.1-6.2): every page gets nu[p] = position
// of the first future command that touches it (kNone if the timeline never does).  The fetch
// list is the non-resident pages with nu < g_cut ordered by (nu, page id); the eviction list is
// the resident pages with nu >= g_cut ordered by (nu descending with kNone first, page id),
// truncated to what the fetches need.  Both orders are "class (a small integer) then page id",
// so the lists come out of one stable counting sort whose classes are the G+1 possible values of
// nu: a wavefront owns a contiguous chunk of the page table, counts its pages per class, a small
// kernel turns the chunk x class counts into absolute output offsets, and a second sweep writes
// each page straight to its final position.  No comparison sort, no per-command bitmaps.
#include <algorithm>

#include "msched_internal.h"

namespace msched {

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ uint64_t lanes_below() { return (1ull << lane_id()) - 1ull; }

// ------------------------------------------------------------------------------------------
// nu[] reset
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_fill(uint32_t *__restrict__ dst, uint64_t n, uint32_t v,
                                               uint32_t *__restrict__ flags) {
    const uint64_t tid = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    const uint64_t nthreads = gridDim.x * (uint64_t)blockDim.x;
    if (tid == 0) *flags = 0;
    const uint64_t n4 = n >> 2;
    uint4 *d4 = reinterpret_cast<uint4 *>(dst);
    const uint4 vv = make_uint4(v, v, v, v);
    for (uint64_t i = tid; i < n4; i += nthreads) d4[i] = vv;
    for (uint64_t i = (n4 << 2) + tid; i < n; i += nthreads) dst[i] = v;
}

// ------------------------------------------------------------------------------------------
// Template expansion + next-use scatter (Sec. 5.2 templates; Sec. 6.2 access order).
// One workgroup per (command g, rule r, split s).  A page's next use only ever decreases while
// this kernel runs, so a plain load that still shows a value <= g lets the atomic be skipped.
// ------------------------------------------------------------------------------------------
struct ExpandArgs {
    const CmdRec *const *cmd_ptrs; uint32_t G;
    const DevKernel *kernels;
    uint32_t *nu; const uint32_t *slot; uint32_t *flags;
    uint64_t V; uint32_t page_shift, n_split;
};

__device__ __forceinline__ void touch(const ExpandArgs &a, uint32_t p, uint32_t g) {
    if (a.slot != nullptr && a.slot[p] == kNone) { atomicOr(a.flags, kStatRange); return; }
    if (a.nu[p] > g) atomicMin(&a.nu[p], g);
}

__device__ __forceinline__ uint64_t formula(const uint64_t *args, uint64_t coeff, const uint8_t *idx, int n) {
    uint64_t v = coeff;
    for (int j = 0; j < n; ++j) v *= args[idx[j]];
    return v;
}

__global__ __launch_bounds__(256) void k_expand(ExpandArgs a) {
    const uint32_t g = blockIdx.x, r = blockIdx.y;
    __shared__ uint64_t s_rec[sizeof(CmdRec) / 8];
    // The record sits in pinned host memory: fetch it once per workgroup (two dependent reads).
    if (threadIdx.x < sizeof(CmdRec) / 8)
        s_rec[threadIdx.x] = reinterpret_cast<const uint64_t *>(a.cmd_ptrs[g])[threadIdx.x];
    __syncthreads();
    const CmdRec *rec = reinterpret_cast<const CmdRec *>(s_rec);
    const DevKernel &k = a.kernels[rec->kernel];
    if (r >= k.n_rules) return;
    const msched_rule q = k.rules[r];
    const uint32_t sh = a.page_shift;
    const uint64_t t0 = blockIdx.z * (uint64_t)blockDim.x + threadIdx.x;
    const uint64_t step = a.n_split * (uint64_t)blockDim.x;

    if (q.kind == MSCHED_RULE_LIST) {
        const uint32_t *ids = rec->ids;
        const uint32_t n = rec->n_ids;
        for (uint64_t i = t0; i < n; i += step) {
            const uint32_t p = ids[i];
            if (p >= a.V) { atomicOr(a.flags, kStatRange); continue; }
            touch(a, p, g);
        }
        return;
    }
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
                    for (uint64_t p = p0; p <= p1; ++p) touch(a, (uint32_t)p, g);
                }
            } else {                                        // few large chunks: threads across pages
                for (uint64_t j = 0; j < count; ++j) {
                    const uint64_t c0 = base + j * stride;
                    const uint64_t p0 = c0 >> sh, n = ((c0 + size - 1) >> sh) - p0 + 1;
                    for (uint64_t i = t0; i < n; i += step) touch(a, (uint32_t)(p0 + i), g);
                }
            }
            return;
        }
    }
    const uint64_t p0 = base >> sh, n = ((base + size - 1) >> sh) - p0 + 1;
    for (uint64_t i = t0; i < n; i += step) touch(a, (uint32_t)(p0 + i), g);
}

// ------------------------------------------------------------------------------------------
// Class of a page: key in [0, K) = not resident with nu = key; key in [K, 2K) = resident with
// nu = key - K; K = G + 1 and class G stands for "never used in the timeline".  Pages that are
// neither resident nor used take part in nothing.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ bool classify(uint32_t frame, uint32_t nu, uint32_t G, uint32_t &key) {
    const bool resident = frame != kNone;
    const uint32_t c = (nu == kNone) ? G : nu;
    key = resident ? (G + 1 + c) : c;
    return resident || c != G;
}

// Count pages per class in this wavefront's chunk; one matrix row per chunk.
__global__ __launch_bounds__(kWave) void k_count(const uint32_t *__restrict__ page_table,
                                                 const uint32_t *__restrict__ nu, uint64_t V,
                                                 uint32_t chunk_pages, uint32_t G,
                                                 uint32_t *__restrict__ matrix) {
    extern __shared__ uint32_t hist[];
    const uint32_t n_keys = 2 * (G + 1);
    const int lane = lane_id();
    for (uint32_t k = lane; k < n_keys; k += kWave) hist[k] = 0;
    const uint64_t p_begin = (uint64_t)blockIdx.x * chunk_pages;
    const uint64_t p_end = min(V, p_begin + chunk_pages);
    for (uint64_t p0 = p_begin; p0 < p_end; p0 += 4 * kWave) {
        uint32_t fr[4], nx[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t p = p0 + u * kWave + lane;
            const bool in = p < p_end;
            fr[u] = in ? page_table[p] : kNone;
            nx[u] = in ? nu[p] : kNone;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            uint32_t key;
            const bool valid = classify(fr[u], nx[u], G, key);
            uint64_t todo = __ballot(valid);
            while (todo) {
                const int leader = __ffsll((long long)todo) - 1;
                const uint32_t k = __builtin_amdgcn_readlane(key, leader);
                const uint64_t same = __ballot(valid && key == k);
                if (lane == leader) hist[k] += __popcll(same);
                todo &= ~same;
            }
        }
    }
    uint32_t *row = matrix + (size_t)blockIdx.x * n_keys;
    for (uint32_t k = lane; k < n_keys; k += kWave) row[k] = hist[k];
}

// Column sums of the count matrix, by row group.
__global__ __launch_bounds__(256) void k_colsum(const uint32_t *__restrict__ matrix, uint32_t n_chunks,
                                                uint32_t n_keys, uint32_t *__restrict__ partial) {
    const uint32_t key = blockIdx.x * 64 + threadIdx.x;
    const uint32_t rg = blockIdx.y * 4 + threadIdx.y;
    if (key >= n_keys) return;
    const uint32_t rows = (n_chunks + kRowGroups - 1) / kRowGroups;
    const uint32_t w0 = rg * rows, w1 = min(n_chunks, w0 + rows);
    uint32_t s = 0;
#pragma unroll 8
    for (uint32_t w = w0; w < w1; ++w) s += matrix[(size_t)w * n_keys + key];
    partial[rg * n_keys + key] = s;
}

// In-place exclusive scan of a[0..n) in LDS by a 1024-thread block; returns the total to all threads.
__device__ uint32_t block_exclusive_scan(uint32_t *a, uint32_t n, uint32_t *wave_sums) {
    const uint32_t tid = threadIdx.x;
    const uint32_t per = (n + 1023) / 1024;
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
    for (uint32_t w = 0; w < 1024 / kWave; ++w) {
        const uint32_t s = wave_sums[w];
        if (w < wave) wave_base += s;
        total += s;
    }
    uint32_t run = wave_base + incl - local;
    for (uint32_t i = i0; i < i1; ++i) { const uint32_t v = a[i]; a[i] = run; run += v; }
    __syncthreads();
    return total;
}

// Budget cut, counts, victim threshold (implicit in the offsets) and per-class output offsets.
//   D(k) = pages with nu < k; g_cut = largest k <= g_end0 with D(k) <= F            (cut)
//   fetch offsets: classes 0..g_cut-1 of non-resident pages, ascending
//   victim offsets: resident classes G (never used), G-1, ..., g_cut, in that order
__global__ __launch_bounds__(1024) void k_cut(uint32_t *__restrict__ partial, uint32_t G, uint32_t g_end0,
                                               uint32_t F, const uint32_t *__restrict__ flags,
                                               uint32_t *__restrict__ offsets, PlanHeader *__restrict__ hdr_dev,
                                               PlanHeader *__restrict__ hdr_host) {
    extern __shared__ uint32_t lds[];
    const uint32_t K = G + 1, n_keys = 2 * K;
    uint32_t *tot = lds;                 // [n_keys]
    uint32_t *sc = lds + n_keys;         // [K]
    __shared__ uint32_t wave_sums[1024 / kWave];
    __shared__ uint32_t s_cut, s_res;
    const uint32_t tid = threadIdx.x;
    if (tid == 0) { s_cut = 0; s_res = 0; }
    for (uint32_t key = tid; key < n_keys; key += 1024) {
        uint32_t run = 0;
        for (uint32_t rg = 0; rg < kRowGroups; ++rg) {
            const uint32_t v = partial[rg * n_keys + key];
            partial[rg * n_keys + key] = run;               // exclusive prefix over row groups
            run += v;
        }
        tot[key] = run;
    }
    __syncthreads();
    // cut
    for (uint32_t c = tid; c < K; c += 1024) sc[c] = (c < g_end0) ? tot[c] + tot[K + c] : 0;
    __syncthreads();
    const uint32_t d_all = block_exclusive_scan(sc, K, wave_sums);   // sc[k] = D(k) for k < K
    uint32_t fit = 0, res = 0;
    for (uint32_t k = 1 + tid; k <= g_end0; k += 1024) {
        const uint32_t d = (k < K) ? sc[k] : d_all;
        fit += (d <= F) ? 1u : 0u;
    }
    for (uint32_t c = tid; c < K; c += 1024) res += tot[K + c];
    if (fit) atomicAdd(&s_cut, fit);
    if (res) atomicAdd(&s_res, res);
    __syncthreads();
    const uint32_t g_cut = s_cut, n_res = s_res;
    // fetch offsets
    for (uint32_t c = tid; c < K; c += 1024) sc[c] = (c < g_cut) ? tot[c] : 0;
    __syncthreads();
    uint32_t n_fetch = block_exclusive_scan(sc, K, wave_sums);
    for (uint32_t c = tid; c < K; c += 1024) offsets[c] = (c < g_cut) ? sc[c] : kSkip;
    __syncthreads();
    // victim offsets, farthest next use first
    for (uint32_t j = tid; j < K; j += 1024) sc[j] = (G - j >= g_cut) ? tot[K + (G - j)] : 0;
    __syncthreads();
    block_exclusive_scan(sc, K, wave_sums);
    for (uint32_t c = tid; c < K; c += 1024) offsets[K + c] = (c >= g_cut) ? sc[G - c] : kSkip;
    if (tid == 0) {
        uint32_t status = *flags;
        if (g_end0 > 0 && g_cut == 0) status |= kStatWset;
        if (status) n_fetch = 0;
        const uint32_t n_free = F - n_res;
        PlanHeader h;
        h.n_fetch = n_fetch;
        h.n_free_used = min(n_free, n_fetch);
        h.n_evict = n_fetch - h.n_free_used;
        h.g_cut = g_cut; h.n_resident = n_res; h.status = status; h.first_free = n_res; h.pad = 0;
        *hdr_dev = h;
        *hdr_host = h;
    }
}

// Turn counts into absolute output positions: matrix[w][key] = offset[key] + pages of that class in
// chunks before w.
__global__ __launch_bounds__(256) void k_offsets(uint32_t *__restrict__ matrix, uint32_t n_chunks, uint32_t n_keys,
                                                 const uint32_t *__restrict__ partial,
                                                 const uint32_t *__restrict__ offsets,
                                                 const PlanHeader *__restrict__ hdr) {
    if (hdr->n_fetch == 0) return;
    const uint32_t key = blockIdx.x * 64 + threadIdx.x;
    const uint32_t rg = blockIdx.y * 4 + threadIdx.y;
    if (key >= n_keys) return;
    const uint32_t rows = (n_chunks + kRowGroups - 1) / kRowGroups;
    const uint32_t w0 = rg * rows, w1 = min(n_chunks, w0 + rows);
    uint32_t run = offsets[key] + partial[rg * n_keys + key];
#pragma unroll 8
    for (uint32_t w = w0; w < w1; ++w) {
        const size_t i = (size_t)w * n_keys + key;
        const uint32_t v = matrix[i];
        matrix[i] = run;
        run += v;
    }
}

// Second sweep: every listed page goes to its final position.
__global__ __launch_bounds__(kWave) void k_emit(const uint32_t *__restrict__ page_table,
                                                const uint32_t *__restrict__ nu, uint64_t V,
                                                uint32_t chunk_pages, uint32_t G,
                                                const uint32_t *__restrict__ matrix,
                                                const PlanHeader *__restrict__ hdr,
                                                uint32_t *__restrict__ fetch_pages,
                                                uint32_t *__restrict__ evict_pages,
                                                uint32_t *__restrict__ evict_frames) {
    extern __shared__ uint32_t pos[];
    const uint32_t n_fetch = hdr->n_fetch, n_evict = hdr->n_evict;
    if (n_fetch == 0) return;
    const uint32_t K = G + 1, n_keys = 2 * K;
    const int lane = lane_id();
    const uint32_t *row = matrix + (size_t)blockIdx.x * n_keys;
    for (uint32_t k = lane; k < n_keys; k += kWave) pos[k] = row[k];
    const uint64_t below = lanes_below();
    const uint64_t p_begin = (uint64_t)blockIdx.x * chunk_pages;
    const uint64_t p_end = min(V, p_begin + chunk_pages);
    for (uint64_t p0 = p_begin; p0 < p_end; p0 += 4 * kWave) {
        uint32_t fr[4], nx[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t p = p0 + u * kWave + lane;
            const bool in = p < p_end;
            fr[u] = in ? page_table[p] : kNone;
            nx[u] = in ? nu[p] : kNone;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            uint32_t key;
            const bool valid = classify(fr[u], nx[u], G, key);
            uint32_t where = kSkip;
            uint64_t todo = __ballot(valid);
            while (todo) {
                const int leader = __ffsll((long long)todo) - 1;
                const uint32_t k = __builtin_amdgcn_readlane(key, leader);
                const uint64_t same = __ballot(valid && key == k);
                uint32_t base = 0;
                if (lane == leader) { base = pos[k]; pos[k] = base + __popcll(same); }
                base = __builtin_amdgcn_readlane(base, leader);
                if (valid && key == k) where = base + __popcll(same & below);
                todo &= ~same;
            }
            const uint32_t p = (uint32_t)(p0 + u * kWave + lane);
            if (valid) {
                if (key < K) {
                    if (where < n_fetch) fetch_pages[where] = p;
                } else if (where < n_evict) {
                    evict_pages[where] = p;
                    evict_frames[where] = fr[u];
                }
            }
        }
    }
}

// Frame of every fetched page: free frames lowest first, then the victims' frames in eviction order
// (Sec. 6.3: target i is populated into the space reclaimed from victim i).  Frames are handed out
// in ascending order and only ever reused through an eviction, so the free ones are [first_free, F).
__global__ __launch_bounds__(256) void k_frames(const PlanHeader *__restrict__ hdr,
                                                const uint32_t *__restrict__ evict_frames,
                                                uint32_t *__restrict__ fetch_frames) {
    const uint32_t n = hdr->n_fetch, nfu = hdr->n_free_used, first = hdr->first_free;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x)
        fetch_frames[i] = (i < nfu) ? first + i : evict_frames[i - nfu];
}

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) return e_; } while (0)

hipError_t launch_plan(msched_ctx *c, const PlanGeom &g) {
    (void)hipGetLastError();   // launches below are checked through the sticky error: start clean
    hipStream_t st = c->stream;
    const bool prof = c->profiling != 0;
    if (prof) CK(hipEventRecord(c->ev[0], st));
    {
        const uint64_t n4 = (c->V + 3) / 4;
        const uint32_t blocks = (uint32_t)std::max<uint64_t>(1, std::min<uint64_t>(4096, (n4 + 255) / 256));
        k_fill<<<blocks, 256, 0, st>>>(c->nu, c->V, kNone, c->flags);
        ExpandArgs a;
        a.cmd_ptrs = c->cmd_ptrs_dev; a.G = g.G; a.kernels = c->kernels_dev;
        a.nu = c->nu; a.slot = c->slot; a.flags = c->flags; a.V = c->V; a.page_shift = c->page_shift;
        a.n_split = (c->V > (1u << 20)) ? 8 : 1;
        k_expand<<<dim3(g.G, c->max_rules, a.n_split), 256, 0, st>>>(a);
    }
    if (prof) CK(hipEventRecord(c->ev[1], st));
    const size_t row_bytes = (size_t)g.n_keys * sizeof(uint32_t);
    k_count<<<g.n_chunks, kWave, row_bytes, st>>>(c->page_table, c->nu, c->V, g.chunk_pages, g.G, c->matrix);
    if (prof) CK(hipEventRecord(c->ev[2], st));
    const dim3 cgrid((g.n_keys + 63) / 64, kRowGroups / 4), cblock(64, 4);
    k_colsum<<<cgrid, cblock, 0, st>>>(c->matrix, g.n_chunks, g.n_keys, c->partial);
    k_cut<<<1, 1024, (size_t)(g.n_keys + g.G + 1) * sizeof(uint32_t), st>>>(
        c->partial, g.G, g.g_end0, c->F, c->flags, c->offsets, c->hdr_dev, c->hdr_host);
    k_offsets<<<cgrid, cblock, 0, st>>>(c->matrix, g.n_chunks, g.n_keys, c->partial, c->offsets, c->hdr_dev);
    if (prof) CK(hipEventRecord(c->ev[3], st));
    k_emit<<<g.n_chunks, kWave, row_bytes, st>>>(c->page_table, c->nu, c->V, g.chunk_pages, g.G, c->matrix,
                                                 c->hdr_dev, c->fetch_pages, c->evict_pages, c->evict_frames);
    const uint32_t fblocks = (uint32_t)std::min<uint64_t>(2048, ((uint64_t)c->F + 255) / 256);
    k_frames<<<fblocks, 256, 0, st>>>(c->hdr_dev, c->evict_frames, c->fetch_frames);
    if (prof) CK(hipEventRecord(c->ev[4], st));
    return hipGetLastError();
}

}  // namespace msched
