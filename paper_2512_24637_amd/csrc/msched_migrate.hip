// Migration copy engine, page-table update and page-table query for gfx950.
//
// Paper (arXiv 2512.24637, Sec. 6.3): swapping a page is unmap victim -> copy victim out ->
// copy target in -> map target, and MSched pipelines the two copies of successive pages on two
// DMA engines so both directions of the host link are busy.  Here the compute units do the
// copy: fetch i and the victim whose frame it reuses are handled by the same lanes, which read
// the victim's bytes from the HBM frame, post them to pinned host memory, read the target's bytes
// from pinned host memory and store them into the same frame.  The frame dependency is therefore
// thread-local (a lane's own load-then-store to one address) and needs no signalling, and every
// workgroup keeps host-bound writes and host reads in flight at once, which is what fills the
// full-duplex link.  Lists are processed in plan order, i.e. in order of first use.
#include <algorithm>
#include <cstdlib>

#include "msched_internal.h"

namespace msched {

struct MigrateArgs {
    uint8_t *pool, *host;
    const uint32_t *slot;
    const uint32_t *evict_pages, *fetch_pages, *fetch_frames;
    uint32_t *page_table, *frame_owner;
    uint32_t n_fetch, n_free_used, page_shift;
    uint32_t chunk_shift;          // log2(bytes one workgroup moves per unit)
    uint32_t hints;                // bit 0: plain (not non-temporal) host stores, bit 1: plain host loads
    uint64_t n_units;              // n_fetch << (page_shift - chunk_shift)
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kLanesBytes = 16;    // one dwordx4 per lane
constexpr int kBatch = 4;          // independent 16-byte transfers in flight per lane and direction

__global__ __launch_bounds__(256) void k_migrate(MigrateArgs a) {
    const uint32_t cpp_shift = a.page_shift - a.chunk_shift;
    const uint32_t chunk_bytes = 1u << a.chunk_shift;
    const uint32_t sweep = 256 * kLanesBytes;                  // bytes one pass of the workgroup covers
    for (uint64_t unit = blockIdx.x; unit < a.n_units; unit += gridDim.x) {
        const uint32_t i = (uint32_t)(unit >> cpp_shift);
        const uint64_t chunk_off = (unit & ((1ull << cpp_shift) - 1)) << a.chunk_shift;
        const uint32_t frame = a.fetch_frames[i];
        const uint32_t fpage = a.fetch_pages[i];
        const bool swap = i >= a.n_free_used;                  // this fetch reuses a victim's frame
        const uint32_t vpage = swap ? a.evict_pages[i - a.n_free_used] : 0;
        const uint64_t fslot = a.slot ? a.slot[fpage] : fpage;
        const uint64_t vslot = swap ? (a.slot ? a.slot[vpage] : vpage) : 0;
        uint8_t *fr = a.pool + ((uint64_t)frame << a.page_shift) + chunk_off;
        const uint8_t *src = a.host + (fslot << a.page_shift) + chunk_off;
        uint8_t *dst = a.host + (vslot << a.page_shift) + chunk_off;
        for (uint32_t off0 = threadIdx.x * kLanesBytes; off0 < chunk_bytes; off0 += sweep * kBatch) {
            u32x4 out[kBatch], in[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const uint32_t off = off0 + u * sweep;
                if (off < chunk_bytes)
                    in[u] = (a.hints & 2) ? *reinterpret_cast<const u32x4 *>(src + off)
                                          : __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + off));
            }
            if (swap) {
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const uint32_t off = off0 + u * sweep;
                    if (off < chunk_bytes) out[u] = *reinterpret_cast<const u32x4 *>(fr + off);
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const uint32_t off = off0 + u * sweep;
                    if (off < chunk_bytes) {
                        if (a.hints & 1) *reinterpret_cast<u32x4 *>(dst + off) = out[u];
                        else __builtin_nontemporal_store(out[u], reinterpret_cast<u32x4 *>(dst + off));
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const uint32_t off = off0 + u * sweep;
                if (off < chunk_bytes) *reinterpret_cast<u32x4 *>(fr + off) = in[u];
            }
        }
        if (chunk_off == 0 && threadIdx.x == 0) {              // unmap the victim, map the target
            if (swap) a.page_table[vpage] = kNone;
            a.page_table[fpage] = frame;
            a.frame_owner[frame] = fpage;
        }
    }
}

__global__ __launch_bounds__(256) void k_fill_u32(uint32_t *dst, uint64_t n, uint32_t v) {
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < n; i += gridDim.x * (uint64_t)blockDim.x)
        dst[i] = v;
}

__global__ __launch_bounds__(256) void k_query(const uint32_t *__restrict__ page_table, const uint32_t *__restrict__ ids,
                                               uint32_t n, uint32_t *__restrict__ out) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = page_table[ids[i]];
}

hipError_t launch_init_tables(msched_ctx *c) {
    (void)hipGetLastError();
    const uint32_t bv = (uint32_t)std::min<uint64_t>(4096, (c->V + 255) / 256);
    const uint32_t bf = (uint32_t)std::min<uint64_t>(4096, ((uint64_t)c->F + 255) / 256);
    k_fill_u32<<<bv, 256, 0, c->stream>>>(c->page_table, c->V, kNone);
    k_fill_u32<<<bf, 256, 0, c->stream>>>(c->frame_owner, c->F, kNone);
    return hipGetLastError();
}

hipError_t launch_query(msched_ctx *c, const uint32_t *ids_dev, uint32_t n, uint32_t *out_dev) {
    if (n == 0) return hipSuccess;
    (void)hipGetLastError();
    k_query<<<(n + 255) / 256, 256, 0, c->stream>>>(c->page_table, ids_dev, n, out_dev);
    return hipGetLastError();
}

hipError_t launch_migrate(msched_ctx *c, const PlanHeader &h) {
    if (h.n_fetch == 0) return hipSuccess;
    (void)hipGetLastError();
    MigrateArgs a;
    a.pool = static_cast<uint8_t *>(c->cfg.hbm_pool);
    a.host = static_cast<uint8_t *>(c->host_dev);
    a.slot = c->slot;
    a.evict_pages = c->evict_pages; a.fetch_pages = c->fetch_pages; a.fetch_frames = c->fetch_frames;
    a.page_table = c->page_table; a.frame_owner = c->frame_owner;
    a.n_fetch = h.n_fetch; a.n_free_used = h.n_free_used; a.page_shift = c->page_shift;
    a.chunk_shift = std::min<uint32_t>(c->page_shift, c->migrate_chunk_shift);
    a.hints = c->migrate_hints;
    a.n_units = (uint64_t)h.n_fetch << (a.page_shift - a.chunk_shift);
    const uint64_t blocks = std::min<uint64_t>(a.n_units, c->migrate_max_blocks);
    k_migrate<<<(uint32_t)blocks, 256, 0, c->stream>>>(a);
    return hipGetLastError();
}

}  // namespace msched
