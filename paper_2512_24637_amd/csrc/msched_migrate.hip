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
#include <atomic>
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
    // early execution (all null / 0 when it is off)
    uint32_t *page_done, *chunks_done, *landed;
    uint32_t early_tag;
    uint32_t *ticket;              // work-unit counter (zero at launch) when units are handed out in order
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kLanesBytes = 16;    // one dwordx4 per lane
constexpr int kBatch = 4;          // independent 16-byte transfers in flight per lane and direction

// kEarly: early execution.  Entries are declared complete one by one while the kernel runs, so a frame's bytes
// must be in memory, not dirty in this XCD's L2, when that happens.  A release fence at device scope would
// write the whole L2 back each time (measured: a third of the copy rate lost); instead the frame is written
// with write-through stores (system-scope relaxed atomic stores of 8 bytes), and waiting for the stores'
// acknowledgements is then all the release that is needed.
template <bool kEarly, bool kTicket>
__global__ __launch_bounds__(256) void k_migrate(MigrateArgs a) {
    const uint32_t cpp_shift = a.page_shift - a.chunk_shift;
    const uint32_t chunk_bytes = 1u << a.chunk_shift;
    const uint32_t sweep = 256 * kLanesBytes;                  // bytes one pass of the workgroup covers
    __shared__ uint32_t s_unit;
    if (kEarly && blockIdx.x == 0 && threadIdx.x == 0)         // when this migration began, for the gates' reports
        __hip_atomic_store(reinterpret_cast<uint64_t *>(a.landed + 2), (uint64_t)wall_clock64(), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (uint64_t unit = blockIdx.x;; unit += gridDim.x) {
        if (kTicket) {
            // Units are handed out in list order from a counter, not dealt round-robin: workgroups
            // get uneven shares of the host link, and a fixed deal would let the slowest one hold `landed` back
            // while the others run far ahead.
            __syncthreads();
            if (threadIdx.x == 0) s_unit = __hip_atomic_fetch_add(a.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            unit = s_unit;
        }
        if (unit >= a.n_units) break;
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
                if (off < chunk_bytes) {
                    if (kEarly) {
                        uint64_t *q = reinterpret_cast<uint64_t *>(fr + off);
                        __hip_atomic_store(q, (uint64_t)in[u].x | (uint64_t)in[u].y << 32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                        __hip_atomic_store(q + 1, (uint64_t)in[u].z | (uint64_t)in[u].w << 32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                    } else {
                        *reinterpret_cast<u32x4 *>(fr + off) = in[u];
                    }
                }
            }
        }
        if (!kEarly) {
            // Unmap the victim, map the target: the last of the four steps of a swap (Sec. 6.3), so it comes after
            // the page's last chunk.  A page of one chunk is mapped by the workgroup that copied it; the chunks of a
            // larger page are counted, and the workgroup whose chunk completes the count maps it.  (Readers of the
            // table are ordered behind the whole kernel by the stream; the order inside it is the paper's.)
            bool complete = true;
            if (cpp_shift) {
                __builtin_amdgcn_s_waitcnt(0);                 // this lane's loads and stores have been acknowledged
                __syncthreads();
                if (threadIdx.x == 0) {
                    complete = __hip_atomic_fetch_add(&a.chunks_done[i], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1 == (1u << cpp_shift);
                    if (complete) __hip_atomic_store(&a.chunks_done[i], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next migration
                }
            }
            if (complete && threadIdx.x == 0) {
                if (swap) a.page_table[vpage] = kNone;
                a.page_table[fpage] = frame;
                a.frame_owner[frame] = fpage;
            }
            continue;
        }
        // Early execution: declare the entry complete and move `landed` over every leading complete entry.
        // All atomics below are relaxed and write through to the device's coherence point; program order between
        // them is kept by waiting for each to be acknowledged.  The wait is written out (s_waitcnt 0: every
        // outstanding load, write-through frame store and non-temporal host store of this lane has been
        // acknowledged) and does not rest on how the compiler lowers a workgroup-scope fence, which it may lower
        // to nothing when a workgroup cannot span compute units.
        __builtin_amdgcn_s_waitcnt(0);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (threadIdx.x == 0) {
            bool complete = true;
            if (cpp_shift) {                                   // the workgroup that copies the last chunk completes the entry
                complete = __hip_atomic_fetch_add(&a.chunks_done[i], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1 == (1u << cpp_shift);
                if (complete) __hip_atomic_store(&a.chunks_done[i], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next migration
            }
            if (complete) {
                if (swap) __hip_atomic_store(&a.page_table[vpage], kNone, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                __hip_atomic_store(&a.page_table[fpage], frame, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                __hip_atomic_store(&a.frame_owner[frame], fpage, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                // "mine is done" then "how far are we", against "we are this far" then "is the next one done":
                // with each step acknowledged before the next is issued, one of two workgroups sees the other's write
                __hip_atomic_store(&a.page_done[i], a.early_tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __builtin_amdgcn_s_waitcnt(0);                 // the table and the mark are out before `landed` is read
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                uint32_t p = __hip_atomic_load(a.landed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                while (p < a.n_fetch &&
                       __hip_atomic_load(&a.page_done[p], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == a.early_tag) {
                    uint32_t expected = p;                     // landed only grows: a failed exchange returns a larger value
                    if (__hip_atomic_compare_exchange_strong(a.landed, &expected, p + 1, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                             __HIP_MEMORY_SCOPE_AGENT))
                        p = p + 1;
                    else
                        p = expected;
                }
            }
        }
    }
}

// The device-side consumer of `landed`: one lane waits until the fetch entries command g needs are complete and
// returns, which lets the next kernel of its stream start.  The wait ends in any case: after timeout_ticks of the
// 100 MHz wall clock it gives up, and says so.  Frames were written with write-through stores before `landed`
// moved over them, and a kernel that starts after this one begins with fresh caches.
__global__ void k_gate(const uint32_t *landed, uint32_t need, uint64_t timeout_ticks, GateRec *out) {
    const uint64_t t0 = wall_clock64();
    uint32_t seen, status = 2;
    for (;;) {
        seen = __hip_atomic_load(landed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (seen >= need) { status = 1; break; }
        if (wall_clock64() - t0 > timeout_ticks) break;
        __builtin_amdgcn_s_sleep(64);
    }
    const uint64_t now = wall_clock64();
    const uint64_t began = __hip_atomic_load(reinterpret_cast<const uint64_t *>(landed + 2), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    out->seen = seen;
    out->ticks = (status == 1 && began != 0 && now > began) ? now - began : 0;
    __threadfence_system();
    __hip_atomic_store(&out->status, status, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ void k_peek(const uint32_t *landed, uint32_t *out) {
    *out = __hip_atomic_load(landed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(256) void k_fill_u32(uint32_t *dst, uint64_t n, uint32_t v) {
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < n; i += gridDim.x * (uint64_t)blockDim.x)
        dst[i] = v;
}

template <typename Id>
__global__ __launch_bounds__(256) void k_query(const uint32_t *__restrict__ page_table, const Id *__restrict__ ids,
                                               uint32_t n, uint32_t *__restrict__ out) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = page_table[ids[i]];
}

// Staging of msched_pagetable_query_static: n 64-bit page ids, then n 32-bit answers.  The array is part of the
// code object, so every GPU the library runs on holds its own copy at its own address; in host code its name is
// only a handle for hipGetSymbolAddress, never an address a kernel or a copy may be given.
constexpr size_t kQueryScratchBytes = (size_t)MSCHED_QUERY_STATIC_MAX * (sizeof(uint64_t) + sizeof(uint32_t));
static __device__ __align__(256) uint8_t scratch[kQueryScratchBytes];
constexpr int kMaxDevices = 64;
// device address of `scratch` on each GPU, once looked up (contexts of different threads may ask at the same time:
// they would store the same address)
static std::atomic<uint8_t *> g_scratch_ptr[kMaxDevices] = {};

// Look the array's address up on the current device (once per device) and keep it.
hipError_t query_scratch_init(uint8_t **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    uint8_t *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        if ((e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch))) != hipSuccess) return e;
        if (ptr == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    if (out) *out = ptr;
    return hipSuccess;
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
    k_query<uint32_t><<<(n + 255) / 256, 256, 0, c->stream>>>(c->page_table, ids_dev, n, out_dev);
    return hipGetLastError();
}

// The same gather through the static staging array: ids in, answers out, no allocation anywhere.
hipError_t query_static(msched_ctx *c, const uint64_t *page_ids, uint32_t n, uint32_t *out) {
    uint8_t *ptr = nullptr;
    hipError_t e = query_scratch_init(&ptr);               // a table look-up after msched_create has run on this device
    if (e != hipSuccess) return e;
    uint64_t *ids_dev = reinterpret_cast<uint64_t *>(ptr);
    uint32_t *out_dev = reinterpret_cast<uint32_t *>(ptr + (size_t)MSCHED_QUERY_STATIC_MAX * sizeof(uint64_t));
    if ((e = hipMemcpyAsync(ids_dev, page_ids, (size_t)n * sizeof(uint64_t), hipMemcpyHostToDevice, c->stream)) != hipSuccess) return e;
    (void)hipGetLastError();
    k_query<uint64_t><<<(n + 255) / 256, 256, 0, c->stream>>>(c->page_table, ids_dev, n, out_dev);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = hipMemcpyAsync(out, out_dev, (size_t)n * sizeof(uint32_t), hipMemcpyDeviceToHost, c->stream)) != hipSuccess) return e;
    return hipStreamSynchronize(c->stream);
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
    a.page_done = a.landed = nullptr; a.early_tag = 0;
    a.chunks_done = c->chunks_done;                            // counts the chunks of pages larger than a work unit (null if none can be)
    if (c->early && c->plan_early) {
        // Workgroups take consecutive chunks, so with chunks much smaller than the whole transfer the
        // entries are worked on, and complete, in list order.
        a.chunk_shift = std::min<uint32_t>(c->page_shift, c->early_chunk_shift);
        while (((uint64_t)h.n_fetch << (a.page_shift - a.chunk_shift)) >> 31) ++a.chunk_shift;   // the unit counter has 32 bits
        a.page_done = c->page_done; a.chunks_done = c->chunks_done; a.landed = c->landed;
        a.early_tag = c->early_tag;
    }
    a.n_units = (uint64_t)h.n_fetch << (a.page_shift - a.chunk_shift);
    const uint64_t blocks = std::min<uint64_t>(a.n_units, c->migrate_max_blocks);
    a.ticket = a.landed ? a.landed + 1 : c->flags + 1;
    if (a.landed) k_migrate<true, true><<<(uint32_t)blocks, 256, 0, c->stream>>>(a);
    else if (c->migrate_ticket) k_migrate<false, true><<<(uint32_t)blocks, 256, 0, c->stream>>>(a);
    else k_migrate<false, false><<<(uint32_t)blocks, 256, 0, c->stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_gate(msched_ctx *c, uint32_t g, uint32_t need, uint64_t timeout_ticks, hipStream_t stream) {
    (void)hipGetLastError();
    GateRec *out = nullptr;
    hipError_t e = hipHostGetDevicePointer((void **)&out, c->gate_host + g, 0);
    if (e != hipSuccess) return e;
    k_gate<<<1, 1, 0, stream>>>(c->landed, need, timeout_ticks, out);
    return hipGetLastError();
}

hipError_t launch_peek(msched_ctx *c) {
    (void)hipGetLastError();
    k_peek<<<1, 1, 0, c->poll_stream>>>(c->landed, c->progress_host);
    return hipGetLastError();
}

}  // namespace msched
