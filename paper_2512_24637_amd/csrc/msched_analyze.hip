// Offline memory analyzer for gfx950 (paper: arXiv 2512.24637, Sec. 5.2 "Memory analyzer"): from the
// launch arguments and touched byte intervals of a kernel's profiled invocations, derive the access
// rules (T1 fixed / T2 linear / T3 strided) that msched_kernel_register consumes.
//
// One wavefront per profiled kernel; kernels of a batch are independent, and a batch of thousands fills
// the chip with many resident wavefronts per compute unit, which is what hides the latency of the
// dependent loads (binary searches, run scans).  Inside a wavefront:
//   * lanes run over (invocation, pointer argument) pairs to decide which 64-bit arguments are base
//     pointers (their value starts a touched interval in every invocation), then over invocations to
//     measure the region at each base (chunk length, stride and count of the run that starts there);
//   * to fit "value = c * product(args[S])", lanes run over the candidate subsets S ({}, singles, pairs,
//     triples of the non-pointer arguments, in that order: at most 232) and screen each on the first few
//     invocations; survivors are then tested in rank order on every invocation with lanes over
//     invocations.  The first that passes is the lowest-ranked fit: the constant beats any product and a
//     single argument beats a pair.
#include <algorithm>
#include <cstddef>
#include <mutex>

#include "msched_internal.h"

// In-kernel timers of the timers build (see msched_plan.hip): thread 0 stores the 100 MHz wall clock at the phase
// boundaries of k_analyze, slot i of the wavefront's row of 16, for the first 65536 kernels of a batch.
#ifdef MSCHED_KERNEL_TIMERS
static __device__ uint64_t *g_ana_ticks = nullptr;
#define ANA_TICK(i)                                                                                          \
    do {                                                                                                    \
        if (threadIdx.x == 0 && g_ana_ticks != nullptr && blockIdx.x < 65536)                               \
            g_ana_ticks[(size_t)blockIdx.x * 16 + (i)] = wall_clock64();                                    \
    } while (0)
extern "C" int msched_debug_set_analyzer_ticks(uint64_t *buf) {
    return hipMemcpyToSymbol(HIP_SYMBOL(g_ana_ticks), &buf, sizeof buf) == hipSuccess ? MSCHED_OK : MSCHED_E_HIP;
}
#else
#define ANA_TICK(i) do { } while (0)
#endif

namespace msched {

constexpr int kAnaMaxInv = 512;
constexpr int kAnaMaxProd = 3;
constexpr int kAnaProbe = 3;                      // invocations a subset is screened on before the full test
constexpr int kAnaMaxSubsets = 1 + 12 + 66 + 220; // {} + singles + pairs + triples of 12 candidates

struct AnaArgs {
    uint32_t n_inv, max_iv;
    const int32_t *n_args; const uint32_t *int64_mask;
    const uint64_t *args, *iv; const uint32_t *n_iv;
    msched_rule *rules; uint32_t *n_rules, *unexplained;
};

// index of the interval of one invocation (sorted by start) that starts at addr, or -1
__device__ __forceinline__ int find_start(const uint64_t *row, uint32_t n, uint64_t addr) {
    uint32_t lo = 0, hi = n;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (row[2 * mid] < addr) lo = mid + 1; else hi = mid;
    }
    return (lo < n && row[2 * lo] == addr) ? (int)lo : -1;
}

// the rank-th subset in the order {} ; {a} ; {a,b} ; {a,b,c} over nc candidates, as positions in the
// candidate list packed one per byte, the size in the top byte
__device__ uint32_t unrank_subset(uint32_t rank, uint32_t nc) {
    if (rank == 0) return 0;
    rank -= 1;
    if (rank < nc) return (1u << 24) | rank;
    rank -= nc;
    for (uint32_t x = 0; x + 1 < nc; ++x) {
        const uint32_t row = nc - 1 - x;
        if (rank < row) return (2u << 24) | x | ((x + 1 + rank) << 8);
        rank -= row;
    }
    for (uint32_t x = 0; x + 2 < nc; ++x)
        for (uint32_t y = x + 1; y + 1 < nc; ++y) {
            const uint32_t row = nc - 1 - y;
            if (rank < row) return (3u << 24) | x | (y << 8) | ((y + 1 + rank) << 16);
            rank -= row;
        }
    return 0;
}

// v / p, p != 0; extents and argument values rarely need more than 32 bits, where the division is far cheaper
__device__ __forceinline__ uint64_t div_u64(uint64_t v, uint64_t p) {
    return ((v | p) >> 32) == 0 ? (uint64_t)((uint32_t)v / (uint32_t)p) : v / p;
}

__device__ __forceinline__ bool mul_ok(uint64_t a, uint64_t b, uint64_t &out) {
    out = a * b;
    return __umul64hi(a, b) == 0;
}

// argument indices of a product; plain members so that they stay in registers
struct Subset {
    int n = 0;
    uint32_t a0 = 0, a1 = 0, a2 = 0;
    __device__ __forceinline__ uint32_t at(int j) const { return j == 0 ? a0 : j == 1 ? a1 : a2; }
};
static_assert(kAnaMaxProd == 3, "Subset holds three indices");

// the invocations a subset is screened on; plain members, selected by comparison, so that they stay in registers
struct Probes {
    int n = 0;
    uint32_t i0 = 0, i1 = 0, i2 = 0;
    __device__ uint32_t at(int t) const { return t == 0 ? i0 : t == 1 ? i1 : i2; }
};
static_assert(kAnaProbe == 3, "Probes holds three invocations");

__device__ __forceinline__ bool product_of(const uint64_t *row, const Subset &S, uint64_t &prod) {
    prod = 1;
    bool ok = true;
    if (S.n > 0) ok &= mul_ok(prod, row[S.a0], prod);
    if (S.n > 1) ok &= mul_ok(prod, row[S.a1], prod);
    if (S.n > 2) ok &= mul_ok(prod, row[S.a2], prod);
    return ok;
}

// One wavefront analyzes one kernel.  Lanes run over invocations (finding intervals, measuring regions,
// testing one formula on all invocations) or over candidate subsets (screening each on a few invocations).
struct Analyzer {
    uint32_t n_inv, lane;
    const uint64_t *s_args;         // LDS [n_inv][12]
    const uint64_t *val;            // LDS [n_inv]: the quantity being fitted
    const uint64_t *count;          // LDS [n_inv]: chunks in the region
    bool multi_only;                // fit over invocations with more than one chunk only
    const uint32_t *subsets;        // global [n_subsets] packed positions (a row of the subset table)
    const uint32_t *cand;           // LDS [nc] argument index of each candidate
    uint32_t n_subsets, n_singles;
    uint32_t first_ranks, next_ranks;   // this lane's entry of the table for the first two screening rounds (ranks 1 + lane
                                        // and 1 + n_singles + lane): every search starts with them, so they are read once

    __device__ __forceinline__ bool used(uint32_t i) const { return !multi_only || count[i] > 1; }

    __device__ __forceinline__ Subset unpack(uint32_t packed) const {
        Subset S;
        S.n = (int)(packed >> 24);
        S.a0 = S.n > 0 ? cand[packed & 0xff] : 0;
        S.a1 = S.n > 1 ? cand[(packed >> 8) & 0xff] : 0;
        S.a2 = S.n > 2 ? cand[(packed >> 16) & 0xff] : 0;
        return S;
    }

    // per lane: could value = c * product(args[S]) hold, judging by the probe invocations alone?
    __device__ __forceinline__ bool screen(const Subset &S, const Probes &probe) const {
        uint64_t c = 0;
        bool have_c = false;
        for (int t = 0; t < kAnaProbe; ++t) {
            if (t >= probe.n) break;
            const uint32_t i = probe.at(t);
            uint64_t prod, want;
            if (!product_of(s_args + i * MSCHED_MAX_ARGS, S, prod)) return false;
            const uint64_t v = val[i];
            if (!have_c) {
                if (prod == 0) { if (v != 0) return false; continue; }
                c = div_u64(v, prod);
                if (c == 0 || c * prod != v) return false;
                have_c = true;
            } else if (!mul_ok(c, prod, want) || want != v) return false;
        }
        return true;
    }

    // whole wave, S uniform: the test on every used invocation; the coefficient comes from the first used
    // invocation whose product is not zero
    __device__ __forceinline__ bool verify(const Subset &S, uint64_t &c_out) const {
        uint64_t c = 0;
        bool have_c = false;
        for (uint32_t i0 = 0; i0 < n_inv && !have_c; i0 += kWave) {
            const uint32_t i = i0 + lane;
            const bool act = i < n_inv && used(i);
            uint64_t prod = 0;
            bool ovf = false;
            if (act) ovf = !product_of(s_args + i * MSCHED_MAX_ARGS, S, prod);
            const uint64_t m = __ballot(act && (ovf || prod != 0));
            if (m) {
                const int l = __ffsll((unsigned long long)m) - 1;
                if (__shfl((int)ovf, l)) return false;
                const uint64_t p = __shfl((unsigned long long)prod, l), v = __shfl((unsigned long long)(act ? val[i] : 0), l);
                c = div_u64(v, p);
                if (c == 0 || c * p != v) return false;
                have_c = true;
            }
        }
        if (!have_c) return false;
        for (uint32_t i0 = 0; i0 < n_inv; i0 += kWave) {
            const uint32_t i = i0 + lane;
            bool bad = false;
            if (i < n_inv && used(i)) {
                uint64_t prod, want;
                bad = !product_of(s_args + i * MSCHED_MAX_ARGS, S, prod) || !mul_ok(c, prod, want) || want != val[i];
            }
            if (__ballot(bad)) return false;
        }
        c_out = c;
        return true;
    }

    // whole wave: verify() for the empty subset, written out - the product is 1, so the coefficient is the first used
    // invocation's value, which must not be zero, and every used invocation must show the same value.  Most regions
    // have an invariant extent and end their search here: no product, no division.
    __device__ __forceinline__ bool verify_invariant(uint64_t &c_out) const {
        uint64_t c = 0;
        bool have_c = false, differs = false;
        for (uint32_t i0 = 0; i0 < n_inv; i0 += kWave) {
            const uint32_t i = i0 + lane;
            const bool act = i < n_inv && used(i);
            const uint64_t v = act ? val[i] : 0;
            if (!have_c) {
                const uint64_t m = __ballot(act);
                if (!m) continue;
                c = __shfl((unsigned long long)v, __ffsll((unsigned long long)m) - 1);
                if (c == 0) return false;
                have_c = true;
            }
            differs |= act && v != c;
        }
        if (!have_c || __ballot(differs)) return false;
        c_out = c;
        return true;
    }

    // whole wave: the lowest-ranked subset that fits
    __device__ __forceinline__ bool search(Subset &S_out, uint64_t &c_out) const {
        // screen on the first (up to three) used invocations of the first 64-invocation block that has any
        Probes probe;
        for (uint32_t i0 = 0; i0 < n_inv && probe.n == 0; i0 += kWave) {
            const uint32_t i = i0 + lane;
            uint64_t m = __ballot(i < n_inv && used(i));
            if (m) { probe.i0 = i0 + __ffsll((unsigned long long)m) - 1; probe.n = 1; m &= m - 1; }
            if (m) { probe.i1 = i0 + __ffsll((unsigned long long)m) - 1; probe.n = 2; m &= m - 1; }
            if (m) { probe.i2 = i0 + __ffsll((unsigned long long)m) - 1; probe.n = 3; }
        }
        if (probe.n == 0) return false;
        // {} first and on its own: most regions have an invariant extent (template T1) and need nothing else;
        // then the single arguments, then pairs and triples a wavefront at a time
        Subset none;
        if (verify_invariant(c_out)) { S_out = none; return true; }
        const uint32_t n_cand = n_singles;
        for (uint32_t r0 = 1; r0 < n_subsets;) {
            const uint32_t r1 = min(r0 <= n_cand ? 1 + n_cand : r0 + kWave, n_subsets);
            const uint32_t rank = r0 + lane;
            uint32_t packed = 0;
            if (r0 == 1) packed = first_ranks;
            else if (r0 == 1 + n_cand) packed = next_ranks;
            else if (rank < r1) packed = subsets[rank];
            const bool pass = rank < r1 && screen(unpack(packed), probe);
            uint64_t m = __ballot(pass);
            while (m) {
                const int l = __ffsll((unsigned long long)m) - 1;      // the lowest rank that passed the screen
                m &= m - 1;
                const Subset S = unpack((uint32_t)__shfl((int)packed, l));
                if (verify(S, c_out)) { S_out = S; return true; }
            }
            r0 = r1;
        }
        return false;
    }
};

// subsets in search order for every possible number of candidates; filled once per device
__device__ uint32_t g_subset_table[MSCHED_MAX_ARGS + 1][kAnaMaxSubsets];

__device__ __host__ constexpr uint32_t subsets_of(uint32_t nc) {
    return 1 + nc + nc * (nc - 1) / 2 + (nc >= 3 ? nc * (nc - 1) * (nc - 2) / 6 : 0);
}

__global__ void k_subset_table() {
    const uint32_t nc = blockIdx.x;
    for (uint32_t r = threadIdx.x; r < subsets_of(nc); r += blockDim.x) g_subset_table[nc][r] = unrank_subset(r, nc);
}

static_assert(sizeof(msched_rule) == 48 && offsetof(msched_rule, size_args) == 5 && offsetof(msched_rule, stride_args) == 9 &&
              offsetof(msched_rule, count_args) == 13 && offsetof(msched_rule, size_coeff) == 24,
              "rule_words packs this layout");

// the first 24 bytes of a msched_rule as three little-endian words
__device__ __forceinline__ void rule_words(uint32_t kind, uint32_t base_arg, const Subset &size, const Subset &stride,
                                           const Subset &count, uint64_t w[3]) {
    auto at = [](const Subset &S, int j) { return (uint64_t)(j < S.n ? S.at(j) : 0); };
    w[0] = kind | (uint64_t)base_arg << 8 | (uint64_t)size.n << 16 | (uint64_t)stride.n << 24 | (uint64_t)count.n << 32 |
           at(size, 0) << 40 | at(size, 1) << 48 | at(size, 2) << 56;
    w[1] = at(stride, 0) << 8 | at(stride, 1) << 16 | at(stride, 2) << 24 | at(count, 0) << 40 | at(count, 1) << 48 |
           at(count, 2) << 56;
    w[2] = 0;
}

constexpr uint32_t kHead = 8;                     // intervals of an invocation that its lane keeps in registers

// intervals mo .. mo + 7 of one invocation's row (indices clamped to the row: every row has max_iv entries allocated)
__device__ __forceinline__ void load8(const ulonglong2 *row, uint32_t mo, uint32_t max_iv, ulonglong2 (&c)[kHead]) {
    #pragma unroll
    for (uint32_t j = 0; j < kHead; ++j) c[j] = row[min(mo + j, max_iv - 1)];
}

// where, among the intervals mo .. mo + 7 of a row of n, does each 64-bit argument (bits of mask) start one?
__device__ __forceinline__ void scan8(const ulonglong2 (&c)[kHead], uint32_t mo, uint32_t n, uint32_t mask,
                                      const ulonglong2 (&av)[MSCHED_MAX_ARGS / 2], uint32_t (&found)[MSCHED_MAX_ARGS]) {
    #pragma unroll
    for (int arg = 0; arg < MSCHED_MAX_ARGS; ++arg) {
        if ((mask >> arg) & 1) {
            const uint64_t v = (arg & 1) ? av[arg / 2].y : av[arg / 2].x;
            #pragma unroll
            for (int j = (int)kHead - 1; j >= 0; --j)
                if (mo + j < n && c[j].x == v) found[arg] = mo + j;
        }
    }
}

constexpr uint32_t kArgBatch = 6;                 // 16-byte loads a lane keeps in flight while staging arguments
constexpr uint32_t kNoInterval = 0xffff;
static_assert(kArgBatch * 2 == MSCHED_MAX_ARGS, "one trip of the staging loop moves 64 whole argument rows");
static_assert(MSCHED_MAX_ARGS % 2 == 0, "argument rows are read two at a time");

// Every phase that reads global memory issues all its loads before it looks at any of them: one wavefront
// has little else to hide a memory round trip behind, and the number of dependent round trips is what its
// run time is made of.
__global__ __launch_bounds__(kWave) void k_analyze(AnaArgs a) {
    extern __shared__ __align__(16) uint64_t ana_lds[];
    const uint32_t k = blockIdx.x, n_inv = a.n_inv, max_iv = a.max_iv, lane = threadIdx.x;
    uint64_t *s_args = ana_lds;                                   // [n_inv][12]
    uint64_t *chunk = s_args + (size_t)n_inv * MSCHED_MAX_ARGS;   // [n_inv]
    uint64_t *stride = chunk + n_inv, *count = stride + n_inv;    // [n_inv] each
    uint32_t *s_niv = reinterpret_cast<uint32_t *>(count + n_inv);                 // [n_inv]
    uint16_t *s_m0 = reinterpret_cast<uint16_t *>(s_niv + n_inv); // [12][n_inv]: interval index at each pointer
    __shared__ uint32_t s_cand[MSCHED_MAX_ARGS];
    const ulonglong2 *g_args = reinterpret_cast<const ulonglong2 *>(a.args + (size_t)k * n_inv * MSCHED_MAX_ARGS);
    const ulonglong2 *g_iv = reinterpret_cast<const ulonglong2 *>(a.iv + (size_t)k * n_inv * max_iv * 2);   // (start, length)
    const uint32_t *g_niv = a.n_iv + (size_t)k * n_inv;
    ANA_TICK(0);
    // A lane keeps the first eight intervals of "its" invocation (the one with its number) in registers from here to
    // the end: pointer matching, and the regions measured at every base, find them there.  They are asked for before
    // anything else, so that they travel together with the arguments; slots beyond a row's count lie inside the row
    // and are ignored.  A row of eight intervals is one 128-byte line, read by one lane.
    ulonglong2 head[kHead];
    load8(g_iv + (size_t)min(lane, n_inv - 1) * max_iv, 0, max_iv, head);
    // 0. arguments and interval counts into LDS
    uint32_t total = 0;
    {
        ulonglong2 *s2 = reinterpret_cast<ulonglong2 *>(s_args);
        const uint32_t n2 = n_inv * (MSCHED_MAX_ARGS / 2);
        for (uint32_t f = lane; f < n2; f += kArgBatch * kWave) {
            // every load is issued (at a clamped index) before any is stored: all six are in flight together
            const ulonglong2 v0 = g_args[min(f, n2 - 1)], v1 = g_args[min(f + kWave, n2 - 1)],
                             v2 = g_args[min(f + 2 * kWave, n2 - 1)], v3 = g_args[min(f + 3 * kWave, n2 - 1)],
                             v4 = g_args[min(f + 4 * kWave, n2 - 1)], v5 = g_args[min(f + 5 * kWave, n2 - 1)];
            const uint32_t i = f / (kArgBatch * kWave) * kWave + lane;   // one invocation per lane and trip: 64 rows are 6 * 64 loads
            uint32_t niv = g_niv[min(i, n_inv - 1)];
            s2[f] = v0;
            if (f + kWave < n2) s2[f + kWave] = v1;
            if (f + 2 * kWave < n2) s2[f + 2 * kWave] = v2;
            if (f + 3 * kWave < n2) s2[f + 3 * kWave] = v3;
            if (f + 4 * kWave < n2) s2[f + 4 * kWave] = v4;
            if (f + 5 * kWave < n2) s2[f + 5 * kWave] = v5;
            if (i < n_inv) { niv = min(niv, max_iv); s_niv[i] = niv; total += niv; }
        }
    }
    const int n_args = min(max(a.n_args[k], 0), MSCHED_MAX_ARGS);
    const uint32_t mask = a.int64_mask[k] & ((1u << n_args) - 1);
    __syncthreads();
    ANA_TICK(1);
    // 1. base pointers: 64-bit arguments whose value starts an interval in every invocation.  A lane takes whole
    //    invocations: the row of arguments from LDS in one go, the row's intervals eight at a time, every start
    //    compared with every 64-bit argument.  (Starts within a row are distinct: at most one interval matches.)
    uint32_t unmatched = 0;                  // bit a: argument a starts no interval in one of this lane's invocations
    if (mask)
        for (uint32_t ib = 0; ib < n_inv; ib += kWave) {
            const uint32_t i = ib + lane;
            if (i >= n_inv) continue;
            const uint32_t n = s_niv[i];
            const ulonglong2 *arow2 = reinterpret_cast<const ulonglong2 *>(s_args + i * MSCHED_MAX_ARGS);
            ulonglong2 av[MSCHED_MAX_ARGS / 2];
            #pragma unroll
            for (int j = 0; j < MSCHED_MAX_ARGS / 2; ++j) av[j] = arow2[j];
            uint32_t found[MSCHED_MAX_ARGS];
            #pragma unroll
            for (int arg = 0; arg < MSCHED_MAX_ARGS; ++arg) found[arg] = kNoInterval;
            if (ib == 0) scan8(head, 0, n, mask, av, found);
            for (uint32_t mo = ib == 0 ? kHead : 0; mo < n; mo += kHead) {
                ulonglong2 c[kHead];
                load8(g_iv + (size_t)i * max_iv, mo, max_iv, c);
                scan8(c, mo, n, mask, av, found);
            }
            #pragma unroll
            for (int arg = 0; arg < MSCHED_MAX_ARGS; ++arg)
                if ((mask >> arg) & 1) {
                    s_m0[arg * n_inv + i] = (uint16_t)found[arg];
                    unmatched |= (found[arg] == kNoInterval ? 1u : 0u) << arg;
                }
        }
    __syncthreads();
    ANA_TICK(2);
    uint32_t nc = 0, base_mask = 0;
    for (int arg = 0; arg < n_args; ++arg) {
        const bool missing = !((mask >> arg) & 1) || ((unmatched >> arg) & 1);
        if (__ballot(missing) == 0) base_mask |= 1u << arg;
        else { if (lane == 0) s_cand[nc] = arg; ++nc; }
    }
    // an argument that equals a lower base in every invocation is an alias and gets no rule
    uint32_t live_mask = 0;
    for (uint32_t rest = base_mask; rest; rest &= rest - 1) {
        const uint32_t arg = __builtin_ctz(rest);
        bool alias = false;
        for (uint32_t lower = base_mask & ((1u << arg) - 1); lower && !alias; lower &= lower - 1) {
            const uint32_t b = __builtin_ctz(lower);
            bool differs = false;
            for (uint32_t i = lane; i < n_inv; i += kWave)
                differs |= s_args[i * MSCHED_MAX_ARGS + arg] != s_args[i * MSCHED_MAX_ARGS + b];
            alias = __ballot(differs) == 0;
        }
        if (!alias) live_mask |= 1u << arg;
    }
    const uint32_t n_subsets = subsets_of(nc);
    Analyzer an;
    an.subsets = g_subset_table[nc];
    an.first_ranks = 1 + lane < n_subsets ? an.subsets[1 + lane] : 0;
    an.next_ranks = 1 + nc + lane < n_subsets ? an.subsets[1 + nc + lane] : 0;
    // Which of the first 32 intervals of invocation i start at a base pointer: a region's run of chunks ends in front
    // of them.  All twelve index entries are read at once (those of other arguments hold nothing and are masked out).
    auto bases_at = [&](uint32_t i) __attribute__((always_inline)) -> uint32_t {
        uint32_t at = 0;
        #pragma unroll
        for (int b = 0; b < MSCHED_MAX_ARGS; ++b) {
            const uint32_t m = s_m0[b * n_inv + i];
            at |= ((base_mask >> b) & 1) && m < 32 ? 1u << m : 0u;
        }
        return at;
    };
    const uint32_t own_bases_at = lane < n_inv ? bases_at(lane) : 0;
    ANA_TICK(3);
    an.n_inv = n_inv; an.lane = lane; an.s_args = s_args; an.count = count;
    an.cand = s_cand; an.n_subsets = n_subsets; an.n_singles = nc;
    uint32_t n_rules = 0, covered = 0, accepted_mask = 0;
    for (uint32_t rest = live_mask; rest; rest &= rest - 1) {
        const uint32_t arg = __builtin_ctz(rest);
        if (n_rules == 0) ANA_TICK(4);
        // 2. the region that starts at this base, per invocation: a run of equal intervals at a regular stride
        bool any_multi = false;
        for (uint32_t i = lane; i < n_inv; i += kWave) {
            const uint64_t *arow = s_args + i * MSCHED_MAX_ARGS;
            const uint32_t n = s_niv[i], m0 = s_m0[arg * n_inv + i];
            const uint32_t at = i < kWave ? own_bases_at : bases_at(i);
            uint64_t len = 0, st = 0, cnt = 1, prev = 0;
            uint32_t m = m0 + 1;                                  // the next interval to look at
            bool stopped = false;
            if (i < kWave && m0 < kHead) {
                // The lane's own first eight intervals are in its registers: walked in order with fixed indices (the
                // run starts at a different one in every lane), which costs a dozen instructions an interval where a
                // select over the eight for a lane's own index costs sixty.
                #pragma unroll
                for (uint32_t j = 0; j < kHead; ++j) {
                    const ulonglong2 cur = head[j];
                    if (j == m0) { len = cur.y; prev = cur.x; }
                    else if (j > m0 && j < n && !stopped) {
                        const uint64_t gap = cur.x - prev;
                        if (cur.y != len || ((at >> j) & 1) || (cnt > 1 && gap != st)) stopped = true;
                        else { st = gap; prev = cur.x; ++cnt; }
                    }
                }
                m = kHead;
            } else {
                const ulonglong2 first = g_iv[(size_t)i * max_iv + m0];
                len = first.y; prev = first.x;
            }
            for (; !stopped && m < n; ++m) {
                const ulonglong2 next = g_iv[(size_t)i * max_iv + m];
                bool other = next.y != len;
                if (m < 32) other |= (at >> m) & 1;
                else
                    for (uint32_t bases = base_mask & ~(1u << arg); bases; bases &= bases - 1)
                        other |= arow[__builtin_ctz(bases)] == next.x;
                const uint64_t gap = next.x - prev;
                if (other || (cnt > 1 && gap != st)) break;
                st = gap; prev = next.x; ++cnt;
            }
            chunk[i] = len; stride[i] = st; count[i] = cnt;
            any_multi |= cnt > 1;
        }
        __syncthreads();
        if (n_rules == 0) ANA_TICK(5);
        const bool strided = __ballot(any_multi) != 0;
        // 3. templates in order: invariant size, size proportional to arguments, strided
        Subset S_size, S_stride, S_count;
        uint64_t c_size = 0, c_stride = 0, c_count = 0;
        bool ok = true;
        for (int q = 0; q < (strided ? 3 : 1) && ok; ++q) {       // size; then stride and count of a strided region
            an.val = q == 0 ? chunk : q == 1 ? stride : count;
            an.multi_only = q == 1;
            Subset S;
            uint64_t c = 0;
            ok = an.search(S, c);
            if (q == 0) { S_size = S; c_size = c; } else if (q == 1) { S_stride = S; c_stride = c; } else { S_count = S; c_count = c; }
        }
        if (n_rules == 0) ANA_TICK(6);
        if (ok && n_rules < MSCHED_MAX_RULES) {
            uint64_t w[3];
            rule_words(strided ? MSCHED_RULE_STRIDED : (S_size.n == 0 ? MSCHED_RULE_FIXED : MSCHED_RULE_LINEAR), arg,
                       S_size, S_stride, S_count, w);
            const uint64_t word = lane == 0 ? w[0] : lane == 1 ? w[1] : lane == 2 ? w[2] : lane == 3 ? c_size :
                                  lane == 4 ? c_stride : c_count;
            if (lane < 6) reinterpret_cast<uint64_t *>(a.rules + (size_t)k * MSCHED_MAX_RULES + n_rules)[lane] = word;
            // What the rule accounts for.  Two bases that hold the same address in an invocation start the
            // same run there (a run never reaches past another base), so it is counted for the first only.
            for (uint32_t i = lane; i < n_inv; i += kWave) {
                bool seen = false;
                for (uint32_t lower = accepted_mask; lower; lower &= lower - 1)
                    seen |= s_args[i * MSCHED_MAX_ARGS + __builtin_ctz(lower)] == s_args[i * MSCHED_MAX_ARGS + arg];
                if (!seen) covered += (uint32_t)count[i];
            }
            accepted_mask |= 1u << arg;
            ++n_rules;
        }
        __syncthreads();                                          // chunk / stride / count are reused by the next base
    }
    ANA_TICK(7);
    int unexplained = (int)total - (int)covered;
    for (int off = kWave / 2; off > 0; off >>= 1) unexplained += __shfl_down(unexplained, off);
    if (lane == 0) {
        a.n_rules[k] = n_rules;
        a.unexplained[k] = (uint32_t)unexplained;
    }
    ANA_TICK(8);
}

}  // namespace msched

using namespace msched;

namespace {

// The subset table is written by a kernel the first time a device is used, and waited for, so that later
// calls on any stream find it complete.
hipError_t ensure_subset_table(hipStream_t stream) {
    static std::mutex mu;
    static bool ready[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (ready[dev]) return hipSuccess;
    (void)hipGetLastError();
    k_subset_table<<<MSCHED_MAX_ARGS + 1, kWave, 0, stream>>>();
    e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e == hipSuccess) ready[dev] = true;
    return e;
}

}  // namespace

extern "C" int msched_analyze(const msched_profile_batch *b, msched_rule *rules, uint32_t *n_rules,
                              uint32_t *unexplained, void *stream) {
    if (!b || !rules || !n_rules || !unexplained) return MSCHED_E_INVAL;
    if (b->n_kernels == 0) return MSCHED_OK;
    if (!b->n_args || !b->int64_mask || !b->args || !b->intervals || !b->n_intervals) return MSCHED_E_INVAL;
    if (b->n_invocations == 0 || b->n_invocations > (uint32_t)kAnaMaxInv || b->max_intervals == 0 ||
        b->max_intervals > 65535u)
        return MSCHED_E_INVAL;
    if (((uintptr_t)b->args | (uintptr_t)b->intervals) & 15 || ((uintptr_t)rules & 7)) return MSCHED_E_INVAL;
    hipError_t e = ensure_subset_table((hipStream_t)stream);
    if (e != hipSuccess) { g_last_hip = (int)e; return MSCHED_E_HIP; }
    AnaArgs a;
    a.n_inv = b->n_invocations; a.max_iv = b->max_intervals;
    a.n_args = b->n_args; a.int64_mask = b->int64_mask; a.args = b->args; a.iv = b->intervals; a.n_iv = b->n_intervals;
    a.rules = rules; a.n_rules = n_rules; a.unexplained = unexplained;
    const size_t lds = (size_t)a.n_inv * ((MSCHED_MAX_ARGS + 3) * 8 + 4 + MSCHED_MAX_ARGS * 2);
    (void)hipGetLastError();
    if (lds > 48 * 1024)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_analyze), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) {
        k_analyze<<<b->n_kernels, kWave, lds, (hipStream_t)stream>>>(a);
        e = hipGetLastError();
    }
    if (e != hipSuccess) { g_last_hip = (int)e; return MSCHED_E_HIP; }
    return MSCHED_OK;
}
