// Offline memory analyzer for gfx950 (paper: arXiv 2512.24637, Sec. 5.2 "Memory analyzer"): from the
// launch arguments and touched byte intervals of a kernel's profiled invocations, derive the access
// rules (T1 fixed / T2 linear / T3 strided) that msched_kernel_register consumes.
//
// One workgroup per profiled kernel; kernels of a batch are independent.  Inside a workgroup:
//   * threads run over invocations to decide which 64-bit arguments are base pointers (their value
//     starts a touched interval in every invocation) and to measure the region at each base
//     (chunk length, stride and chunk count of the run of equal intervals that starts there);
//   * threads run over candidate argument subsets ({}, singles, pairs, triples of the non-pointer
//     arguments, in that order: at most 232) to test "value = c * product(args[S])" on every invocation;
//     the lowest-ranked subset that fits wins, which makes the constant beat any product and a single
//     argument beat a pair.
#include <algorithm>

#include "msched_internal.h"

namespace msched {

constexpr int kAnaThreads = 256;
constexpr int kAnaMaxInv = 512;
constexpr uint32_t kAnaMaxBits = 262144;          // n_invocations * max_intervals at most (coverage bitmap in LDS)
constexpr int kAnaMaxProd = 3;

struct AnaArgs {
    uint32_t n_inv, max_iv;
    const int32_t *n_args; const uint32_t *int64_mask;
    const uint64_t *args, *iv; const uint32_t *n_iv;
    msched_rule *rules; uint32_t *n_rules, *unexplained;
};

// index of the interval of invocation row `iv` (sorted by start) that starts at addr, or -1
__device__ __forceinline__ int find_start(const uint64_t *iv, uint32_t n, uint64_t addr) {
    uint32_t lo = 0, hi = n;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (iv[2 * mid] < addr) lo = mid + 1; else hi = mid;
    }
    return (lo < n && iv[2 * lo] == addr) ? (int)lo : -1;
}

// the rank-th subset in the order {} ; {a} ; {a,b} ; {a,b,c} over nc candidates; returns its size
__device__ __forceinline__ int unrank_subset(uint32_t rank, uint32_t nc, uint32_t *pos) {
    if (rank == 0) return 0;
    rank -= 1;
    if (rank < nc) { pos[0] = rank; return 1; }
    rank -= nc;
    for (uint32_t x = 0; x < nc; ++x) {
        const uint32_t row = nc - 1 - x;
        if (rank < row) { pos[0] = x; pos[1] = x + 1 + rank; return 2; }
        rank -= row;
    }
    for (uint32_t x = 0; x < nc; ++x)
        for (uint32_t y = x + 1; y < nc; ++y) {
            const uint32_t row = nc - 1 - y;
            if (rank < row) { pos[0] = x; pos[1] = y; pos[2] = y + 1 + rank; return 3; }
            rank -= row;
        }
    return -1;
}

__device__ __forceinline__ bool mul_ok(uint64_t a, uint64_t b, uint64_t &out) {
    out = a * b;
    return __umul64hi(a, b) == 0;
}

// Does value_i = c * product(args_i[S]) hold for every invocation with use_i != 0?  (c: from the first
// such invocation whose product is not zero; c >= 1.)
__device__ bool subset_fits(const uint64_t *s_args, uint32_t n_inv, const uint64_t *val, const uint8_t *use,
                            const uint32_t *S, int nS, uint64_t &c_out) {
    uint64_t c = 0;
    bool have_c = false;
    for (uint32_t i = 0; i < n_inv && !have_c; ++i) {
        if (!use[i]) continue;
        uint64_t prod = 1;
        for (int j = 0; j < nS; ++j)
            if (!mul_ok(prod, s_args[i * MSCHED_MAX_ARGS + S[j]], prod)) return false;
        if (prod != 0) {
            if (val[i] % prod) return false;
            c = val[i] / prod;
            have_c = true;
        }
    }
    if (!have_c || c == 0) return false;
    for (uint32_t i = 0; i < n_inv; ++i) {
        if (!use[i]) continue;
        uint64_t prod = 1, want;
        for (int j = 0; j < nS; ++j)
            if (!mul_ok(prod, s_args[i * MSCHED_MAX_ARGS + S[j]], prod)) return false;
        if (!mul_ok(c, prod, want) || want != val[i]) return false;
    }
    c_out = c;
    return true;
}

struct Fit { int n; uint32_t idx[kAnaMaxProd]; uint64_t coeff; };

// Block-wide: first fitting subset (lowest rank) for the values val[] over the invocations use[].
__device__ bool fit_search(const uint64_t *s_args, uint32_t n_inv, const uint32_t *cand, uint32_t nc,
                           const uint64_t *val, const uint8_t *use, uint32_t *s_best, uint64_t *s_coeff, Fit &out) {
    const uint32_t n_subsets = 1 + nc + nc * (nc - 1) / 2 + nc * (nc - 1) * (nc - 2) / 6;
    if (threadIdx.x == 0) *s_best = kNone;
    __syncthreads();
    for (uint32_t rank = threadIdx.x; rank < n_subsets; rank += blockDim.x) {
        uint32_t pos[kAnaMaxProd], S[kAnaMaxProd];
        const int nS = unrank_subset(rank, nc, pos);
        for (int j = 0; j < nS; ++j) S[j] = cand[pos[j]];
        uint64_t c;
        if (*s_best > rank && subset_fits(s_args, n_inv, val, use, S, nS, c)) atomicMin(s_best, rank);
    }
    __syncthreads();
    const uint32_t best = *s_best;
    if (best == kNone) return false;
    uint32_t pos[kAnaMaxProd];
    out.n = unrank_subset(best, nc, pos);
    for (int j = 0; j < out.n; ++j) out.idx[j] = cand[pos[j]];
    if (threadIdx.x == best % blockDim.x) {                 // the thread that tested it recomputes the coefficient
        uint64_t c = 0;
        subset_fits(s_args, n_inv, val, use, out.idx, out.n, c);
        *s_coeff = c;
    }
    __syncthreads();
    out.coeff = *s_coeff;
    __syncthreads();
    return true;
}

__global__ __launch_bounds__(kAnaThreads) void k_analyze(AnaArgs a) {
    extern __shared__ uint64_t ana_lds[];
    const uint32_t k = blockIdx.x, n_inv = a.n_inv, max_iv = a.max_iv, tid = threadIdx.x;
    uint64_t *s_args = ana_lds;                                   // [n_inv][12]
    uint64_t *chunk = s_args + (size_t)n_inv * MSCHED_MAX_ARGS;   // [n_inv]
    uint64_t *stride = chunk + n_inv, *count = stride + n_inv;    // [n_inv] each
    uint32_t *covered = reinterpret_cast<uint32_t *>(count + n_inv);               // [(n_inv * max_iv + 31) / 32]
    const uint32_t cov_words = (n_inv * max_iv + 31) / 32;
    uint8_t *all_inv = reinterpret_cast<uint8_t *>(covered + cov_words);           // [n_inv]
    uint8_t *multi = all_inv + n_inv;                                              // [n_inv]
    __shared__ uint32_t s_flag[MSCHED_MAX_ARGS], s_alias, s_any_multi, s_best, s_covered, s_total, cand[MSCHED_MAX_ARGS];
    __shared__ uint64_t s_coeff;
    __shared__ uint32_t s_n_rules;
    const int n_args = min(max(a.n_args[k], 0), MSCHED_MAX_ARGS);
    const uint32_t mask = a.int64_mask[k];
    const uint64_t *g_args = a.args + (size_t)k * n_inv * MSCHED_MAX_ARGS;
    const uint64_t *g_iv = a.iv + (size_t)k * n_inv * max_iv * 2;
    const uint32_t *g_niv = a.n_iv + (size_t)k * n_inv;
    for (uint32_t i = tid; i < n_inv * MSCHED_MAX_ARGS; i += blockDim.x) s_args[i] = g_args[i];
    for (uint32_t i = tid; i < cov_words; i += blockDim.x) covered[i] = 0;
    for (uint32_t i = tid; i < n_inv; i += blockDim.x) all_inv[i] = 1;
    if (tid < MSCHED_MAX_ARGS) s_flag[tid] = (tid < (uint32_t)n_args && ((mask >> tid) & 1) && n_inv > 0) ? 1u : 0u;
    if (tid == 0) { s_n_rules = 0; s_covered = 0; s_total = 0; }
    __syncthreads();
    // 1. base pointers
    for (int arg = 0; arg < n_args; ++arg) {
        if (!((mask >> arg) & 1)) continue;
        bool ok = true;
        for (uint32_t i = tid; i < n_inv && ok; i += blockDim.x)
            ok = find_start(g_iv + (size_t)i * max_iv * 2, min(g_niv[i], max_iv), s_args[i * MSCHED_MAX_ARGS + arg]) >= 0;
        if (!ok) atomicAnd(&s_flag[arg], 0u);
    }
    uint32_t total = 0;
    for (uint32_t i = tid; i < n_inv; i += blockDim.x) total += min(g_niv[i], max_iv);
    if (total) atomicAdd(&s_total, total);
    __syncthreads();
    uint32_t nc = 0;                                              // candidates for products: the non-pointer arguments
    for (int arg = 0; arg < n_args; ++arg) if (!s_flag[arg]) { if (tid == 0) cand[nc] = arg; ++nc; }
    __syncthreads();
    for (int arg = 0; arg < n_args; ++arg) {
        if (!s_flag[arg]) continue;                               // uniform across the block
        // an argument that equals a lower base in every invocation is an alias
        bool alias = false;
        for (int b = 0; b < arg && !alias; ++b) {
            if (!s_flag[b]) continue;
            if (tid == 0) s_alias = 1;
            __syncthreads();
            bool same = true;
            for (uint32_t i = tid; i < n_inv && same; i += blockDim.x)
                same = s_args[i * MSCHED_MAX_ARGS + arg] == s_args[i * MSCHED_MAX_ARGS + b];
            if (!same) atomicAnd(&s_alias, 0u);
            __syncthreads();
            alias = s_alias != 0;
            __syncthreads();
        }
        if (alias) continue;
        // 2. the region that starts at this base, per invocation
        if (tid == 0) s_any_multi = 0;
        __syncthreads();
        for (uint32_t i = tid; i < n_inv; i += blockDim.x) {
            const uint64_t *row = g_iv + (size_t)i * max_iv * 2;
            const uint32_t n = min(g_niv[i], max_iv);
            const int m0 = find_start(row, n, s_args[i * MSCHED_MAX_ARGS + arg]);
            const uint64_t len = row[2 * m0 + 1];
            uint64_t st = 0, cnt = 1;
            for (uint32_t m = (uint32_t)m0 + 1; m < n; ++m) {
                if (row[2 * m + 1] != len) break;
                bool other = false;
                for (int b = 0; b < n_args; ++b)
                    other |= s_flag[b] && b != arg && s_args[i * MSCHED_MAX_ARGS + b] == row[2 * m];
                if (other) break;
                const uint64_t gap = row[2 * m] - row[2 * (m - 1)];
                if (cnt == 1) st = gap; else if (gap != st) break;
                ++cnt;
            }
            chunk[i] = len; stride[i] = st; count[i] = cnt;
            multi[i] = cnt > 1;
            if (cnt > 1) atomicOr(&s_any_multi, 1u);
        }
        __syncthreads();
        // 3. templates in order
        const bool strided = s_any_multi != 0;
        Fit f_size, f_stride, f_count;
        f_stride.n = f_count.n = 0; f_stride.coeff = f_count.coeff = 0;
        bool ok = fit_search(s_args, n_inv, cand, nc, chunk, all_inv, &s_best, &s_coeff, f_size);
        if (ok && strided) ok = fit_search(s_args, n_inv, cand, nc, stride, multi, &s_best, &s_coeff, f_stride);
        if (ok && strided) ok = fit_search(s_args, n_inv, cand, nc, count, all_inv, &s_best, &s_coeff, f_count);
        if (!ok || s_n_rules == MSCHED_MAX_RULES) { __syncthreads(); continue; }
        if (tid == 0) {
            msched_rule q;
            memset(&q, 0, sizeof q);
            q.kind = strided ? MSCHED_RULE_STRIDED : (f_size.n == 0 ? MSCHED_RULE_FIXED : MSCHED_RULE_LINEAR);
            q.base_arg = (uint8_t)arg;
            q.n_size_args = (uint8_t)f_size.n; q.n_stride_args = (uint8_t)f_stride.n; q.n_count_args = (uint8_t)f_count.n;
            for (int j = 0; j < f_size.n; ++j) q.size_args[j] = (uint8_t)f_size.idx[j];
            for (int j = 0; j < f_stride.n; ++j) q.stride_args[j] = (uint8_t)f_stride.idx[j];
            for (int j = 0; j < f_count.n; ++j) q.count_args[j] = (uint8_t)f_count.idx[j];
            q.size_coeff = f_size.coeff; q.stride_coeff = f_stride.coeff; q.count_coeff = f_count.coeff;
            a.rules[(size_t)k * MSCHED_MAX_RULES + s_n_rules] = q;
        }
        // mark what the rule accounts for
        for (uint32_t i = tid; i < n_inv; i += blockDim.x) {
            const int m0 = find_start(g_iv + (size_t)i * max_iv * 2, min(g_niv[i], max_iv), s_args[i * MSCHED_MAX_ARGS + arg]);
            for (uint64_t j = 0; j < count[i]; ++j) {
                const uint32_t bit = i * max_iv + (uint32_t)m0 + (uint32_t)j;
                const uint32_t old = atomicOr(&covered[bit >> 5], 1u << (bit & 31));
                if (!(old & (1u << (bit & 31)))) atomicAdd(&s_covered, 1u);
            }
        }
        __syncthreads();
        if (tid == 0) s_n_rules += 1;
        __syncthreads();
    }
    if (tid == 0) {
        a.n_rules[k] = s_n_rules;
        a.unexplained[k] = s_total - s_covered;
    }
}

}  // namespace msched

using namespace msched;

extern "C" int msched_analyze(const msched_profile_batch *b, msched_rule *rules, uint32_t *n_rules,
                              uint32_t *unexplained, void *stream) {
    if (!b || !rules || !n_rules || !unexplained) return MSCHED_E_INVAL;
    if (b->n_kernels == 0) return MSCHED_OK;
    if (!b->n_args || !b->int64_mask || !b->args || !b->intervals || !b->n_intervals) return MSCHED_E_INVAL;
    if (b->n_invocations == 0 || b->n_invocations > (uint32_t)kAnaMaxInv || b->max_intervals == 0 ||
        (uint64_t)b->n_invocations * b->max_intervals > kAnaMaxBits)
        return MSCHED_E_INVAL;
    AnaArgs a;
    a.n_inv = b->n_invocations; a.max_iv = b->max_intervals;
    a.n_args = b->n_args; a.int64_mask = b->int64_mask; a.args = b->args; a.iv = b->intervals; a.n_iv = b->n_intervals;
    a.rules = rules; a.n_rules = n_rules; a.unexplained = unexplained;
    const size_t lds = (size_t)a.n_inv * (MSCHED_MAX_ARGS + 3) * 8 + ((size_t)a.n_inv * a.max_iv + 31) / 32 * 4 +
                       2 * (size_t)a.n_inv + 16;
    (void)hipGetLastError();
    hipError_t e = hipSuccess;
    if (lds > 48 * 1024)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_analyze), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) {
        k_analyze<<<b->n_kernels, kAnaThreads, lds, (hipStream_t)stream>>>(a);
        e = hipGetLastError();
    }
    if (e != hipSuccess) { g_last_hip = (int)e; return MSCHED_E_HIP; }
    return MSCHED_OK;
}
