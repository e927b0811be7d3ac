/*
 * analyzer_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * Plain CPU statement of MSched's offline memory analyzer (arXiv 2512.24637, Sec. 5.2 "Memory
 * analyzer"): from the launch arguments and the touched memory regions of a kernel's profiled
 * invocations, derive the access rules (templates T1 fixed / T2 linear / T3 strided) that the online
 * predictor evaluates.  Shares no code with the HIP analyzer.
 *
 * Steps, in the paper's order:
 *   1. scan the argument list for 64-bit values that appear as the beginning address of a touched
 *      region in every invocation: those arguments are base pointers;
 *   2. for each base, take the region that starts there (a run of equal-length intervals at a
 *      regular stride counts as one strided region) and match its extent against the templates in
 *      order: size invariant across all invocations -> T1; otherwise enumerate the remaining
 *      arguments and their products and test linear proportionality with the size (T2) or with the
 *      chunk size, stride and chunk count (T3);
 *   3. on a match record the argument indices and the linear coefficient.
 *
 * Readings where the paper is silent: products of at most three arguments; candidates in order of
 * size then lexicographic index, first match wins (so the constant wins over any product, a single
 * argument over a pair); coefficients are positive integers; a zero product requires a zero value;
 * pointer arguments never enter a product; an argument that equals a lower-indexed base in every
 * invocation is an alias and yields no rule; a strided run stops at an interval of another length,
 * at an irregular gap, or where another base pointer points.
 *
 * Input per kernel: n_inv invocations, each with n_args 64-bit argument values and up to max_iv
 * touched byte intervals (start, length), sorted by start, starts distinct: one per region that a memory
 * instruction of the kernel covers (the profiler instruments every memory instruction and records the
 * addresses it accesses), regions that begin at the same address merged; intervals of different buffers
 * may touch or overlap.
 *
 * Pins: tests/test_oracle_analyzer.py (the paper's vector_add / matrix_mul examples, round trips
 * through an independent rule evaluator, exhaustive first-match search, unexplained regions).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { K_FIXED = 1, K_LINEAR = 2, K_STRIDED = 3 };
enum { MAX_ARGS = 12, MAX_RULES = 8, MAX_PROD = 3 };

typedef struct {          /* one derived rule, field order: size, stride, count */
    int32_t kind, base_arg;
    int32_t n_idx[3];
    int32_t idx[3][4];
    uint64_t coeff[3];
} arule_t;

typedef struct { uint64_t start, len; } iv_t;

typedef struct {
    int n_args, n_inv, max_iv;
    uint32_t ptr_mask;                 /* bit a: argument a is a 64-bit integer (may be a pointer) */
    const uint64_t *args;              /* [n_inv][MAX_ARGS] */
    const iv_t *iv;                    /* [n_inv][max_iv] */
    const uint32_t *n_iv;              /* [n_inv] */
} ktrace_t;

static int find_start(const ktrace_t *k, int i, uint64_t addr) {
    for (uint32_t m = 0; m < k->n_iv[i]; m++)
        if (k->iv[(size_t)i * k->max_iv + m].start == addr) return (int)m;
    return -1;
}

/* value_i = c * product(args_i[S]) for every invocation in `use`; returns 1 and c on success. */
static int fits(const ktrace_t *k, const uint64_t *val, const uint8_t *use, const int *S, int nS, uint64_t *c_out) {
    uint64_t c = 0;
    int have_c = 0;
    for (int pass = 0; pass < 2; pass++) {
        for (int i = 0; i < k->n_inv; i++) {
            if (!use[i]) continue;
            uint64_t prod = 1;
            for (int j = 0; j < nS; j++)
                if (__builtin_mul_overflow(prod, k->args[(size_t)i * MAX_ARGS + S[j]], &prod)) return 0;
            if (pass == 0) {
                if (!have_c && prod != 0) {
                    if (val[i] % prod) return 0;
                    c = val[i] / prod;
                    have_c = 1;
                }
            } else {
                uint64_t want;
                if (__builtin_mul_overflow(c, prod, &want) || want != val[i]) return 0;
            }
        }
        if (pass == 0 && (!have_c || c == 0)) return 0;
    }
    *c_out = c;
    return 1;
}

/* First candidate in the order: {} ; {a} ; {a,b} ; {a,b,c} (indices ascending, non-pointer arguments). */
static int fit_search(const ktrace_t *k, const uint8_t *is_base, const uint64_t *val, const uint8_t *use,
                      int *S_out, int *nS_out, uint64_t *c_out) {
    int cand[MAX_ARGS], nc = 0;
    for (int a = 0; a < k->n_args; a++) if (!is_base[a]) cand[nc++] = a;
    int S[MAX_PROD] = {0};
    if (fits(k, val, use, S, 0, c_out)) { *nS_out = 0; return 1; }
    for (int x = 0; x < nc; x++) {
        S[0] = cand[x];
        if (fits(k, val, use, S, 1, c_out)) { *nS_out = 1; S_out[0] = S[0]; return 1; }
    }
    for (int x = 0; x < nc; x++) for (int y = x + 1; y < nc; y++) {
        S[0] = cand[x]; S[1] = cand[y];
        if (fits(k, val, use, S, 2, c_out)) { *nS_out = 2; S_out[0] = S[0]; S_out[1] = S[1]; return 1; }
    }
    for (int x = 0; x < nc; x++) for (int y = x + 1; y < nc; y++) for (int z = y + 1; z < nc; z++) {
        S[0] = cand[x]; S[1] = cand[y]; S[2] = cand[z];
        if (fits(k, val, use, S, 3, c_out)) { *nS_out = 3; memcpy(S_out, S, sizeof S); return 1; }
    }
    return 0;
}

/* Analyze one kernel.  Writes up to MAX_RULES rules; returns their number.  *unexplained receives the
 * number of (invocation, interval) pairs no rule accounts for. */
int ana_kernel(int n_args, int n_inv, int max_iv, uint32_t ptr_mask, const uint64_t *args, const uint64_t *iv_flat,
               const uint32_t *n_iv, arule_t *rules, uint32_t *unexplained) {
    ktrace_t k = {n_args, n_inv, max_iv, ptr_mask, args, (const iv_t *)iv_flat, n_iv};
    uint8_t is_base[MAX_ARGS] = {0};
    /* 1. base pointers: 64-bit arguments whose value starts a touched interval in every invocation */
    for (int a = 0; a < n_args; a++) {
        if (!((ptr_mask >> a) & 1) || n_inv == 0) continue;
        int ok = 1;
        for (int i = 0; i < n_inv && ok; i++) ok = find_start(&k, i, args[(size_t)i * MAX_ARGS + a]) >= 0;
        is_base[a] = (uint8_t)ok;
    }
    uint8_t *covered = (uint8_t *)calloc((size_t)n_inv * max_iv + 1, 1);
    uint64_t *chunk = (uint64_t *)malloc(sizeof(uint64_t) * (n_inv + 1));
    uint64_t *stride = (uint64_t *)malloc(sizeof(uint64_t) * (n_inv + 1));
    uint64_t *count = (uint64_t *)malloc(sizeof(uint64_t) * (n_inv + 1));
    uint8_t *all_inv = (uint8_t *)malloc(n_inv + 1), *multi = (uint8_t *)malloc(n_inv + 1);
    int n_rules = 0;
    for (int a = 0; a < n_args; a++) {
        if (!is_base[a]) continue;
        int alias = 0;                                       /* same address as a lower base, every time */
        for (int b = 0; b < a && !alias; b++) {
            if (!is_base[b]) continue;
            int same = 1;
            for (int i = 0; i < n_inv && same; i++) same = args[(size_t)i * MAX_ARGS + a] == args[(size_t)i * MAX_ARGS + b];
            alias = same;
        }
        if (alias) continue;
        /* 2. the region that starts at this base, per invocation */
        int any_multi = 0;
        for (int i = 0; i < n_inv; i++) {
            const iv_t *row = k.iv + (size_t)i * max_iv;
            int m0 = find_start(&k, i, args[(size_t)i * MAX_ARGS + a]);
            chunk[i] = row[m0].len; stride[i] = 0; count[i] = 1;
            for (uint32_t m = (uint32_t)m0 + 1; m < n_iv[i]; m++) {
                if (row[m].len != chunk[i]) break;
                int other_base = 0;
                for (int b = 0; b < n_args; b++)
                    if (is_base[b] && b != a && args[(size_t)i * MAX_ARGS + b] == row[m].start) other_base = 1;
                if (other_base) break;
                uint64_t gap = row[m].start - row[m - 1].start;
                if (count[i] == 1) stride[i] = gap; else if (gap != stride[i]) break;
                count[i]++;
            }
            all_inv[i] = 1; multi[i] = count[i] > 1;
            any_multi |= multi[i];
        }
        /* 3. match the extent against the templates in order */
        arule_t r; memset(&r, 0, sizeof r);
        r.base_arg = a;
        int ok;
        if (!any_multi) {
            ok = fit_search(&k, is_base, chunk, all_inv, r.idx[0], &r.n_idx[0], &r.coeff[0]);
            r.kind = r.n_idx[0] == 0 ? K_FIXED : K_LINEAR;
        } else {
            r.kind = K_STRIDED;
            ok = fit_search(&k, is_base, chunk, all_inv, r.idx[0], &r.n_idx[0], &r.coeff[0]) &&
                 fit_search(&k, is_base, stride, multi, r.idx[1], &r.n_idx[1], &r.coeff[1]) &&
                 fit_search(&k, is_base, count, all_inv, r.idx[2], &r.n_idx[2], &r.coeff[2]);
        }
        if (!ok || n_rules == MAX_RULES) continue;
        rules[n_rules++] = r;
        for (int i = 0; i < n_inv; i++) {
            int m0 = find_start(&k, i, args[(size_t)i * MAX_ARGS + a]);
            for (uint64_t j = 0; j < count[i]; j++) covered[(size_t)i * max_iv + m0 + j] = 1;
        }
    }
    uint32_t un = 0;
    for (int i = 0; i < n_inv; i++)
        for (uint32_t m = 0; m < n_iv[i]; m++) un += !covered[(size_t)i * max_iv + m];
    *unexplained = un;
    free(covered); free(chunk); free(stride); free(count); free(all_inv); free(multi);
    return n_rules;
}

/* A batch of kernels with uniform shapes: args [K][n_inv][12], iv [K][n_inv][max_iv][2], n_iv [K][n_inv]. */
void ana_batch(int n_kernels, const int32_t *n_args, int n_inv, int max_iv, const uint32_t *ptr_mask,
               const uint64_t *args, const uint64_t *iv, const uint32_t *n_iv,
               arule_t *rules /* [K][8] */, int32_t *n_rules, uint32_t *unexplained) {
    for (int k = 0; k < n_kernels; k++)
        n_rules[k] = ana_kernel(n_args[k], n_inv, max_iv, ptr_mask[k], args + (size_t)k * n_inv * MAX_ARGS,
                                iv + (size_t)k * n_inv * max_iv * 2, n_iv + (size_t)k * n_inv,
                                rules + (size_t)k * MAX_RULES, &unexplained[k]);
}
