/* CPU oracle for the SP-MoE hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library is checked against.  Only the
 * test-suite, the smoke check and the benchmark's "cpu_baseline" leg may call it; the product
 * path never does.  It shares no code, header, table or helper with the GPU library.
 *
 * What it computes (paper, "Expert Offloading in MoE Inference", Eq. 1):
 *     Output(x) = sum_{i=1..k} G(x)_i * E_i(x)
 * where the gating network scores all experts of the layer, the top-k of them are the token's
 * critical experts, G(x)_i is the gating score of the i-th selected expert and E_i its FFN.
 * Prefetching and caching (Alg. 1, Alg. 2) only change where weights live, never this result, so
 * the oracle is Eq. 1 written out, one token and one expert at a time, with no blocking, fusion
 * or reordering.
 *
 * Readings where the paper is silent (each is listed in the design notes of this repository):
 *   - G(x): softmax over all E gate logits, top-k chosen on the logits (softmax is monotone),
 *     selected probabilities renormalised to sum 1 when `renorm` is set.
 *   - ties: the lower expert index wins; selected experts are kept in descending-score order.
 *   - E_i(x): three-matrix SwiGLU FFN without biases,
 *         E(x) = W_down * ( silu(W_gate x) .* (W_up x) ),   silu(z) = z / (1 + exp(-z)).
 *     (3*d*f 16-bit values reproduce the 336 MB / 150 MB / 16.5 MB expert sizes the paper quotes.)
 *   - shared experts (the DeepSeek-style "two shared experts" of the paper's background section)
 *     are added to every token with weight 1, outside the renormalised routed sum.
 *
 * Precision: every quantity is held in `real`, float by default (the fp32 oracle) or double when
 * built with -DORACLE_REAL=double (used to bound the fp32 oracle's own rounding error).  Sums run
 * in ascending index order.  bf16 weights are upcast exactly; inputs x are fp32.
 *
 * Parity pins (tests/test_oracle_*.py): brute-force stable-sort routing on tiny inputs, constructed
 * ties, sum of weights = 1, E=1/k=1 equals a dense SwiGLU FFN evaluated by a library matmul in
 * fp64, identical experts give the dense FFN whatever the routing, linearity in W_down, token-order
 * equivariance, closed-form values (silu(1), two-expert softmax), float-vs-double agreement.
 * End-to-end latency and hit-rate figures of the paper's evaluation depend on its datasets and
 * trained weights: parity unpinned for those (nothing here claims them).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORACLE_REAL
#define ORACLE_REAL float
#endif
typedef ORACLE_REAL real;

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

int oracle_real_bytes(void) { return (int)sizeof(real); }

/* weight element i of a buffer of the given storage type, upcast exactly */
static inline real wload(const void* w, size_t i, int dtype) {
    if (dtype == ORACLE_BF16) {
        uint32_t u = (uint32_t)((const uint16_t*)w)[i] << 16;
        float f;
        memcpy(&f, &u, 4);
        return (real)f;
    }
    return (real)((const float*)w)[i];
}

static inline real real_exp(real z) { return sizeof(real) == 4 ? (real)expf((float)z) : (real)exp((double)z); }

/* dot product of fp32 vector x[0..n) with row `row` of a row-major [rows][n] weight matrix */
static real dot_row(const float* x, const void* w, size_t row, size_t n, int dtype) {
    real acc = 0;
    for (size_t j = 0; j < n; ++j) acc += (real)x[j] * wload(w, row * n + j, dtype);
    return acc;
}

/* Gate network: logits[t][e] = sum_j x[t][j] * Wg[e][j].   (Alg. 1: expert_scores <- Gates[l](s)) */
void oracle_gate_logits(const float* x, const void* wg, int wdtype, int T, int E, int d, real* logits) {
    for (int t = 0; t < T; ++t)
        for (int e = 0; e < E; ++e)
            logits[(size_t)t * E + e] = dot_row(x + (size_t)t * d, wg, (size_t)e, (size_t)d, wdtype);
}

/* p = softmax(logits) over E experts, with the usual max subtraction */
void oracle_softmax(const real* logits, int E, real* p) {
    real m = logits[0];
    for (int e = 1; e < E; ++e) if (logits[e] > m) m = logits[e];
    real sum = 0;
    for (int e = 0; e < E; ++e) { p[e] = real_exp(logits[e] - m); sum += p[e]; }
    for (int e = 0; e < E; ++e) p[e] = p[e] / sum;
}

/* TopK_Index (Alg. 1): the k largest scores, descending; among equal scores the lower index first. */
void oracle_topk(const real* scores, int E, int k, int32_t* idx) {
    unsigned char* taken = (unsigned char*)calloc((size_t)E, 1);
    for (int r = 0; r < k; ++r) {
        int best = -1;
        for (int e = 0; e < E; ++e) {
            if (taken[e]) continue;
            if (best < 0 || scores[e] > scores[best]) best = e;   /* strict >: first (lowest) index keeps a tie */
        }
        taken[best] = 1;
        idx[r] = best;
    }
    free(taken);
}

/* Routing of T tokens from their logits: idx[t][r] (rank order) and gating scores w[t][r] = G(x_t)_r. */
void oracle_route(const real* logits, int T, int E, int k, int renorm, int32_t* idx, real* w) {
    real* p = (real*)malloc(sizeof(real) * (size_t)E);
    for (int t = 0; t < T; ++t) {
        const real* lg = logits + (size_t)t * E;
        oracle_softmax(lg, E, p);
        oracle_topk(lg, E, k, idx + (size_t)t * k);
        real s = 0;
        for (int r = 0; r < k; ++r) s += p[idx[(size_t)t * k + r]];
        for (int r = 0; r < k; ++r) {
            real pr = p[idx[(size_t)t * k + r]];
            w[(size_t)t * k + r] = renorm ? pr / s : pr;
        }
    }
    free(p);
}

/* Token -> expert grouping: assignments a = t*k + r listed expert by expert, inside one expert by
 * ascending a.  counts[E], offsets[E+1] (exclusive prefix sum), perm[T*k]. */
void oracle_permute(const int32_t* idx, int T, int k, int E, int32_t* counts, int32_t* offsets, int32_t* perm) {
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int a = 0; a < T * k; ++a) counts[idx[a]] += 1;
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
    int pos = 0;
    for (int e = 0; e < E; ++e)
        for (int a = 0; a < T * k; ++a)
            if (idx[a] == e) perm[pos++] = a;
}

/* One expert on one token: y = W_down * ( silu(W_gate x) .* (W_up x) ).
 * W_gate, W_up: [f][d] row-major; W_down: [d][f] row-major. */
void oracle_expert_ffn(const float* x, const void* w_gate, const void* w_up, const void* w_down,
                       int wdtype, int d, int f, real* y) {
    real* h = (real*)malloc(sizeof(real) * (size_t)f);
    #pragma omp parallel for schedule(static)
    for (int n = 0; n < f; ++n) {
        real g = dot_row(x, w_gate, (size_t)n, (size_t)d, wdtype);
        real u = dot_row(x, w_up, (size_t)n, (size_t)d, wdtype);
        real silu = g / ((real)1 + real_exp(-g));
        h[n] = silu * u;
    }
    #pragma omp parallel for schedule(static)
    for (int i = 0; i < d; ++i) {
        real acc = 0;
        for (int n = 0; n < f; ++n) acc += h[n] * wload(w_down, (size_t)i * f + n, wdtype);
        y[i] = acc;
    }
    free(h);
}

/* The MoE block of one layer on a batch of T tokens (Eq. 1), plus optional shared experts.
 *   x[T][d] fp32; wg[E][d]; expert e = (w_gate[e], w_up[e], w_down[e]); shared expert s likewise.
 *   out[T][d]; idx[T][k]; w[T][k]; logits[T][E] are all written.
 * Combination order: routed experts in rank order r = 0..k-1, then shared experts in index order. */
void oracle_moe_layer(const float* x, int T, int d, int f, int E, int k, int n_shared, int renorm,
                      int wdtype, const void* wg,
                      const void* const* w_gate, const void* const* w_up, const void* const* w_down,
                      const void* const* s_gate, const void* const* s_up, const void* const* s_down,
                      real* out, int32_t* idx, real* w, real* logits) {
    oracle_gate_logits(x, wg, wdtype, T, E, d, logits);
    oracle_route(logits, T, E, k, renorm, idx, w);
    real* y = (real*)malloc(sizeof(real) * (size_t)d);
    for (int t = 0; t < T; ++t) {
        const float* xt = x + (size_t)t * d;
        real* ot = out + (size_t)t * d;
        for (int i = 0; i < d; ++i) ot[i] = 0;
        for (int r = 0; r < k; ++r) {
            int e = idx[(size_t)t * k + r];
            oracle_expert_ffn(xt, w_gate[e], w_up[e], w_down[e], wdtype, d, f, y);
            real g = w[(size_t)t * k + r];
            for (int i = 0; i < d; ++i) ot[i] += g * y[i];
        }
        for (int s = 0; s < n_shared; ++s) {
            oracle_expert_ffn(xt, s_gate[s], s_up[s], s_down[s], wdtype, d, f, y);
            for (int i = 0; i < d; ++i) ot[i] += y[i];
        }
    }
    free(y);
}
