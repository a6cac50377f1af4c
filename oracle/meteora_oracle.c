/*
 * CPU oracle for the forward pass of the MeteoRA linear layer.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, double-precision
 * evaluation of the layer's definition, written from the paper, used only to
 * check the GPU library and to time a CPU baseline.  The GPU library shares no
 * code with it and must never call it.
 *
 * What it computes (paper, Sec. 3.1; row-vector convention of Sec. 2, Eq. 1):
 *
 *   G(x)   = x * W_gate (+ bias)                    gating network, R^d -> R^n
 *   I(x)   = the k indices with the largest G_i(x)  top-k selection
 *   w_i    = exp(G_i) / sum_{j in I(x)} exp(G_j)    Eq. 3, softmax over the k
 *                                                   selected logits only
 *   o      = x * W_base + s * sum_{i in I(x)} w_i * ((x * A_i) * B_i)   Eq. 2
 *
 * s is the LoRA scaling alpha/r of Sec. 4.1 (alpha=16, r=8 -> 2); Eq. 2 itself
 * carries no scale, so s=1 is Eq. 2 as printed.
 *
 * Storage (row-major): x[T,d_in], W[d_out,d_in] (so o[t,c] = sum_i x[t,i]*W[c,i]),
 * W_gate[d_in,N], bias[N] or NULL, A[N,d_in,r], B[N,r,d_out] (the two stacked
 * tensors of Sec. 3.3).  Inputs arrive as float: the values the storage dtype
 * (fp32 or bf16) holds, exactly.  Every sum is accumulated in double, in index
 * order, with no blocking and no reordering.
 *
 * Readings where the paper is silent:
 *   - ties in the top-k go to the lower adapter index; I(x) is listed by
 *     descending logit, equal logits by ascending index;
 *   - logits are rounded to fp32 before they are compared and before Eq. 3,
 *     because the layer's gate is defined to produce fp32 logits;
 *   - no intermediate (x*A_i, the LoRA sum) is rounded.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py
 * (hand-worked example, brute-force dense evaluation, invariants, fp64 matmul
 * special cases).  One reading is "parity unpinned": the softmax temperature
 * of App. A.6, for which the paper prints values (15, 20, 30) but no formula.
 * It is read as softmax(g / tau) over the k selected logits; the tests pin
 * the arithmetic of that reading (closed forms), not the reading itself.
 * inv_temperature = 1 is Eq. 3 as printed and is fully pinned.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Row index of the i-th evaluated row: rows[i] if a subset is given, else i. */
static inline int64_t row_of(const int32_t* rows, int64_t i) {
    return rows ? (int64_t)rows[i] : i;
}

/*
 * Gate logits G(x) = x * W_gate (+ bias), Sec. 3.1, in double.
 * logits64[i, j] for the i-th evaluated row.  rows==NULL: all T rows (nrows=T).
 */
void oracle_gate_logits(const float* x, const float* W_gate, const float* bias,
                        int d_in, int N, const int32_t* rows, int nrows,
                        double* logits64) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        const float* xt = x + row_of(rows, i) * (int64_t)d_in;
        for (int j = 0; j < N; ++j) {
            double g = 0.0;
            for (int c = 0; c < d_in; ++c)
                g += (double)xt[c] * (double)W_gate[(int64_t)c * N + j];
            if (bias) g += (double)bias[j];
            logits64[i * N + j] = g;
        }
    }
}

/*
 * Top-k selection I(x) and the normalised weights of Eq. 3, from fp32 logits.
 * idx[i, 0..k) sorted by descending logit, ties by ascending index.
 * w[i, j] = exp(g_j - g_max) / sum over the k selected (double).
 * inv_temperature multiplies the selected logits inside the softmax
 * (1.0 = Eq. 3 as printed; the composite-task temperature of App. A.6 is
 * read as softmax(g / tau), i.e. inv_temperature = 1/tau).
 */
void oracle_topk_softmax(const float* logits32, int nrows, int N, int k,
                         double inv_temperature, int32_t* idx, double* w) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        const float* g = logits32 + i * N;
        int32_t* I = idx + i * k;
        double* wi = w + i * k;
        for (int s = 0; s < k; ++s) {
            int best = -1;
            for (int j = 0; j < N; ++j) {
                int taken = 0;
                for (int q = 0; q < s; ++q) taken |= (I[q] == j);
                if (taken) continue;
                /* strict > keeps the lowest index among equal logits */
                if (best < 0 || g[j] > g[best]) best = j;
            }
            I[s] = best;
        }
        double m = (double)g[I[0]];
        double den = 0.0;
        for (int s = 0; s < k; ++s) {
            wi[s] = exp(((double)g[I[s]] - m) * inv_temperature);
            den += wi[s];
        }
        for (int s = 0; s < k; ++s) wi[s] /= den;
    }
}

/*
 * Per-adapter token sets {x | i in I(x)} of Sec. 3.3 (loop-original's X_i),
 * as index lists: a stable counting sort of the (token, slot) pairs by
 * adapter, visiting tokens in ascending order and slots in ascending order.
 * counts[N], offsets[N+1] (exclusive scan), bucket_tok/bucket_slot[T*k].
 */
void oracle_bucket(const int32_t* idx, int T, int k, int N, int32_t* counts,
                   int32_t* offsets, int32_t* bucket_tok, int32_t* bucket_slot) {
    for (int j = 0; j < N; ++j) counts[j] = 0;
    for (int64_t p = 0; p < (int64_t)T * k; ++p) counts[idx[p]]++;
    offsets[0] = 0;
    for (int j = 0; j < N; ++j) offsets[j + 1] = offsets[j] + counts[j];
    for (int j = 0; j < N; ++j) {
        int32_t pos = offsets[j];
        for (int t = 0; t < T; ++t)
            for (int s = 0; s < k; ++s)
                if (idx[(int64_t)t * k + s] == j) {
                    bucket_tok[pos] = t;
                    bucket_slot[pos] = s;
                    ++pos;
                }
    }
}

/* Base projection o_base = x * W_base (first term of Eq. 1 / Eq. 2). */
void oracle_base(const float* x, const float* W, int d_in, int d_out,
                 const int32_t* rows, int nrows, double* y) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        const float* xt = x + row_of(rows, i) * (int64_t)d_in;
        for (int c = 0; c < d_out; ++c) {
            const float* wc = W + (int64_t)c * d_in;
            double acc = 0.0;
            for (int q = 0; q < d_in; ++q) acc += (double)xt[q] * (double)wc[q];
            y[i * d_out + c] = acc;
        }
    }
}

/*
 * LoRA term of Eq. 2: delta[i,:] = s * sum_{slot} w[i,slot] * ((x_t * A_a) * B_a),
 * a = idx[i,slot].  idx and w are given per evaluated row (the i-th entry
 * belongs to row rows[i]).  h (optional, [nrows,k,r]) receives x_t * A_a.
 */
void oracle_lora_delta(const float* x, const float* A, const float* B,
                       const int32_t* idx, const double* w, int d_in, int d_out,
                       int r, int k, double scale, const int32_t* rows,
                       int nrows, double* delta, double* h) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nrows; ++i) {
        const float* xt = x + row_of(rows, i) * (int64_t)d_in;
        double* dl = delta + i * d_out;
        for (int c = 0; c < d_out; ++c) dl[c] = 0.0;
        for (int s = 0; s < k; ++s) {
            const int a = idx[i * k + s];
            const float* Aa = A + (int64_t)a * d_in * r;
            const float* Ba = B + (int64_t)a * r * d_out;
            double hq[r > 0 ? r : 1];   /* C99 variable-length array: any rank */
            for (int q = 0; q < r; ++q) {
                double acc = 0.0;
                for (int c = 0; c < d_in; ++c)
                    acc += (double)xt[c] * (double)Aa[(int64_t)c * r + q];
                hq[q] = acc;
                if (h) h[(i * k + s) * r + q] = acc;
            }
            for (int c = 0; c < d_out; ++c) {
                double acc = 0.0;
                for (int q = 0; q < r; ++q)
                    acc += hq[q] * (double)Ba[(int64_t)q * d_out + c];
                dl[c] += scale * w[i * k + s] * acc;
            }
        }
    }
}

/*
 * Whole layer on a set of rows (Eq. 2): gate -> fp32 logits -> top-k ->
 * Eq. 3 -> base + LoRA.  Outputs: y[nrows,d_out] double, and the routing
 * (logits32[nrows,N], idx[nrows,k], w[nrows,k]) it used.
 * scratch64 must hold nrows*N doubles; delta must hold nrows*d_out doubles.
 * inv_temperature as in oracle_topk_softmax (1.0 = Eq. 3).
 */
void oracle_linear_forward(const float* x, const float* W, const float* W_gate,
                           const float* bias, const float* A, const float* B,
                           int d_in, int d_out, int N, int r, int k, double scale,
                           double inv_temperature,
                           const int32_t* rows, int nrows, double* y,
                           float* logits32, int32_t* idx, double* w,
                           double* scratch64, double* delta) {
    oracle_gate_logits(x, W_gate, bias, d_in, N, rows, nrows, scratch64);
    for (int64_t p = 0; p < (int64_t)nrows * N; ++p) logits32[p] = (float)scratch64[p];
    oracle_topk_softmax(logits32, nrows, N, k, inv_temperature, idx, w);
    oracle_base(x, W, d_in, d_out, rows, nrows, y);
    oracle_lora_delta(x, A, B, idx, w, d_in, d_out, r, k, scale, rows, nrows, delta, NULL);
    for (int64_t p = 0; p < (int64_t)nrows * d_out; ++p) y[p] += delta[p];
}
