// Gate logits of a token from the K-split partial products of x * Wcat^T (Sec. 3.1: G(x) = x * W_gate).
//
// Wcat's first 3*NP rows hold W_gate split into three bf16 terms (hi | mid | lo, NP columns each), so the
// fp32 logit of adapter `col` is the sum over the K splits, in split order, of (lo + mid) + hi, plus the bias.
// Every kernel that ranks from these partials (forward selection, gate gradients) sums them with this
// routine, so that all of them see bit-identical logits and therefore the same top-k.
#pragma once
#include "common.hpp"

namespace meteora {

// part[S][T][CR]; lane `col` (< N) of G token groups: token t0 + lt[i] (clamped to T-1).  UNR splits'
// loads are in flight at a time (the sum is taken in split order whatever UNR is).  -0 is turned into +0 so that equal logits have equal ranking keys.
template <int NP, int G, int UNR = 4>
__device__ __forceinline__ void dense_logits(const float* __restrict__ part, int S, int CR,
                                             const float* __restrict__ bias, int T, int N, int t0,
                                             const int (&lt)[G], int col, float (&g)[G]) {
#pragma unroll
    for (int i = 0; i < G; ++i) g[i] = 0.f;
    if (col >= N) return;
    for (int s0 = 0; s0 < S; s0 += UNR) {
        float v[UNR][3][G];
#pragma unroll
        for (int u = 0; u < UNR; ++u)
#pragma unroll
            for (int term = 0; term < 3; ++term)
#pragma unroll
                for (int i = 0; i < G; ++i) {
                    const int t = min(t0 + lt[i], T - 1);
                    v[u][term][i] = s0 + u < S ? part[((size_t)(s0 + u) * T + t) * CR + term * NP + col] : 0.f;
                }
#pragma unroll
        for (int u = 0; u < UNR; ++u)
#pragma unroll
            for (int i = 0; i < G; ++i) g[i] += (v[u][2][i] + v[u][1][i]) + v[u][0][i];
    }
    const float b = bias != nullptr ? bias[col] : 0.f;
#pragma unroll
    for (int i = 0; i < G; ++i) {
        g[i] += b;
        if (g[i] == 0.f) g[i] = 0.f;
    }
}

}  // namespace meteora
