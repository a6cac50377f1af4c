// Wavefront top-k of the gate (Sec. 3.1: I(x) = top-k of G(x), ties to the lowest index) and the softmax over
// the k selected logits (Eq. 3), shared by the routing kernels so that every path ranks identically.
//
// A logit and its adapter index are packed into one 64-bit key, (order-preserving bits of the fp32 value)
// << 32 | (0xffffffff - index): the maximum of the keys is the largest logit, and among equal logits the
// lowest index.
#pragma once
#include "common.hpp"

namespace meteora {

__device__ __forceinline__ uint64_t logit_key(float g, int index) {
    uint32_t u = __float_as_uint(g);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);   // monotonic map of finite floats to unsigned; -0 < +0 never ties with an index swap
    return ((uint64_t)u << 32) | (uint64_t)(0xffffffffu - (uint32_t)index);
}
__device__ __forceinline__ float key_logit(uint64_t key) {
    uint32_t u = (uint32_t)(key >> 32);
    u = (u & 0x80000000u) ? (u & 0x7fffffffu) : ~u;
    return __uint_as_float(u);
}

// A token's NP (32 or 64) logit columns sit in NP adjacent lanes (col = lane % NP), so a wavefront ranks
// 64/NP tokens per group and G interleaved groups (their shuffle latencies overlap).  g[i] is this lane's
// logit of group i (lanes col >= N are padding; -0 must already be +0).  Selecting k adapters is k butterfly
// maxima over the NP lanes; lanes that are padding or already selected carry key 0 and can never win.
// On return lane col = s < k of each token holds its s-th choice: sel_i[i] = adapter, sel_w[i] = Eq. 3 weight.
template <int NP, int G>
__device__ __forceinline__ void wave_topk_softmax(const float (&g)[G], int lane, int N, int k, float inv_temperature,
                                                  int (&sel_i)[G], float (&sel_w)[G]) {
    const int col = lane & (NP - 1);
    uint64_t key[G];
    float sel_g[G];
#pragma unroll
    for (int i = 0; i < G; ++i) { key[i] = col < N ? logit_key(g[i], col) : 0ull; sel_g[i] = 0.f; sel_i[i] = 0; }
    for (int s = 0; s < k; ++s) {
        uint64_t best[G];
#pragma unroll
        for (int i = 0; i < G; ++i) best[i] = key[i];
#pragma unroll
        for (int off = NP / 2; off >= 1; off >>= 1) {
#pragma unroll
            for (int i = 0; i < G; ++i) {
                const uint64_t o = __shfl_xor((unsigned long long)best[i], off);
                best[i] = o > best[i] ? o : best[i];
            }
        }
#pragma unroll
        for (int i = 0; i < G; ++i) {
            const int win = (int)(0xffffffffu - (uint32_t)best[i]);
            if (col == win) key[i] = 0ull;
            if (col == s) { sel_g[i] = key_logit(best[i]); sel_i[i] = win; }
        }
    }
    if (k == 1) {
        // Top-1 strategy (App. A.1): the softmax over a single logit is exactly 1 whatever the logit and the
        // temperature, so neither the exponential nor the normalising sum is evaluated
#pragma unroll
        for (int i = 0; i < G; ++i) sel_w[i] = col == 0 ? 1.f : 0.f;
        return;
    }
#pragma unroll
    for (int i = 0; i < G; ++i) {
        const float gmax = __shfl(sel_g[i], lane & ~(NP - 1));
        const float e = (col < k) ? expf((sel_g[i] - gmax) * inv_temperature) : 0.f;
        float sum = e;
#pragma unroll
        for (int off = 1; off < kMaxTopK; off <<= 1) sum += __shfl_xor(sum, off);
        sel_w[i] = e / sum;
    }
}

}  // namespace meteora
