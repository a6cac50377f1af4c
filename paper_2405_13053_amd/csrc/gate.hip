// Gate network and top-k routing of the MeteoRA layer (paper Sec. 3.1):
//   G(x) = x * W_gate (+ bias), I(x) = top-k of G(x), w = softmax over the k selected (Eq. 3).
//
// Two stages:
//   1. logit partial sums  partials[ks][t][j] = sum_{i in K-slice ks} x[t,i] * W_gate[i,j]
//   2. per token, one wavefront: sum the K-slices in a fixed order, add the bias, select the
//      top-k with a wavefront-wide arg-max (ties -> lowest adapter index), softmax over the k.
#include "common.hpp"
#include "kernels.hpp"

namespace meteora {

// ------------------------------------------------------------------------------------------
// Stage 1, plain-FMA version (fp32 inputs, or shapes the MFMA version does not take).
// One workgroup per token; wave w sums the w-th quarter of d_in; lane j owns adapter j.
// ------------------------------------------------------------------------------------------
template <typename TX>
__global__ __launch_bounds__(256) void gate_logits_fma_kernel(const TX* __restrict__ x,
                                                              const float* __restrict__ W_gate,
                                                              int T, int d_in, int N, int NP,
                                                              float* __restrict__ partials) {
    __shared__ float red[4][kMaxAdapters];
    const int t = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int per = ceil_div(d_in, 4);
    const int i0 = wave * per, i1 = min(d_in, i0 + per);
    const TX* xt = x + (size_t)t * d_in;
    float acc = 0.f;
    if (lane < N) {
        for (int i = i0; i < i1; ++i) acc = fmaf(to_float(xt[i]), W_gate[(size_t)i * N + lane], acc);
    }
    red[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && lane < NP) {
        float s = (lane < N) ? ((red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane])) : 0.f;
        partials[(size_t)t * NP + lane] = s;
    }
}

// ------------------------------------------------------------------------------------------
// Stage 2: one wavefront per token.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void argmax_step(float& v, int& i, int offset) {
    const float v2 = __shfl_xor(v, offset);
    const int i2 = __shfl_xor(i, offset);
    // candidates that are out of play carry i = INT_MAX and lose every comparison
    const bool take = (i2 != 0x7fffffff) && (i == 0x7fffffff || v2 > v || (v2 == v && i2 < i));
    if (take) { v = v2; i = i2; }
}

constexpr int kTopkTokensPerWave = 4;

__global__ __launch_bounds__(256) void gate_topk_kernel(const float* __restrict__ partials, int KS,
                                                        const float* __restrict__ bias, int T, int N,
                                                        int NP, int k, float inv_temperature,
                                                        int32_t* __restrict__ topk_idx,
                                                        float* __restrict__ topk_w,
                                                        float* __restrict__ logits) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = (blockIdx.x * 4 + wave) * kTopkTokensPerWave;
    const float b = (bias != nullptr && lane < N) ? bias[lane] : 0.f;
    for (int tt = 0; tt < kTopkTokensPerWave; ++tt) {
        const int t = t0 + tt;
        if (t >= T) return;   // uniform per wave
        float g = 0.f;
        if (lane < N) {
            for (int s = 0; s < KS; ++s) g += partials[((size_t)s * T + t) * NP + lane];
            g += b;
            if (logits) logits[(size_t)t * N + lane] = g;
        }
        bool live = lane < N;
        float sel_g = 0.f;   // lane s < k keeps the s-th selected logit
        int sel_i = 0;
        for (int s = 0; s < k; ++s) {
            float v = g;
            int i = live ? lane : 0x7fffffff;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) argmax_step(v, i, off);
            if (lane == i) live = false;
            if (lane == s) { sel_g = v; sel_i = i; }
        }
        const float gmax = __shfl(sel_g, 0);
        float e = (lane < k) ? expf((sel_g - gmax) * inv_temperature) : 0.f;
        float sum = e;
#pragma unroll
        for (int off = 1; off < kMaxTopK; off <<= 1) sum += __shfl_xor(sum, off);
        if (lane < k) {
            topk_idx[(size_t)t * k + lane] = sel_i;
            topk_w[(size_t)t * k + lane] = e / sum;
        }
    }
}

int gate_kslices(int d_in, bool bf16) {
    (void)d_in; (void)bf16;
    return 1;
}

size_t gate_wsplit_bytes(int d_in, int N, bool bf16) {
    (void)d_in; (void)N; (void)bf16;
    return 0;
}

hipError_t launch_gate_logits(const void* x, const float* W_gate, int T, int d_in, int N, bool bf16,
                              void* wsplit, float* partials, hipStream_t stream) {
    (void)wsplit;
    const int NP = padded_adapters(N);
    if (bf16)
        gate_logits_fma_kernel<bf16_t><<<T, 256, 0, stream>>>((const bf16_t*)x, W_gate, T, d_in, N, NP, partials);
    else
        gate_logits_fma_kernel<float><<<T, 256, 0, stream>>>((const float*)x, W_gate, T, d_in, N, NP, partials);
    return hipGetLastError();
}

hipError_t launch_gate_topk(const float* partials, int KS, const float* bias, int T, int N, int k,
                            float inv_temperature, int32_t* topk_idx, float* topk_w, float* logits,
                            hipStream_t stream) {
    const int NP = padded_adapters(N);
    const int tokens_per_block = 4 * kTopkTokensPerWave;
    gate_topk_kernel<<<ceil_div(T, tokens_per_block), 256, 0, stream>>>(partials, KS, bias, T, N, NP, k,
                                                                        inv_temperature, topk_idx, topk_w,
                                                                        logits);
    return hipGetLastError();
}

}  // namespace meteora
