// Grouped LoRA expand (second product and weighted sum of Eq. 2 / Eq. 5):
//   out[t,:] (+)= scale * sum_slot w[t,slot] * h[t,slot,:] * B_a,   a = I(t)_slot.
//
// A workgroup owns whole output rows, so every output element has exactly one writer:
// no atomics, and the k contributions of a token are added in slot order (deterministic).
#include "common.hpp"
#include "kernels.hpp"

namespace meteora {

// Plain-FMA version: one workgroup per token, threads stride over d_out.
template <typename TX>
__global__ __launch_bounds__(256) void expand_fma_kernel(const float* __restrict__ h32, const TX* __restrict__ B,
                                                         const int32_t* __restrict__ topk_idx,
                                                         const float* __restrict__ topk_w, int d_out, int N,
                                                         int r, int k, float scale, TX* __restrict__ out,
                                                         int accumulate) {
    __shared__ float hs[kMaxTopK * kMaxRank];   // scale * w * h for the k slots
    __shared__ int as[kMaxTopK];
    const int t = blockIdx.x;
    for (int i = threadIdx.x; i < k * r; i += 256) {
        const int slot = i / r;
        hs[i] = scale * topk_w[(size_t)t * k + slot] * h32[(size_t)t * k * r + i];
    }
    if (threadIdx.x < k) {
        const int a = topk_idx[(size_t)t * k + threadIdx.x];
        as[threadIdx.x] = (a >= 0 && a < N) ? a : -1;
    }
    __syncthreads();
    for (int c = threadIdx.x; c < d_out; c += 256) {
        float acc = accumulate ? to_float(out[(size_t)t * d_out + c]) : 0.f;
        for (int slot = 0; slot < k; ++slot) {
            const int a = as[slot];
            if (a < 0) continue;
            const TX* Ba = B + (size_t)a * r * d_out + c;
            float d = 0.f;
            for (int q = 0; q < r; ++q) d = fmaf(hs[slot * r + q], to_float(Ba[(size_t)q * d_out]), d);
            acc += d;
        }
        out[(size_t)t * d_out + c] = from_float<TX>(acc);
    }
}

hipError_t launch_expand(const float* h32, const void* B, const int32_t* topk_idx, const float* topk_w,
                         int T, int d_out, int N, int r, int k, float scale, bool bf16, void* out,
                         int accumulate, hipStream_t stream) {
    if (bf16)
        expand_fma_kernel<bf16_t><<<T, 256, 0, stream>>>(h32, (const bf16_t*)B, topk_idx, topk_w, d_out, N, r, k,
                                                         scale, (bf16_t*)out, accumulate);
    else
        expand_fma_kernel<float><<<T, 256, 0, stream>>>(h32, (const float*)B, topk_idx, topk_w, d_out, N, r, k,
                                                        scale, (float*)out, accumulate);
    return hipGetLastError();
}

}  // namespace meteora
