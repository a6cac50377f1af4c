// Grouped LoRA shrink (first product of Eq. 2):  h[t,slot,:] = x[t,:] * A_a,  a = I(t)_slot.
//
// Work is grouped by adapter through the bucket lists: a tile is a run of pairs that share one
// adapter, so A_a is fetched once per tile and the gathered token rows stream past it.
#include "common.hpp"
#include "kernels.hpp"

namespace meteora {

// ------------------------------------------------------------------------------------------
// Plain-FMA version (fp32 inputs, ranks other than 8/16, odd shapes).  One workgroup per
// (token, slot) pair in bucket order; thread (part, q) sums a stripe of d_in for rank column q.
// ------------------------------------------------------------------------------------------
template <typename TX>
__global__ __launch_bounds__(256) void shrink_fma_kernel(const TX* __restrict__ x, const TX* __restrict__ A,
                                                         const int32_t* __restrict__ topk_idx,
                                                         const float* __restrict__ topk_w,
                                                         const int32_t* __restrict__ bucket_tok,
                                                         const int32_t* __restrict__ bucket_slot,
                                                         int T, int d_in, int N, int r, int RP, int k, float scale,
                                                         float* __restrict__ h32, bf16_t* __restrict__ hdense,
                                                         int ext_stride) {
    __shared__ float red[256];
    const int pos = blockIdx.x;
    const int t = bucket_tok[pos], slot = bucket_slot[pos];
    if (t < 0 || t >= T || slot < 0 || slot >= k) return;   // uniform per workgroup; malformed lists are skipped
    const int a = topk_idx[(size_t)t * k + slot];
    if (a < 0 || a >= N) return;
    const int q = threadIdx.x % RP, part = threadIdx.x / RP, parts = 256 / RP;
    const TX* xt = x + (size_t)t * d_in;
    const TX* Aa = A + (size_t)a * d_in * r;
    float acc = 0.f;
    if (q < r)
        for (int i = part; i < d_in; i += parts) acc = fmaf(to_float(xt[i]), to_float(Aa[(size_t)i * r + q]), acc);
    red[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x < r) {
        float s = 0.f;
        for (int p = 0; p < parts; ++p) s += red[p * RP + threadIdx.x];
        if (h32) h32[((size_t)t * k + slot) * r + threadIdx.x] = s;
        if (hdense) {
            const float w = topk_w[(size_t)t * k + slot];
            hdense[(size_t)t * ext_stride + a * r + threadIdx.x] = from_float<bf16_t>(scale * w * s);
        }
    }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(u32x4* __restrict__ p, size_t n16) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) p[i] = u32x4{0u, 0u, 0u, 0u};
}

hipError_t launch_shrink(const void* x, const void* A, const int32_t* topk_idx, const float* topk_w,
                         const int32_t* offsets, const int32_t* bucket_tok, const int32_t* bucket_slot,
                         int T, int d_in, int N, int r, int k, float scale, bool bf16,
                         float* h32, void* hdense, int ext_stride, hipStream_t stream) {
    (void)offsets;
    int RP = 1;
    while (RP < r) RP <<= 1;
    const int64_t pairs = (int64_t)T * k;
    if (hdense) {   // columns of adapters a token did not select must read as zero
        const size_t n16 = (size_t)T * ext_stride * sizeof(bf16_t) / 16;
        fill_zero_kernel<<<(unsigned)ceil_div64((int64_t)n16, 256), 256, 0, stream>>>((u32x4*)hdense, n16);
    }
    if (bf16)
        shrink_fma_kernel<bf16_t><<<(unsigned)pairs, 256, 0, stream>>>(
            (const bf16_t*)x, (const bf16_t*)A, topk_idx, topk_w, bucket_tok, bucket_slot, T, d_in, N, r, RP, k,
            scale, h32, (bf16_t*)hdense, ext_stride);
    else
        shrink_fma_kernel<float><<<(unsigned)pairs, 256, 0, stream>>>(
            (const float*)x, (const float*)A, topk_idx, topk_w, bucket_tok, bucket_slot, T, d_in, N, r, RP, k,
            scale, h32, (bf16_t*)hdense, ext_stride);
    return hipGetLastError();
}

}  // namespace meteora
