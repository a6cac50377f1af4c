// Base projection of the layer, first term of Eq. 1 / Eq. 2:  out = x * W_base, with W stored
// [d_out, d_in] so both operands are contiguous along the contraction.
#include "common.hpp"
#include "gemm_mfma.hpp"
#include "kernels.hpp"

namespace meteora {

// ------------------------------------------------------------------------------------------
// Plain-FMA version (fp32 inputs and shapes the MFMA version does not take): 64x64 output tile,
// K step 16, each of 256 threads owns a 4x4 block, fp32 accumulation.
// ------------------------------------------------------------------------------------------
template <typename TX>
__global__ __launch_bounds__(256) void gemm_fma_kernel(const TX* __restrict__ x, const TX* __restrict__ W, int T,
                                                       int d_in, int d_out, TX* __restrict__ out, int accumulate) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float xs[BK][BM + 4];
    __shared__ float ws[BK][BN + 4];
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    float acc[4][4] = {};
    const int lr = threadIdx.x / 4;         // 0..63: row of the tile this thread loads
    const int lk = (threadIdx.x % 4) * 4;   // 0,4,8,12: first of its 4 k values
    for (int k0 = 0; k0 < d_in; k0 += BK) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int kk = k0 + lk + j;
            const int m = m0 + lr, n = n0 + lr;
            xs[lk + j][lr] = (m < T && kk < d_in) ? to_float(x[(size_t)m * d_in + kk]) : 0.f;
            ws[lk + j][lr] = (n < d_out && kk < d_in) ? to_float(W[(size_t)n * d_in + kk]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = xs[kk][ty * 4 + i]; b[i] = ws[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= T) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= d_out) continue;
            float v = acc[i][j];
            if (accumulate) v += to_float(out[(size_t)m * d_out + n]);
            out[(size_t)m * d_out + n] = from_float<TX>(v);
        }
    }
}

template <int MI, int NI>
static hipError_t launch_mfma(GemmArgs a, hipStream_t stream) {
    constexpr int BM = MI * 64, BN = NI * 64;
    constexpr int smem = 2 * (BM + BN) * kGemmBK * (int)sizeof(bf16_t);
    static bool attr_set = false;   // raising the dynamic-LDS limit is a host-side attribute, set once
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_kernel<MI, NI>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_dma_kernel<MI, NI>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    a.tiles_m = ceil_div(a.T, BM);
    a.tiles_n = ceil_div(a.d_out, BN);
    // the pipelined kernel needs whole K tiles and byte offsets inside x and W that fit 32 bits
    const bool dma_ok = a.d_in % kGemmBK == 0 && (a.ext_k == 0 || a.ext_stride % kGemmBK == 0) &&
                        (uint64_t)a.T * a.d_in * 2 < (1ull << 32) && (uint64_t)a.d_out * a.d_in * 2 < (1ull << 32);
    if (dma_ok)
        gemm_mfma_dma_kernel<MI, NI><<<a.tiles_m * a.tiles_n, 256, smem, stream>>>(a);
    else
        gemm_mfma_kernel<MI, NI><<<a.tiles_m * a.tiles_n, 256, smem, stream>>>(a);
    return hipGetLastError();
}

bool gemm_fuses_expand(bool bf16) { return bf16; }

hipError_t launch_gemm(const void* x, const void* W, int T, int d_in, int d_out, bool bf16,
                       const void* hdense, int ext_stride, const void* B, int ext_k,
                       void* out, int accumulate, hipStream_t stream) {
    if (bf16) {
        GemmArgs a{};
        a.x = (const bf16_t*)x; a.W = (const bf16_t*)W; a.hd = (const bf16_t*)hdense; a.Bst = (const bf16_t*)B;
        a.out = (bf16_t*)out; a.T = T; a.d_in = d_in; a.d_out = d_out;
        a.ext_k = hdense ? ext_k : 0; a.ext_stride = ext_stride; a.accumulate = accumulate;
        const int64_t big_tiles = (int64_t)ceil_div(T, 256) * ceil_div(d_out, 256);
        if (T > 128 && big_tiles >= 128) return launch_mfma<4, 4>(a, stream);
        if (T > 64) return launch_mfma<2, 2>(a, stream);
        return launch_mfma<1, 1>(a, stream);
    }
    dim3 grid(ceil_div(d_out, 64), ceil_div(T, 64));
    gemm_fma_kernel<float><<<grid, 256, 0, stream>>>((const float*)x, (const float*)W, T, d_in, d_out,
                                                     (float*)out, accumulate);
    return hipGetLastError();
}

}  // namespace meteora
