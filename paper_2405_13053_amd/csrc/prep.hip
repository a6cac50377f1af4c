// Per-call repacking of the small weight operands into MFMA fragment order (see prep.hpp):
//   - W_gate (fp32) -> three bf16 terms hi + mid + lo that add up to the fp32 value exactly
//     (8 + 8 + 8 significand bits), so that bf16 MFMAs reproduce fp32-level gate logits;
//   - stacked LoRA A[N, d_in, r] (Sec. 3.3) -> fragments with the rank padded to 32 columns.
// Both run in ONE launch (disjoint workgroup ranges); a wavefront writes one fragment.
#include "common.hpp"
#include "kernels.hpp"
#include "prep.hpp"

namespace meteora {

// fragment (ks, wq, s, cb): blocks ((((ks*4+wq)*8+s)*3 + term)*NCB + cb); lane l holds
// k = ks*512 + wq*128 + s*16 + (l>>5)*8 + j of column n = cb*32 + (l&31).
__device__ __forceinline__ void wsplit_fragment(const float* __restrict__ W_gate, int d_in, int N, int NCB,
                                                int frag, int lane, u32x4* __restrict__ wsp) {
    const int cb = frag % NCB;
    const int s = (frag / NCB) % 8;
    const int wq = (frag / (NCB * 8)) % 4;
    const int ks = frag / (NCB * 32);
    const int n = cb * 32 + (lane & 31);
    const int k0 = ks * kSkinnyKSL + wq * kSkinnyKW + s * 16 + (lane >> 5) * 8;
    union { uint16_t h[8]; u32x4 v; } hi, mid, lo;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int k = k0 + j;
        const float w = (k < d_in && n < N) ? W_gate[(size_t)k * N + n] : 0.f;
        const bf16_t h = static_cast<bf16_t>(w);
        const float r1 = w - static_cast<float>(h);     // exact
        const bf16_t m = static_cast<bf16_t>(r1);
        const float r2 = r1 - static_cast<float>(m);    // exact, fits 8 bits
        const bf16_t l = static_cast<bf16_t>(r2);
        hi.h[j] = __builtin_bit_cast(uint16_t, h);
        mid.h[j] = __builtin_bit_cast(uint16_t, m);
        lo.h[j] = __builtin_bit_cast(uint16_t, l);
    }
    const size_t base = ((size_t)((ks * 4 + wq) * 8 + s) * 3 * NCB + cb) * 64 + lane;
    wsp[base] = hi.v;
    wsp[base + (size_t)NCB * 64] = mid.v;
    wsp[base + (size_t)2 * NCB * 64] = lo.v;
}

// fragment ((a*S16 + s16)*RCB + cb): lane l holds A[a][s16*16 + (l>>5)*8 + j][cb*32 + (l&31)].
__device__ __forceinline__ void apack_fragment(const bf16_t* __restrict__ A, int d_in, int r, int RCB, int S16,
                                               int64_t frag, int lane, u32x4* __restrict__ apk) {
    const int cb = (int)(frag % RCB);
    const int s16 = (int)((frag / RCB) % S16);
    const int a = (int)(frag / ((int64_t)RCB * S16));
    const int q = cb * 32 + (lane & 31);
    const int k0 = s16 * 16 + (lane >> 5) * 8;
    union { uint16_t h[8]; u32x4 v; } p;
    const uint16_t* Aa = reinterpret_cast<const uint16_t*>(A) + (size_t)a * d_in * r;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int kk = k0 + j;
        p.h[j] = (kk < d_in && q < r) ? Aa[(size_t)kk * r + q] : (uint16_t)0;
    }
    apk[frag * 64 + lane] = p.v;
}

__global__ __launch_bounds__(256) void prep_kernel(const float* __restrict__ W_gate, const bf16_t* __restrict__ A,
                                                   int d_in, int N, int r, int wblocks, int wfrags, int64_t afrags,
                                                   u32x4* __restrict__ wsp, u32x4* __restrict__ apk) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if ((int)blockIdx.x < wblocks) {
        const int frag = blockIdx.x * 4 + wave;
        if (frag < wfrags) wsplit_fragment(W_gate, d_in, N, padded_adapters(N) / 32, frag, lane, wsp);
    } else {
        const int64_t frag = (int64_t)(blockIdx.x - wblocks) * 4 + wave;
        if (frag < afrags)
            apack_fragment(A, d_in, r, ceil_div(r, 32), skinny_kslices(d_in) * (kSkinnyKSL / 16), frag, lane, apk);
    }
}

hipError_t launch_prep(const float* W_gate, void* wsplit, const void* A, void* apack, int d_in, int N, int r,
                       hipStream_t stream) {
    const int wfrags = (W_gate && wsplit) ? wsplit_fragments(d_in, N) : 0;
    const int64_t afrags = (A && apack) ? apack_fragments(d_in, N, r) : 0;
    const int wblocks = ceil_div(wfrags, 4);
    const int64_t blocks = wblocks + ceil_div64(afrags, 4);
    if (blocks == 0) return hipSuccess;
    prep_kernel<<<(unsigned)blocks, 256, 0, stream>>>(W_gate, (const bf16_t*)A, d_in, N, r, wblocks, wfrags, afrags,
                                                      (u32x4*)wsplit, (u32x4*)apack);
    return hipGetLastError();
}

}  // namespace meteora
