// Per-call repacking of the small weight operands into MFMA fragment order (see prep.hpp):
//   - W_gate (fp32) -> three bf16 terms hi + mid + lo that add up to the fp32 value exactly
//     (8 + 8 + 8 significand bits), so that bf16 MFMAs reproduce fp32-level gate logits;
//   - stacked LoRA A[N, d_in, r] (Sec. 3.3) -> fragments with the rank padded to 32 columns;
//   - stacked LoRA B[N, r, d_out] viewed as [N*r, d_out] -> its transpose Bt[d_out, ext_stride]
//     (columns >= N*r zero), the layout the GEMM's K-extension streams like W.
//   - for the dense routing path, Wcat[3*NP + N*r, d_in]: the three gate terms and every column of every
//     A_i as rows contiguous along d_in, the layout the GEMM kernel streams like W.
// All run in ONE launch (disjoint workgroup ranges); a wavefront writes one fragment, a workgroup
// one 64x64 tile of a transpose.
#include "common.hpp"
#include "kernels.hpp"
#include "prep.hpp"

namespace meteora {

// The three bf16 terms of an fp32 gate weight: hi + mid + lo == w exactly (8 + 8 + 8 significand bits).
__device__ __forceinline__ void split3(float w, uint16_t& hi, uint16_t& mid, uint16_t& lo) {
    const bf16_t h = static_cast<bf16_t>(w);
    const float r1 = w - static_cast<float>(h);     // exact
    const bf16_t m = static_cast<bf16_t>(r1);
    const float r2 = r1 - static_cast<float>(m);    // exact, fits 8 bits
    const bf16_t l = static_cast<bf16_t>(r2);
    hi = __builtin_bit_cast(uint16_t, h);
    mid = __builtin_bit_cast(uint16_t, m);
    lo = __builtin_bit_cast(uint16_t, l);
}

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
        split3(w, hi.h[j], mid.h[j], lo.h[j]);
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

// tile (tj, tc): Bt[tc*64 + c][tj*64 + j] = B[tj*64 + j][tc*64 + c], zero where j >= ext_k.
// 16-byte loads along c, a padded LDS tile, 2 x 16-byte stores along j (d_out % 8 == 0, so a
// chunk of 8 columns is all inside or all outside the matrix).
__device__ __forceinline__ void btrans_tile(const uint16_t* __restrict__ B, int d_out, int ext_k, int ext_stride,
                                            int tile, int tid, uint16_t* __restrict__ Bt) {
    constexpr int LD = 72;   // 144-byte rows: 16-byte aligned, odd multiple of 16 B across banks
    __shared__ __attribute__((aligned(16))) uint16_t t[64 * LD];
    const int tiles_j = ext_stride / 64;
    const int j0 = (tile % tiles_j) * 64, c0 = (tile / tiles_j) * 64;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int j = i * 32 + (tid >> 3), c = (tid & 7) * 8;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (j0 + j < ext_k && c0 + c < d_out) v = *reinterpret_cast<const u32x4*>(B + (size_t)(j0 + j) * d_out + c0 + c);
        *reinterpret_cast<u32x4*>(&t[j * LD + c]) = v;
    }
    __syncthreads();
    const int c = tid >> 2, jq = (tid & 3) * 16;
    if (c0 + c < d_out) {
        union { uint16_t h[16]; u32x4 v[2]; } p;
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) p.h[jj] = t[(jq + jj) * LD + c];
        u32x4* dst = reinterpret_cast<u32x4*>(Bt + (size_t)(c0 + c) * ext_stride + j0 + jq);
        dst[0] = p.v[0];
        dst[1] = p.v[1];
    }
}

// tile (ti, tr) of Wcat[rows, d_in]: row R = term*NP + j (term 0..2 = hi, mid, lo of W_gate[:, j]; zero for
// j >= N), then row 3*NP + a*r + q = A[a][:, q], then zero rows up to `rows`.  Sources are read along the
// row index (contiguous in W_gate and, per adapter, in A), transposed through LDS, stored along d_in.
__device__ __forceinline__ void wcat_tile(const float* __restrict__ W_gate, const uint16_t* __restrict__ A, int d_in,
                                          int N, int NP, int r, int rows, int tile, int tid,
                                          uint16_t* __restrict__ Wcat) {
    constexpr int LD = 66;
    __shared__ uint16_t t[64 * LD];   // t[i][row]
    const int tiles_i = d_in / 64;
    const int i0 = (tile % tiles_i) * 64, R0 = (tile / tiles_i) * 64;
    // Rows come in groups of 8 that never straddle a region (NP, r and the region starts are multiples of 8): a group
    // of gate rows is 8 consecutive columns j of one term; a group of A rows is columns q0..q0+7 of one adapter,
    // one 16-byte load per i, consecutive threads along i so that a wavefront reads 1 KB of A contiguously.
    // All index arithmetic is per group, i.e. uniform across the 64 threads that share it.
    for (int item = tid; item < 8 * 64; item += 256) {
        const int g = item >> 6, ii = item & 63;
        const int Rg = R0 + g * 8, i = i0 + ii;
        union { uint16_t h[8]; uint32_t w[4]; u32x4 v; } p;
        p.v = u32x4{0u, 0u, 0u, 0u};
        if (Rg < 3 * NP) {
            const int term = Rg / NP, j0 = Rg - term * NP;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                if (j0 + jj < N) {
                    uint16_t h, m, l;
                    split3(W_gate[(size_t)i * N + j0 + jj], h, m, l);
                    p.h[jj] = term == 0 ? h : (term == 1 ? m : l);
                }
            }
        } else if (Rg < 3 * NP + N * r) {
            const int c = Rg - 3 * NP, a = c / r, q0 = c - a * r;
            p.v = *reinterpret_cast<const u32x4*>(A + ((size_t)a * d_in + i) * r + q0);
        }
        uint32_t* dst = reinterpret_cast<uint32_t*>(&t[ii * LD + g * 8]);
        dst[0] = p.w[0]; dst[1] = p.w[1]; dst[2] = p.w[2]; dst[3] = p.w[3];
    }
    __syncthreads();
    const int rr = tid >> 2, iq = (tid & 3) * 16;
    if (R0 + rr < rows) {
        union { uint16_t h[16]; u32x4 v[2]; } p;
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) p.h[jj] = t[(iq + jj) * LD + rr];
        u32x4* dst = reinterpret_cast<u32x4*>(Wcat + (size_t)(R0 + rr) * d_in + i0 + iq);
        dst[0] = p.v[0];
        dst[1] = p.v[1];
    }
}

__global__ __launch_bounds__(256) void prep_kernel(const float* __restrict__ W_gate, const bf16_t* __restrict__ A,
                                                   int d_in, int N, int r, int wblocks, int wfrags, int64_t afrags,
                                                   u32x4* __restrict__ wsp, u32x4* __restrict__ apk,
                                                   const uint16_t* __restrict__ B, uint16_t* __restrict__ Bt,
                                                   int d_out, int ext_stride, int bblocks,
                                                   uint16_t* __restrict__ Wcat, int cat_rows, int cblocks) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if ((int)blockIdx.x < bblocks) {   // uniform per workgroup
        btrans_tile(B, d_out, N * r, ext_stride, blockIdx.x, threadIdx.x, Bt);
        return;
    }
    if ((int)blockIdx.x < bblocks + cblocks) {
        wcat_tile(W_gate, reinterpret_cast<const uint16_t*>(A), d_in, N, padded_adapters(N), r, cat_rows,
                  blockIdx.x - bblocks, threadIdx.x, Wcat);
        return;
    }
    const int blk = blockIdx.x - bblocks - cblocks;
    if (blk < wblocks) {
        const int frag = blk * 4 + wave;
        if (frag < wfrags) wsplit_fragment(W_gate, d_in, N, padded_adapters(N) / 32, frag, lane, wsp);
    } else {
        const int64_t frag = (int64_t)(blk - wblocks) * 4 + wave;
        if (frag < afrags)
            apack_fragment(A, d_in, r, ceil_div(r, 32), skinny_kslices(d_in) * (kSkinnyKSL / 16), frag, lane, apk);
    }
}

size_t prep_btrans_bytes(int d_out, int N, int r, bool bf16) {
    return bf16 ? (size_t)d_out * align_up((size_t)N * r, 64) * sizeof(uint16_t) : 0;
}

int prep_wcat_rows(int N, int r) { return (int)align_up((size_t)3 * padded_adapters(N) + (size_t)N * r, 8); }

size_t prep_wcat_bytes(int d_in, int N, int r, bool bf16) {
    return (bf16 && d_in % 64 == 0) ? (size_t)prep_wcat_rows(N, r) * d_in * sizeof(uint16_t) : 0;
}

hipError_t launch_prep(const float* W_gate, void* wsplit, const void* A, void* apack, const void* B, void* btrans,
                       void* wcat, int d_in, int d_out, int N, int r, hipStream_t stream) {
    const int wfrags = (W_gate && wsplit) ? wsplit_fragments(d_in, N) : 0;
    const int64_t afrags = (A && apack) ? apack_fragments(d_in, N, r) : 0;
    const int ext_stride = (int)align_up((size_t)N * r, 64);
    const int bblocks = (B && btrans) ? (ext_stride / 64) * ceil_div(d_out, 64) : 0;
    const int wblocks = ceil_div(wfrags, 4);
    const int cat_rows = prep_wcat_rows(N, r);
    if (wcat && (!W_gate || !A || d_in % 64 != 0 || r % 8 != 0)) return hipErrorInvalidValue;
    const int cblocks = wcat ? ceil_div(cat_rows, 64) * (d_in / 64) : 0;
    const int64_t blocks = (int64_t)bblocks + cblocks + wblocks + ceil_div64(afrags, 4);
    if (blocks == 0) return hipSuccess;
    prep_kernel<<<(unsigned)blocks, 256, 0, stream>>>(W_gate, (const bf16_t*)A, d_in, N, r, wblocks, wfrags, afrags,
                                                      (u32x4*)wsplit, (u32x4*)apack, (const uint16_t*)B,
                                                      (uint16_t*)btrans, d_out, ext_stride, bblocks, (uint16_t*)wcat,
                                                      cat_rows, cblocks);
    return hipGetLastError();
}

}  // namespace meteora
