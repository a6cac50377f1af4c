// Layout of the two weight operands that the skinny MFMA kernels (gate logits, grouped shrink)
// read as ready-made v_mfma_f32_32x32x16_bf16 fragments: 64 lanes x 16 bytes = one contiguous
// 1 KB block per fragment, lane l holding 8 consecutive k of column (l & 31), k-half (l >> 5).
// Both kernels cut d_in into 512-wide K-slices, a quarter (128) per wavefront, 16 per k-step.
#pragma once
#include "common.hpp"

namespace meteora {

constexpr int kSkinnyKSL = 512;   // K-slice per workgroup
constexpr int kSkinnyKW = 128;    // K per wavefront (8 k-steps of 16)

__host__ __device__ constexpr int skinny_kslices(int d_in) { return ceil_div(d_in, kSkinnyKSL); }

// fragments of the split gate weight: (ks, wq, s, cb), three 1 KB blocks (hi, mid, lo) each
__host__ __device__ constexpr int wsplit_fragments(int d_in, int N) {
    return skinny_kslices(d_in) * 4 * 8 * (padded_adapters(N) / 32);
}
// fragments of the packed LoRA A: (adapter, k-step of 16, column block of 32)
__host__ __device__ constexpr int64_t apack_fragments(int d_in, int N, int r) {
    return (int64_t)N * skinny_kslices(d_in) * (kSkinnyKSL / 16) * ceil_div(r, 32);
}

}  // namespace meteora
