// Shared device-side helpers for the gfx950 MeteoRA kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace meteora {

constexpr int kWave = 64;        // CDNA wavefront width
constexpr int kMaxAdapters = 64; // N <= 64: one wavefront lane per adapter in the top-k
constexpr int kMaxTopK = 8;
constexpr int kMaxRank = 64;

typedef __bf16 bf16_t;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16_t v) { return static_cast<float>(v); }

template <typename T> __device__ __forceinline__ T from_float(float v);
template <> __device__ __forceinline__ float from_float<float>(float v) { return v; }
// float -> bf16, round to nearest even (v_cvt_pk_bf16_f32 on gfx950)
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float v) { return static_cast<bf16_t>(v); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    union { bf16_t h[2]; uint32_t u; } p;
    p.h[0] = static_cast<bf16_t>(lo);
    p.h[1] = static_cast<bf16_t>(hi);
    return p.u;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
    return __uint_as_float(bits16 << 16);
}

__host__ __device__ constexpr int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ constexpr int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }
__host__ __device__ constexpr size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Number of logit columns the gate kernels carry: N padded to 32 or 64.
__host__ __device__ constexpr int padded_adapters(int N) { return N <= 32 ? 32 : 64; }

}  // namespace meteora
