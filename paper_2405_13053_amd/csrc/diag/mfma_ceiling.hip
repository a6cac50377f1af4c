// Measurement tool (not part of the library): what the matrix cores of this GPU sustain on a loop of nothing but
// bf16 MFMAs (v_mfma_f32_32x32x16_bf16, register operands, no memory traffic), with operands that are constants
// and with operands that look like the layer's data (zero-mean random values).  The chip lowers its shader clock
// with the power the operands' bit activity draws, so the second figure, not the published peak, is the ceiling
// that a GEMM on Gaussian data works under; the base projection's roofline fraction is reported against the
// published peak and read against this one.
//
//   mfma_ceiling [iterations per launch, default 2000]
//
// One workgroup of 4 wavefronts per CU slot (1024 workgroups), 64 MFMAs per iteration and wavefront over 16
// independent accumulators; each case runs three times after a warm-up launch and the last is reported.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

__device__ unsigned mix(unsigned x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// RANDOM: operands uniform in (-1, 1) and (-0.02, 0.02) (like x and W); otherwise ones and zeros.
// DISTINCT: 4 + 4 different operand registers combined as a 4 x 4 block (like a 128 x 128 wavefront tile);
// otherwise every MFMA reads the same two registers.
template <bool RANDOM, bool DISTINCT, int CHAIN = 1>
__global__ __launch_bounds__(256) void mfma_loop(float* out, int iters) {
    bf16x8 a[4], b[4];
    for (int r = 0; r < 4; ++r)
        for (int j = 0; j < 8; ++j) {
            const unsigned h = mix((blockIdx.x * 256 + threadIdx.x) * 64 + r * 8 + j);
            a[r][j] = (__bf16)(RANDOM ? ((h & 0xffff) / 32768.f - 1.f) : 1.f);
            b[r][j] = (__bf16)(RANDOM ? ((h >> 16) / 32768.f - 1.f) * 0.02f : 0.f);
        }
    f32x16 acc[16];
    for (int i = 0; i < 16; ++i)
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
        // CHAIN consecutive MFMAs accumulate into the same block (the k-steps of a tile taken per block) before the
        // next block's turn; CHAIN = 1 visits all 16 blocks per k-step
#pragma unroll
        for (int r = 0; r < 4 / CHAIN; ++r)
#pragma unroll
            for (int i = 0; i < 16; ++i)
#pragma unroll
                for (int c = 0; c < CHAIN; ++c)
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[DISTINCT ? ((i + c) & 3) : 0],
                                                                     b[DISTINCT ? ((i >> 2) ^ c) & 3 : 0], acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 16; ++i)
        for (int j = 0; j < 16; ++j) s += acc[i][j];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The same arithmetic per iteration with v_mfma_f32_16x16x32_bf16: 8 + 8 operand registers as an 8 x 8 block of
// 16 x 16 accumulators (again a 128 x 128 wavefront tile), 128 MFMAs of 16 cycles per iteration.  Per
// multiply-add this shape reads twice the operand registers and half the accumulator registers of 32x32x16.
template <bool RANDOM>
__global__ __launch_bounds__(256) void mfma_loop_16(float* out, int iters) {
    bf16x8 a[8], b[8];
    for (int r = 0; r < 8; ++r)
        for (int j = 0; j < 8; ++j) {
            const unsigned h = mix((blockIdx.x * 256 + threadIdx.x) * 64 + r * 8 + j);
            a[r][j] = (__bf16)(RANDOM ? ((h & 0xffff) / 32768.f - 1.f) : 1.f);
            b[r][j] = (__bf16)(RANDOM ? ((h >> 16) / 32768.f - 1.f) * 0.02f : 0.f);
        }
    f32x4 acc[64];
    for (int i = 0; i < 64; ++i)
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int i = 0; i < 64; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 7], b[i >> 3], acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 64; ++i)
        for (int j = 0; j < 4; ++j) s += acc[i][j];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

#define CHECK(e)                                                                      \
    do {                                                                              \
        hipError_t err_ = (e);                                                        \
        if (err_ != hipSuccess) {                                                     \
            fprintf(stderr, "%s: %s\n", #e, hipGetErrorString(err_));                 \
            return 1;                                                                 \
        }                                                                             \
    } while (0)

template <bool RANDOM, bool DISTINCT, int CHAIN = 1>
int run(const char* name, float* out, int iters, int blocks) {
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const double flops = 2.0 * 32 * 32 * 16 * 64.0 * iters * 4.0 * blocks;
    float ms = 0.f;
    for (int rep = 0; rep < 4; ++rep) {
        CHECK(hipEventRecord(e0));
        mfma_loop<RANDOM, DISTINCT, CHAIN><<<blocks, 256>>>(out, iters);
        CHECK(hipGetLastError());
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        CHECK(hipEventElapsedTime(&ms, e0, e1));
    }
    printf("%-44s %9.1f us  %8.1f TFLOP/s  (%.3f of 2500)\n", name, ms * 1e3, flops / ms / 1e9, flops / ms / 1e9 / 2500.0);
    fflush(stdout);
    return 0;
}

template <bool RANDOM>
int run16(const char* name, float* out, int iters, int blocks) {
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const double flops = 2.0 * 16 * 16 * 32 * 128.0 * iters * 4.0 * blocks;
    float ms = 0.f;
    for (int rep = 0; rep < 4; ++rep) {
        CHECK(hipEventRecord(e0));
        mfma_loop_16<RANDOM><<<blocks, 256>>>(out, iters);
        CHECK(hipGetLastError());
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        CHECK(hipEventElapsedTime(&ms, e0, e1));
    }
    printf("%-44s %9.1f us  %8.1f TFLOP/s  (%.3f of 2500)\n", name, ms * 1e3, flops / ms / 1e9, flops / ms / 1e9 / 2500.0);
    fflush(stdout);
    return 0;
}

int main(int argc, char** argv) {
    const int iters = argc > 1 ? atoi(argv[1]) : 2000;
    if (iters < 1 || iters > 100000) { fprintf(stderr, "iterations out of range\n"); return 2; }
    const int blocks = 1024;
    float* out = nullptr;
    CHECK(hipMalloc(&out, (size_t)blocks * 256 * sizeof(float)));
    printf("bf16 MFMA 32x32x16 loop, %d workgroups x 4 wavefronts, %d x 64 MFMAs per wavefront\n", blocks, iters);
    if (run<false, false>("constant operands, one register pair", out, iters, blocks)) return 1;
    if (run<false, true>("constant operands, 4 x 4 register block", out, iters, blocks)) return 1;
    if (run<true, false>("random operands, one register pair", out, iters, blocks)) return 1;
    if (run<true, true>("random operands, 4 x 4 register block", out, iters, blocks)) return 1;
    if (run<false, true>("constant operands again (clock recovered?)", out, iters, blocks)) return 1;
    if (run<false, true, 2>("constant, 4 x 4 block, 2 MFMAs per block in a row", out, iters, blocks)) return 1;
    if (run<true, true, 2>("random, 4 x 4 block, 2 MFMAs per block in a row", out, iters, blocks)) return 1;
    if (run<false, true, 4>("constant, 4 x 4 block, 4 MFMAs per block in a row", out, iters, blocks)) return 1;
    if (run<true, true, 4>("random, 4 x 4 block, 4 MFMAs per block in a row", out, iters, blocks)) return 1;
    if (run<true, true>("random, 4 x 4 block, one per block (again)", out, iters, blocks)) return 1;
    printf("bf16 MFMA 16x16x32 loop, same arithmetic per wavefront (%d x 128 MFMAs)\n", iters);
    if (run16<false>("16x16x32 constant operands, 8 x 8 block", out, iters, blocks)) return 1;
    if (run16<true>("16x16x32 random operands, 8 x 8 block", out, iters, blocks)) return 1;
    if (run<true, true>("32x32x16 random, 4 x 4 block, again", out, iters, blocks)) return 1;
    if (run16<true>("16x16x32 random operands, again", out, iters, blocks)) return 1;
    CHECK(hipFree(out));
    return 0;
}
