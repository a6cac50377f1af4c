// Measurement tool (not part of the library): what the operand traffic of the 256 x 256 GEMM costs the matrix
// cores, piece by piece.  One workgroup of 4 wavefronts per CU runs the GEMM's per-K-tile instruction mix on
// synthetic data, with no barriers and no dependence between the loads and the arithmetic:
//   0  64 v_mfma_f32_32x32x16_bf16 per wavefront and K tile, operands loaded once
//   1  + the fragment reads: 8 ds_read_b128 per 16 MFMAs from 64 KB of LDS
//   2  + the operand tiles as global->LDS loads: 16 buffer_load ... lds (16 B per lane) per wavefront and K tile
//   3  + the same bytes through registers instead: 16 global_load_dwordx4 and 16 ds_write_b128
// on zero or on random data (like x and W of the layer), the global working set 2 MB (L2 hits).
//
//   operand_path_probe [K tiles per launch, default 4000] [1 = zero data]
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#include <cstring>
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
__device__ unsigned mix(unsigned x) { x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16; return x; }

template <int MODE>
__global__ __launch_bounds__(256) void probe(const u32x4* __restrict__ g, size_t gmask16, float* out, int iters, int zero) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // region A: 64 KB of random operands; region B: 64 KB landing zone
    u32x4* la = reinterpret_cast<u32x4*>(smem);
    for (int i = threadIdx.x; i < 4096; i += 256) {
        u32x4 v;
        for (int j = 0; j < 4; ++j) {
            const unsigned h = mix(i * 4 + j + blockIdx.x * 16384);
            // two bf16: x-like (-1,1) in low, w-like small in high
            const float a = (h & 0xffff) / 32768.f - 1.f, b = ((h >> 16) / 32768.f - 1.f) * 0.02f;
            v[j] = zero ? 0u : ((__builtin_bit_cast(uint32_t, a) >> 16) | (__builtin_bit_cast(uint32_t, b) & 0xffff0000u));
        }
        la[i] = v;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    f32x16 acc[16];
    for (int i = 0; i < 16; ++i) for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    bf16x8 a[4], b[4];
    for (int i = 0; i < 4; ++i) { a[i] = __builtin_bit_cast(bf16x8, la[(lane + i * 64) & 4095]); b[i] = __builtin_bit_cast(bf16x8, la[(lane + i * 64 + 256) & 4095]); }
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<u32x4*>(g), 0, 0xffffffffu, 0x00020000);
    size_t gpos = ((size_t)blockIdx.x * 4 + wave) * 1024;   // in 16-byte units
    for (int it = 0; it < iters; ++it) {
        if constexpr (MODE == 2) {
#pragma unroll
            for (int p = 0; p < 16; ++p) {
                const uint32_t off = (uint32_t)(((gpos + (size_t)p * 64 + lane) & gmask16) * 16);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)(smem + 65536 + (wave * 16 + p) * 1024), 16, off, 0, 0, 0);
            }
        }
        u32x4 stage[16];
        if constexpr (MODE == 3) {
#pragma unroll
            for (int p = 0; p < 16; ++p) stage[p] = g[(gpos + (size_t)p * 64 + lane) & gmask16];
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if constexpr (MODE >= 1) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    a[i] = __builtin_bit_cast(bf16x8, la[(lane + (it * 8 + ks * 2) * 64 + i * 512) & 4095]);
                    b[i] = __builtin_bit_cast(bf16x8, la[(lane + (it * 8 + ks * 2 + 1) * 64 + i * 512) & 4095]);
                }
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3], b[i >> 2], acc[i], 0, 0, 0);
        }
        if constexpr (MODE == 3) {
#pragma unroll
            for (int p = 0; p < 16; ++p) reinterpret_cast<u32x4*>(smem + 65536)[(wave * 16 + p) * 64 + lane] = stage[p];
        }
        gpos += 1048576;   // next 16 MB slab
    }
    if constexpr (MODE == 2) __builtin_amdgcn_s_waitcnt(0);
    float s = 0.f;
    for (int i = 0; i < 16; ++i) for (int j = 0; j < 16; ++j) s += acc[i][j];
    if (MODE >= 2) s += reinterpret_cast<float*>(smem + 65536)[threadIdx.x];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}
#define CHECK(e) do { hipError_t err_ = (e); if (err_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #e, hipGetErrorString(err_)); return 1; } } while (0)
static int g_zero = 0;
template <int MODE> int run(const char* name, const u32x4* g, size_t gmask16, float* out, int iters) {
    hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&probe<MODE>), hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
    const int blocks = 256;
    const double flops = 2.0 * 32 * 32 * 16 * 64.0 * iters * 4.0 * blocks;
    float ms = 0;
    for (int rep = 0; rep < 4; ++rep) {
        CHECK(hipEventRecord(e0));
        probe<MODE><<<blocks, 256, 131072>>>(g, gmask16, out, iters, g_zero);
        CHECK(hipGetLastError());
        CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1)); CHECK(hipEventElapsedTime(&ms, e0, e1));
    }
    printf("%-60s %9.1f us %8.1f TFLOP/s\n", name, ms * 1e3, flops / ms / 1e9); fflush(stdout);
    return 0;
}
int main(int argc, char** argv) {
    const int iters = argc > 1 ? atoi(argv[1]) : 4000;
    g_zero = argc > 2 ? atoi(argv[2]) : 0;
    const size_t gbytes = 64u << 20;   // 64 MB: L2 + Infinity Cache resident, like x and W of the layer
    u32x4* g; float* out;
    CHECK(hipMalloc(&g, gbytes)); CHECK(hipMalloc(&out, 256 * 256 * 4));
    {   // random fill
        uint32_t* h = (uint32_t*)malloc(gbytes);
        for (size_t i = 0; i < gbytes / 4; ++i) { uint32_t x = (uint32_t)i * 2654435761u; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 13; h[i] = (x & 0x3fff3fffu) | 0x3c003c00u ^ (x & 0x80008000u); }
        if (g_zero) memset(h, 0, gbytes);
        CHECK(hipMemcpy(g, h, gbytes, hipMemcpyHostToDevice)); free(h);
    }
    for (size_t ws : {(size_t)(2u << 20)}) {
    const size_t gmask16 = ws / 16 - 1;
    printf("global working set %zu MB\n", ws >> 20);
    if (run<0>("MFMA only (1 WG of 4 waves per CU, 256 WGs)", g, gmask16, out, iters)) return 1;
    if (run<1>("+ 8 ds_read_b128 per 16 MFMAs", g, gmask16, out, iters)) return 1;
    if (run<2>("+ 16 global->LDS DMA (16 B/lane) per wave per 64 MFMAs", g, gmask16, out, iters)) return 1;
    if (run<3>("+ same bytes via global_load_dwordx4 + ds_write_b128", g, gmask16, out, iters)) return 1;
    if (run<2>("+ DMA again", g, gmask16, out, iters)) return 1;
    }
    return 0;
}
