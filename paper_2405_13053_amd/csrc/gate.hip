// Gate network and top-k routing of the MeteoRA layer (paper Sec. 3.1):
//   G(x) = x * W_gate (+ bias), I(x) = top-k of G(x), w = softmax over the k selected (Eq. 3).
//
// Two stages:
//   1. logit partial sums  partials[ks][t][j] = sum_{i in K-slice ks} x[t,i] * W_gate[i,j]
//   2. per token, one wavefront: sum the K-slices in a fixed order, add the bias, select the
//      top-k with a wavefront-wide arg-max (ties -> lowest adapter index), softmax over the k.
#include "common.hpp"
#include "kernels.hpp"
#include "topk_key.hpp"
#include "prep.hpp"

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
// Stage 2: wavefront-level top-k.
//
// A token's NP (32 or 64) logit columns sit in NP adjacent lanes, so a wavefront ranks 64/NP tokens
// at a time (wave_topk_softmax); the groups a wavefront owns are interleaved so their shuffle
// latencies overlap.
//
// A workgroup of 16 wavefronts owns one bucketing chunk of 64 tokens (4 per wavefront) and also
// leaves the chunk's adapter histogram for the scatter pass.
// ------------------------------------------------------------------------------------------
constexpr int kTopkTokensPerWave = 4;
constexpr int kTopkWaves = kBucketChunkTokens / kTopkTokensPerWave;
static_assert(kTopkWaves * 64 <= 1024, "one workgroup per bucketing chunk");

template <int NP>
__global__ __launch_bounds__(kTopkWaves * 64) void gate_topk_kernel(
    const float* __restrict__ partials, int KS, const float* __restrict__ bias, int T, int N, int k,
    float inv_temperature, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, float* __restrict__ logits,
    int32_t* __restrict__ chunk_counts) {
    constexpr int TPP = 64 / NP;                     // tokens ranked per pass
    constexpr int G = kTopkTokensPerWave / TPP;      // passes (groups) per wavefront
    __shared__ int hist[kMaxAdapters];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & (NP - 1), sub = lane / NP;
    if (threadIdx.x < kMaxAdapters) hist[threadIdx.x] = 0;
    __syncthreads();
    const int t0 = blockIdx.x * kBucketChunkTokens + wave * kTopkTokensPerWave;

    float g[G];
    int tok[G];
#pragma unroll
    for (int i = 0; i < G; ++i) { g[i] = 0.f; tok[i] = t0 + i * TPP + sub; }
    if (col < N) {
        // fixed order over K-slices; 16 slices' loads are issued together, from clamped addresses so that no
        // branch separates them (the loop is latency-bound); a slice past the end is not added
        for (int s0 = 0; s0 < KS; s0 += 16) {
            float v[16][G];
#pragma unroll
            for (int u = 0; u < 16; ++u)
#pragma unroll
                for (int i = 0; i < G; ++i)
                    v[u][i] = partials[((size_t)min(s0 + u, KS - 1) * T + min(tok[i], T - 1)) * NP + col];
#pragma unroll
            for (int u = 0; u < 16; ++u)
#pragma unroll
                for (int i = 0; i < G; ++i)
                    if (s0 + u < KS) g[i] += v[u][i];
        }
        const float b = bias != nullptr ? bias[col] : 0.f;
#pragma unroll
        for (int i = 0; i < G; ++i) {
            g[i] += b;
            if (g[i] == 0.f) g[i] = 0.f;   // -0 -> +0 so equal logits have equal keys
            if (logits && tok[i] < T) logits[(size_t)tok[i] * N + col] = g[i];
        }
    }
    int sel_i[G];     // lane col = s < k of each token keeps its s-th selected adapter and weight
    float sel_w[G];
    wave_topk_softmax<NP, G>(g, lane, N, k, inv_temperature, sel_i, sel_w);
#pragma unroll
    for (int i = 0; i < G; ++i) {
        if (col < k && tok[i] < T) {
            topk_idx[(size_t)tok[i] * k + col] = sel_i[i];
            topk_w[(size_t)tok[i] * k + col] = sel_w[i];
            atomicAdd(&hist[sel_i[i]], 1);
        }
    }
    __syncthreads();
    if (chunk_counts && threadIdx.x < N) chunk_counts[(size_t)blockIdx.x * N + threadIdx.x] = hist[threadIdx.x];
}

// ------------------------------------------------------------------------------------------
// Stage 1, MFMA version for bf16 tokens.
//
// The gate is a skinny contraction x[T,d_in] * W_gate[d_in,N] that must keep fp32-level logits
// (they decide the routing).  x is bf16, W_gate is fp32: W_gate is split once per call into three
// bf16 terms hi+mid+lo that add up to the fp32 value exactly (8+8+8 significand bits), every
// bf16 x bf16 product is exact in fp32, and v_mfma_f32_32x32x16_bf16 accumulates in fp32; only
// the summation order differs from a plain fp32 dot product.
//
// Work split: a workgroup takes 128 tokens x one 512-wide K-slice; its 4 wavefronts take a
// quarter of the slice each (no barrier in the main loop).  A wavefront
//   - streams its 128 x 128 piece of x from HBM straight into its own 32 KB of LDS with 16-byte
//     global->LDS loads (16 lanes cover one 256-byte row segment: fully coalesced),
//     chunks XOR-swizzled by row so the later ds_read_b128 are conflict free,
//   - reads the split W_gate fragments, pre-arranged in MFMA operand order so that each
//     fragment is one contiguous 1 KB block, directly from L2 into registers and reuses each
//     for the 4 row blocks of 32 tokens.
// The 4 partial tiles are summed through LDS in a fixed order and written as
// partials[ks][t][NP]; the top-k kernel adds the K-slices in order.
// ------------------------------------------------------------------------------------------
constexpr int kGateKSL = kSkinnyKSL; // K-slice per workgroup
constexpr int kGateKW = kSkinnyKW;   // K per wavefront
// LDS bytes per wavefront: its RB*32 x 256 B piece of x, reused for the padded fp32 reduction tile
__host__ __device__ constexpr int gate_region_bytes(int NCB, int RB) {
    const int xbytes = RB * 32 * 256, red = RB * 32 * (NCB * 128 + 16);
    return (int)align_up((size_t)(xbytes > red ? xbytes : red), 1024);
}

template <int NCB, int RB>
__global__ __launch_bounds__(256) void gate_logits_mfma_kernel(const bf16_t* __restrict__ x,
                                                               const u32x4* __restrict__ wsp, int T, int d_in,
                                                               int KS, float* __restrict__ partials) {
    constexpr int NP = NCB * 32;
    constexpr int TM = RB * 32;                                   // tokens per workgroup
    constexpr int kRegion = gate_region_bytes(NCB, RB);           // LDS bytes per wavefront
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int lane = threadIdx.x & 63, wq = threadIdx.x >> 6;
    const int ks = blockIdx.x % KS, tile = blockIdx.x / KS;
    const int t0 = tile * TM;
    unsigned char* region = smem + wq * kRegion;
    const int kbase = ks * kGateKSL + wq * kGateKW;

    // ---- x piece: 128 rows x 256 B, HBM -> LDS, 4 rows per instruction --------------------
    {
        const int rsub = lane >> 4, p = lane & 15;
#pragma unroll
        for (int j = 0; j < RB * 8; ++j) {
            const int row = 4 * j + rsub;
            int t = t0 + row;
            t = t < T ? t : T - 1;
            int kk = kbase + ((p ^ (row & 15)) << 3);
            kk = kk <= d_in - 8 ? kk : d_in - 8;   // past-the-end columns meet zero weights; keep the address in range
            const bf16_t* src = x + (size_t)t * d_in + kk;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)(region + j * 1024), 16, 0, 0);
        }
    }
    // ---- W fragments of this wavefront's K quarter: 8 k-steps x 3 terms x NCB ---------------
    bf16x8 wf[8][3][NCB];
    {
        const u32x4* wbase = wsp + (size_t)((ks * 4 + wq) * 8) * 3 * NCB * 64 + lane;
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int sp = 0; sp < 3; ++sp)
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) {
                    const u32x4 v = wbase[(size_t)((s * 3 + sp) * NCB + cb) * 64];
                    wf[s][sp][cb] = __builtin_bit_cast(bf16x8, v);
                }
    }
    __builtin_amdgcn_s_waitcnt(0);   // everything issued above has landed (vmcnt = lgkmcnt = 0)
    __builtin_amdgcn_wave_barrier();

    f32x16 acc[RB][NCB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[rb][cb][i] = 0.f;

    const int lrow = lane & 31, khalf = lane >> 5;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int row = rb * 32 + lrow;
            const int pos = (s * 2 + khalf) ^ (row & 15);
            const bf16x8 xf = *reinterpret_cast<const bf16x8*>(region + row * 256 + pos * 16);
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[s][0][cb], xf, acc[rb][cb], 0, 0, 0);
                acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[s][1][cb], xf, acc[rb][cb], 0, 0, 0);
                acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[s][2][cb], xf, acc[rb][cb], 0, 0, 0);
            }
        }
    }

    // ---- sum the 4 K quarters through LDS (fixed order), write partials[ks][t][:] ------------
    constexpr int kRowBytes = NP * 4 + 16;   // padded: consecutive tokens start 4 banks apart
    __builtin_amdgcn_wave_barrier();          // this wavefront's own ds_reads are done before it overwrites
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int m = rb * 32 + lrow, n = cb * 32 + g * 8 + khalf * 4;
                f32x4 v = {acc[rb][cb][g * 4 + 0], acc[rb][cb][g * 4 + 1], acc[rb][cb][g * 4 + 2],
                           acc[rb][cb][g * 4 + 3]};
                *reinterpret_cast<f32x4*>(region + m * kRowBytes + n * 4) = v;
            }
    __syncthreads();
    constexpr int kChunksPerRow = NP / 4;
    for (int c = threadIdx.x; c < TM * kChunksPerRow; c += 256) {
        const int m = c / kChunksPerRow, n4 = c % kChunksPerRow;
        const int t = t0 + m;
        if (t >= T) continue;
        const int off = m * kRowBytes + n4 * 16;
        f32x4 v0 = *reinterpret_cast<const f32x4*>(smem + off);
        f32x4 v1 = *reinterpret_cast<const f32x4*>(smem + kRegion + off);
        f32x4 v2 = *reinterpret_cast<const f32x4*>(smem + 2 * kRegion + off);
        f32x4 v3 = *reinterpret_cast<const f32x4*>(smem + 3 * kRegion + off);
        f32x4 r = (v0 + v1) + (v2 + v3);
        *reinterpret_cast<f32x4*>(partials + ((size_t)ks * T + t) * NP + n4 * 4) = r;
    }
}

int gate_kslices(int d_in, bool bf16) { return bf16 ? ceil_div(d_in, kGateKSL) : 1; }

size_t gate_wsplit_bytes(int d_in, int N, bool bf16) {
    if (!bf16) return 0;
    return (size_t)gate_kslices(d_in, true) * kGateKSL * padded_adapters(N) * 3 * sizeof(bf16_t);
}

hipError_t launch_gate_logits(const void* x, const float* W_gate, int T, int d_in, int N, bool bf16,
                              void* wsplit, float* partials, hipStream_t stream) {
    const int NP = padded_adapters(N);
    if (!bf16) {
        gate_logits_fma_kernel<float><<<T, 256, 0, stream>>>((const float*)x, W_gate, T, d_in, N, NP, partials);
        return hipGetLastError();
    }
    const int KS = gate_kslices(d_in, true), NCB = NP / 32;
    // wsplit has been filled by launch_prep
    // 64 tokens per workgroup: two workgroups share a CU, so one loads while the other computes
    // (measured faster than 32 or 128 tokens on every configuration, 4096 to 16384 tokens)
    auto launch = [&](auto kern, int rb) -> hipError_t {
        const int smem = 4 * gate_region_bytes(NCB, rb);
        hipError_t err = ensure_lds_limit(reinterpret_cast<const void*>(kern), smem);
        if (err != hipSuccess) return err;
        kern<<<ceil_div(T, rb * 32) * KS, 256, smem, stream>>>((const bf16_t*)x, (const u32x4*)wsplit, T, d_in, KS,
                                                              partials);
        return hipGetLastError();
    };
    if (NCB == 1) return launch(gate_logits_mfma_kernel<1, 2>, 2);
    return launch(gate_logits_mfma_kernel<2, 2>, 2);
}

hipError_t gate_init_kernels() {
    hipError_t e = ensure_lds_limit(reinterpret_cast<const void*>(&gate_logits_mfma_kernel<1, 2>), 4 * gate_region_bytes(1, 2));
    if (e != hipSuccess) return e;
    return ensure_lds_limit(reinterpret_cast<const void*>(&gate_logits_mfma_kernel<2, 2>), 4 * gate_region_bytes(2, 2));
}

hipError_t launch_gate_topk(const float* partials, int KS, const float* bias, int T, int N, int k,
                            float inv_temperature, int32_t* topk_idx, float* topk_w, float* logits,
                            int32_t* chunk_counts, hipStream_t stream) {
    if (padded_adapters(N) == 32)
        gate_topk_kernel<32><<<bucket_chunks(T), kTopkWaves * 64, 0, stream>>>(
            partials, KS, bias, T, N, k, inv_temperature, topk_idx, topk_w, logits, chunk_counts);
    else
        gate_topk_kernel<64><<<bucket_chunks(T), kTopkWaves * 64, 0, stream>>>(
            partials, KS, bias, T, N, k, inv_temperature, topk_idx, topk_w, logits, chunk_counts);
    return hipGetLastError();
}

}  // namespace meteora
