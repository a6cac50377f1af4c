// Base projection of the layer, first term of Eq. 1 / Eq. 2:  out = x * W_base, with W stored
// [d_out, d_in] so both operands are contiguous along the contraction.
#include <stdlib.h>
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

// Sum the fp32 split-K tiles in a fixed order (deterministic), add the old output if asked, round once.
__global__ __launch_bounds__(256) void gemm_splitk_reduce_kernel(const float* __restrict__ partial, int nsplit,
                                                                 int T, int d_out, bf16_t* __restrict__ out,
                                                                 int accumulate) {
    const size_t n8 = (size_t)T * d_out / 8;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < nsplit; ++s) {
        const float* src = partial + (size_t)s * T * d_out + i * 8;
        lo += *reinterpret_cast<const f32x4*>(src);
        hi += *reinterpret_cast<const f32x4*>(src + 4);
    }
    u32x4* dst = reinterpret_cast<u32x4*>(out) + i;
    if (accumulate) {
        const u32x4 old = *dst;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            lo[2 * e] += bf16_bits_to_float(old[e] & 0xffffu);
            lo[2 * e + 1] += bf16_bits_to_float(old[e] >> 16);
            hi[2 * e] += bf16_bits_to_float(old[2 + e] & 0xffffu);
            hi[2 * e + 1] += bf16_bits_to_float(old[2 + e] >> 16);
        }
    }
    u32x4 pk;
    pk[0] = pack_bf16x2(lo[0], lo[1]); pk[1] = pack_bf16x2(lo[2], lo[3]);
    pk[2] = pack_bf16x2(hi[0], hi[1]); pk[3] = pack_bf16x2(hi[2], hi[3]);
    *dst = pk;
}

// Decode: the fixed-order sum of the split-K tiles plus the LoRA expand of Eq. 2 from the fp32 shrink outputs,
//   out[t, c] = bf16( sum_s partial[s][t][c] + sum_slot sum_q hs[t][slot][q] * B[idx[t][slot]][q][c] ),
// hs = scale * w * h.  A thread owns 8 consecutive columns of one token: B rows are read as 16-byte pieces,
// coalesced across the threads of a token.
struct ReduceExpandArgs {
    struct Member {
        const float* partial;   // [S][T][d_out]
        const float* hs;        // [T,k,r]
        const int32_t* idx;     // [T,k]
        const bf16_t* B;        // [N,r,d_out]
        bf16_t* out;            // [T,d_out]
        int d_out, block0;      // first workgroup of this member
    } m[kMaxDecodeGroup];
    int G;
};

__global__ __launch_bounds__(256) void gemm_splitk_reduce_expand_kernel(const ReduceExpandArgs ra, int nsplit, int T,
                                                                        int k, int r) {
    int g = 0;
    for (int i = 1; i < ra.G; ++i)
        if ((int)blockIdx.x >= ra.m[i].block0) g = i;   // uniform
    const float* __restrict__ partial = ra.m[g].partial;
    const float* __restrict__ hs = ra.m[g].hs;
    const int32_t* __restrict__ idx = ra.m[g].idx;
    const bf16_t* __restrict__ B = ra.m[g].B;
    bf16_t* __restrict__ out = ra.m[g].out;
    const int d_out = ra.m[g].d_out;
    const int c8 = d_out / 8;
    const size_t i = (size_t)(blockIdx.x - ra.m[g].block0) * 256 + threadIdx.x;
    if (i >= (size_t)T * c8) return;
    const int t = (int)(i / c8), c = (int)(i - (size_t)t * c8) * 8;
    f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < nsplit; s0 += 8) {   // tiles in order, 8 tiles' loads in flight
        f32x4 v0[8], v1[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float* src = partial + ((size_t)min(s0 + u, nsplit - 1) * T + t) * d_out + c;
            v0[u] = *reinterpret_cast<const f32x4*>(src);
            v1[u] = *reinterpret_cast<const f32x4*>(src + 4);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (s0 + u < nsplit) { lo += v0[u]; hi += v1[u]; }
    }
    for (int slot = 0; slot < k; ++slot) {
        const int a = idx[(size_t)t * k + slot];
        const float* h = hs + ((size_t)t * k + slot) * r;
        const bf16_t* Ba = B + (size_t)a * r * d_out + c;
        for (int q0 = 0; q0 < r; q0 += 8) {   // r % 8 == 0; 8 rows of B in flight
            u32x4 b[8];
            float hv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                b[u] = *reinterpret_cast<const u32x4*>(Ba + (size_t)(q0 + u) * d_out);
                hv[u] = h[q0 + u];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                lo[0] = fmaf(hv[u], bf16_bits_to_float(b[u][0] & 0xffffu), lo[0]);
                lo[1] = fmaf(hv[u], bf16_bits_to_float(b[u][0] >> 16), lo[1]);
                lo[2] = fmaf(hv[u], bf16_bits_to_float(b[u][1] & 0xffffu), lo[2]);
                lo[3] = fmaf(hv[u], bf16_bits_to_float(b[u][1] >> 16), lo[3]);
                hi[0] = fmaf(hv[u], bf16_bits_to_float(b[u][2] & 0xffffu), hi[0]);
                hi[1] = fmaf(hv[u], bf16_bits_to_float(b[u][2] >> 16), hi[1]);
                hi[2] = fmaf(hv[u], bf16_bits_to_float(b[u][3] & 0xffffu), hi[2]);
                hi[3] = fmaf(hv[u], bf16_bits_to_float(b[u][3] >> 16), hi[3]);
            }
        }
    }
    u32x4 pk;
    pk[0] = pack_bf16x2(lo[0], lo[1]); pk[1] = pack_bf16x2(lo[2], lo[3]);
    pk[2] = pack_bf16x2(hi[0], hi[1]); pk[3] = pack_bf16x2(hi[2], hi[3]);
    reinterpret_cast<u32x4*>(out)[i] = pk;
}

// Skinny batches (decode): one 64-row tile per 64 output columns leaves most CUs idle while W streams
// from HBM, so K is split over workgroups.  Returns the number of main-K splits (0 = do not split).
int gemm_splitk_splits(int T, int d_in, int d_out, bool bf16) {
    if (!bf16 || T < 1 || T > 64 || d_in % kGemmBK != 0) return 0;
    const int tiles = ceil_div(T, 64) * ceil_div(d_out, 64), nk = d_in / kGemmBK;
    if (tiles >= 512 || nk < 8) return 0;
    int S = ceil_div(512, tiles);   // about two workgroups per CU (measured: 384 to 1536 tried)
    if (S > nk / 4) S = nk / 4;
    return S >= 2 ? S : 0;
}

size_t gemm_splitk_bytes(int T, int d_in, int d_out, bool bf16) {
    const int S = gemm_splitk_splits(T, d_in, d_out, bf16);
    return S == 0 ? 0 : (size_t)(S + 1) * T * d_out * sizeof(float);   // +1: the expand extension
}

template <int MI, int NI>
static hipError_t launch_mfma(GemmArgs a, hipStream_t stream) {
    constexpr int BM = MI * 64, BN = NI * 64;
    constexpr int smem = gemm_lds_bytes<MI, NI>();
    hipError_t e0 = ensure_lds_limit(reinterpret_cast<const void*>(&gemm_mfma_kernel<MI, NI>), smem);
    if (e0 != hipSuccess) return e0;
    e0 = ensure_lds_limit(reinterpret_cast<const void*>(&gemm_mfma_dma_kernel<MI, NI>), smem);
    if (e0 != hipSuccess) return e0;
    a.tiles_m = ceil_div(a.T, BM);
    a.tiles_n = ceil_div(a.d_out, BN);
    // the pipelined kernel needs whole K tiles and byte offsets inside x and W that fit 32 bits
    const uint64_t widest = (uint64_t)(a.d_in > a.ext_stride ? a.d_in : a.ext_stride) * 2;
    const bool dma_ok = a.d_in % kGemmBK == 0 && ((uint64_t)a.T + BM) * widest < (1ull << 32) &&
                        ((uint64_t)a.d_out + BN) * widest < (1ull << 32);
    if (dma_ok && a.partial != nullptr) {
        const int nsplit = a.splits + (a.ext_k > 0 ? 1 : 0);
        gemm_mfma_dma_kernel<MI, NI><<<dim3(a.tiles_m * a.tiles_n, nsplit), 256, smem, stream>>>(a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        const size_t n8 = (size_t)a.T * a.d_out / 8;
        gemm_splitk_reduce_kernel<<<(unsigned)((n8 + 255) / 256), 256, 0, stream>>>(a.partial, nsplit, a.T, a.d_out,
                                                                                   a.out, a.accumulate);
    } else if (dma_ok && ((MI == 4 && NI == 4) || (MI == 2 && NI == 2))) {
        constexpr int M3 = MI == 4 ? 4 : 2;   // the instantiations of the three-deep-ring kernel that exist
        // the epilogue form is a compile-time parameter of this kernel: plain store (the layer's GEMM) or accumulate
        auto go = [&](auto kern) -> hipError_t {
            const hipError_t e1 = ensure_lds_limit(reinterpret_cast<const void*>(kern), gemm_w3_lds_bytes<M3, M3>());
            if (e1 != hipSuccess) return e1;
            kern<<<a.tiles_m * a.tiles_n, 256, gemm_w3_lds_bytes<M3, M3>(), stream>>>(a);
            return hipSuccess;
        };
        const hipError_t e1 = a.accumulate ? go(&gemm_mfma_w3_kernel<M3, M3, kEpiAccumulate>)
                                           : go(&gemm_mfma_w3_kernel<M3, M3, kEpiStore>);
        if (e1 != hipSuccess) return e1;
    } else if (dma_ok) {
        gemm_mfma_dma_kernel<MI, NI><<<a.tiles_m * a.tiles_n, 256, smem, stream>>>(a);
    } else {
        gemm_mfma_kernel<MI, NI><<<a.tiles_m * a.tiles_n, 256, smem, stream>>>(a);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Dense routing operand: partial[split][T][rows] = x[T, K-range of split] * Wcat[rows, same K]^T in fp32,
// no reduction (the select kernel adds the splits in order).
// ------------------------------------------------------------------------------------------
// Up to 4096 tokens: 128 x 128 tiles, two workgroups per CU (one computes while the other waits for its
// loads), about 384 workgroups; above: 128 x 320 tiles (x is read once), one workgroup per CU.  Both with
// the three-deep W ring.  Measured on T = 4096 and 8192, d_in = 4096 and 14336.
static bool dense_small_tiles(int T) { return T <= 4096; }

bool gemm_dense_splitk_ok(int T, int d_in, int rows) {
    const uint64_t widest = (uint64_t)d_in * 2;
    return d_in % kGemmBK == 0 && rows % 8 == 0 && ((uint64_t)T + 2 * 64) * widest < (1ull << 32) &&
           ((uint64_t)rows + 5 * 64) * widest < (1ull << 32);
}

int gemm_dense_splits(int T, int d_in, int rows) {
    const bool small = dense_small_tiles(T);
    const int tiles = ceil_div(T, 128) * ceil_div(rows, small ? 128 : 320), nk = d_in / kGemmBK;
    int S = ((small ? 384 : 256) + tiles / 2) / tiles;
    if (S > nk / 4) S = nk / 4;                // at least 4 K tiles per split
    if (S > 8) S = 8;                          // more splits cost the kernel that adds them more than they save here
    return S < 1 ? 1 : S;
}

template <int MI, int NI>
static hipError_t launch_dense(GemmArgs a, hipStream_t stream) {   // three-deep W ring, fp32 split-K tiles
    constexpr int smem = gemm_w3_lds_bytes<MI, NI>();
    auto kern = &gemm_mfma_w3_kernel<MI, NI, kEpiPartial>;
    const hipError_t ea = ensure_lds_limit(reinterpret_cast<const void*>(kern), smem);
    if (ea != hipSuccess) return ea;
    a.tiles_m = ceil_div(a.T, MI * 64);
    a.tiles_n = ceil_div(a.d_out, NI * 64);
    kern<<<dim3(a.tiles_m * a.tiles_n, a.splits), 256, smem, stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_gemm_dense_splitk(const void* x, const void* Wcat, int T, int d_in, int rows, float* partial,
                                    hipStream_t stream) {
    if (!gemm_dense_splitk_ok(T, d_in, rows)) return hipErrorInvalidValue;
    GemmArgs a{};
    a.x = (const bf16_t*)x; a.W = (const bf16_t*)Wcat; a.T = T; a.d_in = d_in; a.d_out = rows;
    a.partial = partial;
    a.splits = gemm_dense_splits(T, d_in, rows);
    a.tiles_per_split = ceil_div(d_in / kGemmBK, a.splits);
    return dense_small_tiles(T) ? launch_dense<2, 2>(a, stream) : launch_dense<2, 5>(a, stream);
}

// Several matrices in one split-K launch (few-tile batches): ops[i].partial[s][T][rows_i] = x * W_i^T over the K
// range of split s, the 128-column tiles of all of them in one grid.  The tiles are 128 rows high up to 128 tokens
// and 256 rows above (a wavefront's 128 x 64 piece needs 0.75 fragment reads per MFMA against 1.0 at 128 x 128),
// one workgroup per CU at most, so the number of K splits is capped for them.  Measured, 256 x 128 against 128 x
// 128 tiles, whole call at 4096 -> 4096: T = 160 24.2 against 26.1 us, T = 400 34.5 against 43.6, T = 512 37.1
// against 44.6, T = 640 44.1 against 50.7; at 14336 -> 4096 T = 512 77.3 against 97.9.
bool gemm_multi_big_rows(int T) { return T > 128; }
int gemm_multi_cap_splits(int T, int col_tiles, int S) {
    if (!gemm_multi_big_rows(T)) return S;
    const int cap = 256 / (ceil_div(T, 256) * (col_tiles > 0 ? col_tiles : 1));   // 256 CUs
    return S > cap ? (cap > 0 ? cap : 1) : S;
}

hipError_t launch_gemm_dense_splitk_multi(const void* x, const DenseOperand* ops, int n_ops, int S, int T, int d_in,
                                          hipStream_t stream) {
    if (S < 1 || n_ops < 1 || n_ops > GemmArgs::kMaxSegments) return hipErrorInvalidValue;
    GemmArgs a{};
    a.x = (const bf16_t*)x; a.T = T; a.d_in = d_in;
    a.splits = S; a.tiles_per_split = ceil_div(d_in / kGemmBK, S);
    int tile0 = 0;
    for (int i = 0; i < n_ops; ++i) {
        if (!gemm_dense_splitk_ok(T, d_in, ops[i].rows)) return hipErrorInvalidValue;
        a.seg[i] = {(const bf16_t*)ops[i].W, ops[i].partial, ops[i].rows, tile0};
        tile0 += ceil_div(ops[i].rows, 128);
    }
    a.nseg = n_ops;
    a.W = a.seg[0].W; a.d_out = a.seg[0].rows; a.partial = a.seg[0].partial;   // replaced per workgroup
    a.tiles_n = tile0;
    if (gemm_multi_big_rows(T)) {
        if (((uint64_t)T + 256) * ((uint64_t)d_in * 2) >= (1ull << 32)) return hipErrorInvalidValue;
        constexpr int smem = gemm_w3_lds_bytes<4, 2>();
        const hipError_t ea = ensure_lds_limit(reinterpret_cast<const void*>(&gemm_mfma_w3_kernel<4, 2, kEpiPartial>), smem);
        if (ea != hipSuccess) return ea;
        a.tiles_m = ceil_div(T, 256);
        gemm_mfma_w3_kernel<4, 2, kEpiPartial><<<dim3(a.tiles_m * a.tiles_n, S), 256, smem, stream>>>(a);
        return hipGetLastError();
    }
    constexpr int smem = gemm_w3_lds_bytes<2, 2>();
    const hipError_t ea = ensure_lds_limit(reinterpret_cast<const void*>(&gemm_mfma_w3_kernel<2, 2, kEpiPartial>), smem);
    if (ea != hipSuccess) return ea;
    a.tiles_m = ceil_div(T, 128);
    gemm_mfma_w3_kernel<2, 2, kEpiPartial><<<dim3(a.tiles_m * a.tiles_n, S), 256, smem, stream>>>(a);
    return hipGetLastError();
}

// Decode in two launches: (1) the main K splits of x * W^T with the rows of Wcat as extra column
// tiles (fp32 tiles into `partial` and `gpartial`), (2) routing on the gate tiles, then the reduction with the
// expand from the shrink tiles (route_small.hip).  A group of G layers that share x runs through the same two
// launches: the column tiles of all their W and Wcat form one grid, all with the same number S of K splits.
int gemm_group_splits(int T, int d_in, const int* d_out, int G, int gate_rows) {
    if (T < 1 || T > 64 || d_in % kGemmBK != 0) return 0;
    const int nk = d_in / kGemmBK;
    if (nk < 8) return 0;
    int tiles = 0;
    for (int g = 0; g < G; ++g) tiles += ceil_div(d_out[g], 64) + ceil_div(gate_rows, 64);
    if (G == 1) return gemm_splitk_splits(T, d_in, d_out[0], true);   // same split as the single-layer call
    int S = ceil_div(512, tiles);   // about two workgroups per CU (measured: 384 to 1536 tried)
    if (S > nk / 4) S = nk / 4;
    return S < 1 ? 1 : S;
}

hipError_t launch_gemm_decode_main(const void* x, const DecodeMember* mem, int G, int gate_rows, int S, int T,
                                   int d_in, hipStream_t stream) {
    if (S <= 0 || gate_rows % 8 != 0 || G < 1 || 2 * G > GemmArgs::kMaxSegments) return hipErrorInvalidValue;
    GemmArgs a{};
    a.x = (const bf16_t*)x; a.T = T; a.d_in = d_in;
    a.splits = S; a.tiles_per_split = ceil_div(d_in / kGemmBK, S);
    const uint64_t widest = (uint64_t)d_in * 2;
    if (d_in % kGemmBK != 0 || ((uint64_t)T + 64) * widest >= (1ull << 32)) return hipErrorInvalidValue;
    int tile0 = 0;
    for (int g = 0; g < G; ++g) {
        if (((uint64_t)mem[g].d_out + 64) * widest >= (1ull << 32)) return hipErrorInvalidValue;
        a.seg[2 * g] = {(const bf16_t*)mem[g].W, mem[g].partial, mem[g].d_out, tile0};
        tile0 += ceil_div(mem[g].d_out, 64);
        a.seg[2 * g + 1] = {(const bf16_t*)mem[g].wg3, mem[g].gpartial, gate_rows, tile0};
        tile0 += ceil_div(gate_rows, 64);
    }
    a.nseg = 2 * G;
    a.W = a.seg[0].W; a.d_out = a.seg[0].rows; a.partial = a.seg[0].partial;   // replaced per workgroup
    constexpr int smem = gemm_lds_bytes<1, 1>();
    const hipError_t ea = ensure_lds_limit(reinterpret_cast<const void*>(&gemm_mfma_dma_kernel<1, 1>), smem);
    if (ea != hipSuccess) return ea;
    a.tiles_m = ceil_div(T, 64);
    a.tiles_n = tile0;
    gemm_mfma_dma_kernel<1, 1><<<dim3(a.tiles_m * a.tiles_n, S), 256, smem, stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_gemm_decode_finish(const DecodeMember* mem, int G, int S, int T, int k, int r,
                                     hipStream_t stream) {
    if (S <= 0 || r % 8 != 0 || G < 1 || G > kMaxDecodeGroup) return hipErrorInvalidValue;
    ReduceExpandArgs ra{};
    unsigned blocks = 0;
    for (int g = 0; g < G; ++g) {
        ra.m[g] = {mem[g].partial, mem[g].hs, mem[g].idx, (const bf16_t*)mem[g].B, (bf16_t*)mem[g].out, mem[g].d_out,
                   (int)blocks};
        blocks += (unsigned)(((size_t)T * mem[g].d_out / 8 + 255) / 256);
    }
    ra.G = G;
    gemm_splitk_reduce_expand_kernel<<<blocks, 256, 0, stream>>>(ra, S, T, k, r);
    return hipGetLastError();
}

bool gemm_fuses_expand(bool bf16) { return bf16; }

template <int MI, int NI>
static hipError_t init_tile_kernels() {
    hipError_t e = ensure_lds_limit(reinterpret_cast<const void*>(&gemm_mfma_kernel<MI, NI>), gemm_lds_bytes<MI, NI>());
    if (e != hipSuccess) return e;
    return ensure_lds_limit(reinterpret_cast<const void*>(&gemm_mfma_dma_kernel<MI, NI>), gemm_lds_bytes<MI, NI>());
}

// every kernel of this file that a launcher above may start with more than the default dynamic LDS
hipError_t gemm_init_kernels() {
    hipError_t e = init_tile_kernels<4, 4>();
    if (e == hipSuccess) e = init_tile_kernels<2, 2>();
    if (e == hipSuccess) e = init_tile_kernels<1, 1>();
    auto lim = [&](auto kern, int bytes) {
        if (e == hipSuccess) e = ensure_lds_limit(reinterpret_cast<const void*>(kern), bytes);
    };
    lim(&gemm_mfma_w3_kernel<4, 4, kEpiStore>, gemm_w3_lds_bytes<4, 4>());
    lim(&gemm_mfma_w3_kernel<4, 4, kEpiAccumulate>, gemm_w3_lds_bytes<4, 4>());
    lim(&gemm_mfma_w3_kernel<4, 2, kEpiStore>, gemm_w3_lds_bytes<4, 2>());
    lim(&gemm_mfma_w3_kernel<4, 2, kEpiAccumulate>, gemm_w3_lds_bytes<4, 2>());
    lim(&gemm_mfma_w3_kernel<4, 2, kEpiPartial>, gemm_w3_lds_bytes<4, 2>());
    lim(&gemm_mfma_w3_kernel<2, 2, kEpiStore>, gemm_w3_lds_bytes<2, 2>());
    lim(&gemm_mfma_w3_kernel<2, 2, kEpiAccumulate>, gemm_w3_lds_bytes<2, 2>());
    lim(&gemm_mfma_w3_kernel<2, 2, kEpiPartial>, gemm_w3_lds_bytes<2, 2>());
    lim(&gemm_mfma_w3_kernel<2, 5, kEpiPartial>, gemm_w3_lds_bytes<2, 5>());
    return e;
}

hipError_t launch_gemm(const void* x, const void* W, int T, int d_in, int d_out, bool bf16,
                       const void* hdense, int ext_stride, const void* Bt, int ext_k,
                       void* out, int accumulate, float* splitk_ws, hipStream_t stream) {
    if (bf16) {
        if (hdense && (ext_stride % kGemmBK != 0 || ext_stride < ext_k || !Bt)) return hipErrorInvalidValue;
        GemmArgs a{};
        a.x = (const bf16_t*)x; a.W = (const bf16_t*)W; a.hd = (const bf16_t*)hdense; a.Bt = (const bf16_t*)Bt;
        a.out = (bf16_t*)out; a.T = T; a.d_in = d_in; a.d_out = d_out;
        a.ext_k = hdense ? ext_k : 0; a.ext_stride = ext_stride; a.accumulate = accumulate;
        const int S = splitk_ws ? gemm_splitk_splits(T, d_in, d_out, true) : 0;
        if (S > 0 && d_in > 0) {
            a.partial = splitk_ws;
            a.splits = S;
            a.tiles_per_split = ceil_div(d_in / kGemmBK, S);
            return launch_mfma<1, 1>(a, stream);
        }
        const int64_t big_tiles = (int64_t)ceil_div(T, 256) * ceil_div(d_out, 256);
        // 256 x 256 tiles once they fill most of the 256 CUs; below that 128 x 128 tiles keep more CUs busy
        // (T = 2048, 4096 -> 4096: 128 tiles of 256 x 256 take 109 us, 512 tiles of 128 x 128 take 98 us)
        // ... except a little more than one tile per CU (257 to 328 tiles), where the second, nearly empty round of
        // 256 x 256 tiles costs more than the smaller tiles' lower efficiency (4096 -> 4096: T = 4608, 288 tiles, 174
        // us against 155 with 128 x 128 tiles; T = 5120 176 against 163; 336 tiles and more: the big tiles win again,
        // and with two rounds or more they always do: 544 tiles 275 against 279)
        if (T > 128 && big_tiles >= 160 && !(big_tiles > 256 && big_tiles <= 328)) return launch_mfma<4, 4>(a, stream);
        // between the two: 256 x 128 tiles where 160 to 256 of them cover the output, one per CU (a wavefront's
        // 128 x 64 piece needs 0.75 fragment reads per MFMA against 1.0 at 128 x 128).  Measured against 128 x 128
        // tiles: T = 1280 at 4096 -> 4096 (160 tiles) 50.2 against 55.2 us, T = 2048 (256 tiles) 62.3 against 66.0,
        // T = 512 at 4096 -> 14336 59.2 against 63.6, T = 2048 at 14336 -> 4096 199 against 219; with 128 tiles
        // (T = 1024) 47.0 against 39.1, so not below 160
        const int64_t mid_tiles = (int64_t)ceil_div(T, 256) * ceil_div(d_out, 128);
        const uint64_t widest = (uint64_t)(d_in > ext_stride ? d_in : ext_stride) * 2;
        if (T > 128 && mid_tiles >= 160 && mid_tiles <= 256 && d_in % kGemmBK == 0 &&
            ((uint64_t)T + 256) * widest < (1ull << 32) && ((uint64_t)d_out + 128) * widest < (1ull << 32)) {
            a.tiles_m = ceil_div(T, 256);
            a.tiles_n = ceil_div(d_out, 128);
            auto go = [&](auto kern) -> hipError_t {
                const hipError_t e1 = ensure_lds_limit(reinterpret_cast<const void*>(kern), gemm_w3_lds_bytes<4, 2>());
                if (e1 != hipSuccess) return e1;
                kern<<<a.tiles_m * a.tiles_n, 256, gemm_w3_lds_bytes<4, 2>(), stream>>>(a);
                return hipGetLastError();
            };
            return a.accumulate ? go(&gemm_mfma_w3_kernel<4, 2, kEpiAccumulate>) : go(&gemm_mfma_w3_kernel<4, 2, kEpiStore>);
        }
        if (T > 64) return launch_mfma<2, 2>(a, stream);
        return launch_mfma<1, 1>(a, stream);
    }
    dim3 grid(ceil_div(d_out, 64), ceil_div(T, 64));
    gemm_fma_kernel<float><<<grid, 256, 0, stream>>>((const float*)x, (const float*)W, T, d_in, d_out,
                                                     (float*)out, accumulate);
    return hipGetLastError();
}

}  // namespace meteora
