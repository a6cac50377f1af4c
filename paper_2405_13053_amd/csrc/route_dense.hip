// Mid-sized batches (a few hundred to a few thousand tokens): routing and LoRA shrink without bucket lists.
//
// At these sizes the gate logits, top-k, bucketing, grouped shrink and its finalize are five short launches
// that each read little and sit on launch and fill/drain time.  Here one MFMA launch computes, for every
// token, the split-bf16 gate logits (Sec. 3.1) AND x * A_i for EVERY adapter i (the shrink of Eq. 2 before
// the selection): x[T, d_in] times Wcat[3*NP + N*r, d_in]^T, a 320-column GEMM at N = 28, r = 8, whose
// extra flops (N/k times the selected adapters') are cheap next to a second gathered pass over x.
// This file's kernel then, per token, adds the K-splits in a fixed order, picks the top-k (ties to the lowest
// index), takes the softmax over the k selected (Eq. 3) and writes the token's row of the dense expand
// operand: hdense[t, a*r + q] = bf16(scale * w * h) for the selected adapters a, zero elsewhere.
// The values are those of the bucketed path up to fp32 summation order; the ranking routine is the same.
#include "common.hpp"
#include "kernels.hpp"
#include "topk_key.hpp"
#include "dense_logits.hpp"

namespace meteora {

constexpr int kWcatMaxRows = 640;
constexpr int kSelNP = 32;   // gate columns per term in Wcat: the path takes N <= 32 only (more adapters exceed its row limit)

// WIDE (more than 4 K splits): twice as many splits' loads in flight
// Members of one launch (blockIdx.y): layers that share x and the shapes T, N, r, k, S, CR, each with its own
// partial products, bias and outputs.
struct SelectMembers {
    struct Member {
        const float* part;   // [S][T][CR]
        const float* bias;   // [N] or NULL
        int32_t* topk_idx;   // [T,k]
        float* topk_w;       // [T,k]
        bf16_t* hdense;      // [T][ext_stride] or NULL
        float* hs;           // [T,k,r] or NULL
    } m[kMaxDecodeGroup];
};

// Independent wavefronts, no LDS and no barrier: a wavefront ranks two tokens (one per half, NP = 32 lanes each)
// and writes their rows, a 16-byte piece (8 columns of one adapter, r % 8 == 0) per lane and round.  Two rounds of
// loads: the gate terms of every K split, then the selected adapters' shrink columns.  (A workgroup form of it — 16
// tokens per workgroup, the choices handed from the ranking wavefront to the row writers through LDS behind a
// barrier — took 7.9 us at config 2 and 9.3 us at T = 1024 where this one takes 5.6 and 5.3.)
constexpr int kSelThreads = 256;
template <bool WIDE>
__global__ __launch_bounds__(kSelThreads) void route_dense_select_kernel(const SelectMembers sm, int S, int CR, int T,
                                                                         int N, int r, int k, float inv_temperature,
                                                                         float scale, int ext_stride) {
    const float* __restrict__ part = sm.m[blockIdx.y].part;
    const float* __restrict__ bias = sm.m[blockIdx.y].bias;
    int32_t* __restrict__ topk_idx = sm.m[blockIdx.y].topk_idx;
    float* __restrict__ topk_w = sm.m[blockIdx.y].topk_w;
    bf16_t* __restrict__ hdense = sm.m[blockIdx.y].hdense;
    float* __restrict__ hs = sm.m[blockIdx.y].hs;
    constexpr int NP = kSelNP;
    const int lane = threadIdx.x & 63, col = lane & (NP - 1), sub = lane / NP;
    const int t0 = (blockIdx.x * (kSelThreads / 64) + (threadIdx.x >> 6)) * 2;
    if (t0 >= T) return;   // the whole wavefront
    float g[1];
    const int lt[1] = {sub};
    dense_logits<NP, 1, WIDE ? 8 : 4>(part, S, CR, bias, T, N, t0, lt, col, g);
    int sel_i[1];
    float sel_w[1];
    wave_topk_softmax<NP, 1>(g, lane, N, k, inv_temperature, sel_i, sel_w);   // lane col = s < k: the s-th choice
    if (col < k && t0 + sub < T) {
        topk_idx[(size_t)(t0 + sub) * k + col] = sel_i[0];
        topk_w[(size_t)(t0 + sub) * k + col] = sel_w[0];
    }
    const int C8 = ext_stride / 8;
    for (int e0 = 0; e0 < 2 * C8; e0 += 64) {   // uniform trip count: every lane takes part in the exchanges
        const int e = e0 + lane;
        const bool active = e < 2 * C8;
        const int th = active ? e / C8 : 0, c0 = active ? (e - th * C8) * 8 : 0;
        const int t = active ? t0 + th : T;
        const int a = c0 / r;
        bool hit = false;
        float sw = 0.f;
        int slot = 0;
        for (int s = 0; s < k; ++s) {
            const int ai = __shfl(sel_i[0], th * NP + s);
            const float wi = __shfl(sel_w[0], th * NP + s);
            if (c0 < N * r && ai == a) { hit = true; sw = scale * wi; slot = s; }
        }
        u32x4 pk = {0u, 0u, 0u, 0u};
        if (hit && t < T) {
            f32x4 h0 = {0.f, 0.f, 0.f, 0.f}, h1 = {0.f, 0.f, 0.f, 0.f};
            const float* src = part + (size_t)t * CR + 3 * NP + c0;
            constexpr int HU = WIDE ? 8 : 4;
            for (int s0 = 0; s0 < S; s0 += HU) {   // splits in order, 2 * HU loads in flight
                f32x4 v0[HU], v1[HU];
#pragma unroll
                for (int u = 0; u < HU; ++u) {
                    const float* p = src + (size_t)min(s0 + u, S - 1) * T * CR;
                    v0[u] = *reinterpret_cast<const f32x4*>(p);
                    v1[u] = *reinterpret_cast<const f32x4*>(p + 4);
                }
#pragma unroll
                for (int u = 0; u < HU; ++u)
                    if (s0 + u < S) { h0 += v0[u]; h1 += v1[u]; }
            }
            if (hs != nullptr) {   // fp32 rows for the expand inside a split-K reduction
                float* dst = hs + ((size_t)t * k + slot) * r + (c0 - a * r);
                *reinterpret_cast<f32x4*>(dst) = f32x4{sw * h0[0], sw * h0[1], sw * h0[2], sw * h0[3]};
                *reinterpret_cast<f32x4*>(dst + 4) = f32x4{sw * h1[0], sw * h1[1], sw * h1[2], sw * h1[3]};
            }
            pk[0] = pack_bf16x2(sw * h0[0], sw * h0[1]); pk[1] = pack_bf16x2(sw * h0[2], sw * h0[3]);
            pk[2] = pack_bf16x2(sw * h1[0], sw * h1[1]); pk[3] = pack_bf16x2(sw * h1[2], sw * h1[3]);
        }
        if (hdense != nullptr && t < T) *reinterpret_cast<u32x4*>(hdense + (size_t)t * ext_stride + c0) = pk;
    }
}

// Shapes the dense path takes, whatever the batch size (decides whether Wcat is part of the packed weights).
bool route_dense_possible(int d_in, int N, int r, bool bf16) {
    // up to 640 rows of Wcat (28 adapters of rank 16: 544): measured against the bucketed sequence on 4096 -> 4096,
    // rank 16, the dense forms are faster or equal from T = 8 to 8192 (T = 128: 35 against 55 us)
    return bf16 && r % 8 == 0 && d_in % 64 == 0 && padded_adapters(N) == kSelNP && prep_wcat_rows(N, r) <= kWcatMaxRows;
}

// Measured against the bucketed sequence (gate logits, top-k, scatter, whole-K shrink) on 4096 -> 4096 and
// 14336 -> 4096 at T = 12000 ... 65536: with 320 rows of Wcat (28 adapters of rank 8) the dense form wins at every
// size (whole call: 357.6 against 377.0 us at T = 12000, 918.9 against 984.8 at 32768, 1830 against 1985 at 65536);
// with 544 rows (rank 16) it wins by 0.3-8% where the products' 128 x 320 tiles fill the CUs (T = 16384: 496.7 against
// 515.2 us, 1631 against 1680 with d_in = 14336) and loses where they do not (T = 12000, d_in = 14336: 188 workgroups
// of a full K sweep each, 1269 against 1231 us).
bool route_dense_applies(int T, int d_in, int N, int r, bool bf16) {
    const int CR = prep_wcat_rows(N, r);
    if (!route_dense_possible(d_in, N, r, bf16) || T <= 64 || !gemm_dense_splitk_ok(T, d_in, CR)) return false;
    if (T <= kRouteDenseMaxTokens || CR <= 320) return true;
    const int64_t wgs = (int64_t)ceil_div(T, 128) * ceil_div(CR, 320) * gemm_dense_splits(T, d_in, CR);
    return wgs * 10 >= (wgs + 255) / 256 * 256 * 9;   // at least 90% of the CUs' slots over the launch
}

size_t route_dense_part_bytes(int T, int d_in, int N, int r, bool bf16) {
    if (!route_dense_applies(T, d_in, N, r, bf16)) return 0;
    const int CR = prep_wcat_rows(N, r);
    return (size_t)gemm_dense_splits(T, d_in, CR) * T * CR * sizeof(float);
}

hipError_t launch_route_dense_products(const void* x, const void* wcat, int T, int d_in, int N, int r, float* part,
                                       hipStream_t stream) {
    return launch_gemm_dense_splitk(x, wcat, T, d_in, prep_wcat_rows(N, r), part, stream);
}

static hipError_t launch_select(const SelectMembers& sm, int G, int S, int T, int N, int r, int k,
                                float inv_temperature, float scale, int ext_stride, hipStream_t stream) {
    const int CR = prep_wcat_rows(N, r);
    const dim3 grid(ceil_div(T, 2 * (kSelThreads / 64)), G);
    if (S > 4)
        route_dense_select_kernel<true><<<grid, kSelThreads, 0, stream>>>(sm, S, CR, T, N, r, k, inv_temperature, scale,
                                                                          ext_stride);
    else
        route_dense_select_kernel<false><<<grid, kSelThreads, 0, stream>>>(sm, S, CR, T, N, r, k, inv_temperature, scale,
                                                                           ext_stride);
    return hipGetLastError();
}

hipError_t launch_route_dense_select(const float* part, const float* bias, int T, int d_in, int N, int r, int k,
                                     float inv_temperature, float scale, int32_t* topk_idx, float* topk_w,
                                     void* hdense, int ext_stride, hipStream_t stream, float* hs, int splits) {
    const int S = splits > 0 ? splits : gemm_dense_splits(T, d_in, prep_wcat_rows(N, r));
    SelectMembers sm{};
    sm.m[0] = {part, bias, topk_idx, topk_w, (bf16_t*)hdense, hs};
    return launch_select(sm, 1, S, T, N, r, k, inv_temperature, scale, ext_stride, stream);
}

// The members of a group in one launch: mem[g].gpartial holds x * Wcat_g^T in S splits, results go to mem[g].idx,
// mem[g].w and mem[g].hs.
hipError_t launch_route_dense_select_group(const DecodeMember* mem, int G, int S, int T, int N, int r, int k,
                                           float inv_temperature, float scale, hipStream_t stream) {
    if (G < 1 || G > kMaxDecodeGroup || S < 1) return hipErrorInvalidValue;
    SelectMembers sm{};
    for (int g = 0; g < G; ++g) sm.m[g] = {mem[g].gpartial, mem[g].bias, mem[g].idx, mem[g].w, nullptr, mem[g].hs};
    // ext_stride only enumerates the 8-column pieces of a token's N*r shrink values here (no hdense is written)
    return launch_select(sm, G, S, T, N, r, k, inv_temperature, scale, (int)align_up((size_t)N * r, 64), stream);
}

}  // namespace meteora
