// Small batches (decode: a few dozen tokens, fewer tokens than adapters is the paper's hard case,
// Sec. 3.3): top-k + softmax (Eq. 3) and the LoRA shrink h = x * A_a of the selected adapters in ONE
// launch, one workgroup per token, token-major.  With so few (token, slot) pairs the bucket lists buy
// nothing: a pair's A_a (d_in x r, contiguous) is streamed once by the token's own workgroup, so the
// top-k, scatter, shrink and finalize launches of the large-batch path (each on a ~2.5 us launch
// floor) collapse into this one.  Consumes the same K-slice logit partials as gate_topk_kernel, adds
// them in the same order and ranks with the same routine, so the routing is identical.
#include "common.hpp"
#include "kernels.hpp"
#include "topk_key.hpp"
#include "dense_logits.hpp"

namespace meteora {

constexpr int kSmallThreads = 1024;   // 16 wavefronts per token: the shrink is latency-bound, so many short loops
constexpr int kSmallWaves = kSmallThreads / 64;

template <int R8>   // R8 = r / 8: 16-byte pieces per row of A_a
__global__ __launch_bounds__(kSmallThreads) void route_shrink_small_kernel(
    const bf16_t* __restrict__ x, const float* __restrict__ partials, int KS, const float* __restrict__ bias,
    const bf16_t* __restrict__ A, int T, int d_in, int N, int NP, int k, float inv_temperature, float scale,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, bf16_t* __restrict__ hdense, int ext_stride) {
    constexpr int r = R8 * 8;
    constexpr int ROWS = 8 / R8;   // rows of A_a per slot whose loads are in flight together
    __shared__ int sel_idx[kMaxTopK];
    __shared__ float sel_w[kMaxTopK];
    __shared__ float red[kSmallWaves][kMaxTopK][r];
    const int t = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    // this token's row of the dense expand operand starts as zeros
    if (hdense != nullptr) {
        u32x4* row = reinterpret_cast<u32x4*>(hdense + (size_t)t * ext_stride);
        for (int i = threadIdx.x; i < ext_stride / 8; i += kSmallThreads) row[i] = u32x4{0u, 0u, 0u, 0u};
    }
    if (wave == 0) {   // top-k and softmax: lane = adapter
        float g = 0.f;
        if (lane < N) {
            for (int s0 = 0; s0 < KS; s0 += 16) {   // K-slices in order, 16 loads in flight
                float v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = s0 + u < KS ? partials[((size_t)(s0 + u) * T + t) * NP + lane] : 0.f;
#pragma unroll
                for (int u = 0; u < 16; ++u) g += v[u];
            }
            g += bias != nullptr ? bias[lane] : 0.f;
            if (g == 0.f) g = 0.f;   // -0 -> +0 so equal logits have equal keys
        }
        const float gg[1] = {g};
        int my_i[1];
        float my_w[1];
        wave_topk_softmax<64, 1>(gg, lane, N, k, inv_temperature, my_i, my_w);
        if (lane < k) {
            sel_idx[lane] = my_i[0];
            sel_w[lane] = my_w[0];
            topk_idx[(size_t)t * k + lane] = my_i[0];
            topk_w[(size_t)t * k + lane] = my_w[0];
        }
    }
    __syncthreads();

    // shrink: thread `tid` takes rows tid, tid + 1024, ... of A_a (r bf16 = R8 16-byte pieces each); two slots
    // at a time so that both adapters' loads are in flight together
    const bf16_t* xt = x + (size_t)t * d_in;
    for (int slot0 = 0; slot0 < k; slot0 += 2) {
        const bool two = slot0 + 1 < k;   // uniform
        const bf16_t* Aa0 = A + (size_t)sel_idx[slot0] * d_in * r;
        const bf16_t* Aa1 = A + (size_t)sel_idx[two ? slot0 + 1 : slot0] * d_in * r;
        float acc0[r], acc1[r];
#pragma unroll
        for (int q = 0; q < r; ++q) { acc0[q] = 0.f; acc1[q] = 0.f; }
        for (int i0 = threadIdx.x; i0 < d_in; i0 += kSmallThreads * ROWS) {
            u32x4 v0[ROWS][R8], v1[ROWS][R8];
            float xv[ROWS];
#pragma unroll
            for (int u = 0; u < ROWS; ++u) {
                const int i = i0 + kSmallThreads * u;
                const int ic = i < d_in ? i : d_in - 1;
                xv[u] = i < d_in ? to_float(xt[ic]) : 0.f;   // rows past the end contribute x = 0
#pragma unroll
                for (int c = 0; c < R8; ++c) {
                    v0[u][c] = reinterpret_cast<const u32x4*>(Aa0 + (size_t)ic * r)[c];
                    // an odd last slot (the only one with the top-1 strategy of App. A.1) has no partner: its half
                    // of the loads and of the arithmetic below is skipped
                    v1[u][c] = two ? reinterpret_cast<const u32x4*>(Aa1 + (size_t)ic * r)[c] : u32x4{0u, 0u, 0u, 0u};
                }
            }
#pragma unroll
            for (int u = 0; u < ROWS; ++u)
#pragma unroll
                for (int c = 0; c < R8; ++c)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int q = c * 8 + 2 * e;
                        acc0[q] = fmaf(xv[u], bf16_bits_to_float(v0[u][c][e] & 0xffffu), acc0[q]);
                        acc0[q + 1] = fmaf(xv[u], bf16_bits_to_float(v0[u][c][e] >> 16), acc0[q + 1]);
                        if (two) {
                            acc1[q] = fmaf(xv[u], bf16_bits_to_float(v1[u][c][e] & 0xffffu), acc1[q]);
                            acc1[q + 1] = fmaf(xv[u], bf16_bits_to_float(v1[u][c][e] >> 16), acc1[q + 1]);
                        }
                    }
        }
        // Wavefront sums of the 2r values a lane holds, in a fixed order.  A plain butterfly per value would cost
        // 6 cross-lane exchanges for each of them (the 16 wavefronts of the workgroup queue on the CU's one
        // exchange path: measured 3 us of a 12 us kernel).  Instead every halving step also halves the values a
        // lane carries: lanes whose bit `off` is clear keep the lower half and take the partner's lower half,
        // the others the upper halves; when one value per lane is left, plain steps finish the sum.  2r-1 (+1 or
        // 2) exchanges instead of 12r.  Lane l ends up with value index = its bits 5, 4, ... read as a number.
        float v[2 * r];
#pragma unroll
        for (int q = 0; q < r; ++q) { v[q] = acc0[q]; v[r + q] = acc1[q]; }
        int cnt = 2 * r, off = 32;
#pragma unroll
        for (; cnt > 1 && off >= 1; cnt >>= 1, off >>= 1) {
            const bool upper = (lane & off) != 0;
#pragma unroll
            for (int i = 0; i < cnt / 2; ++i) {
                const float give = upper ? v[i] : v[i + cnt / 2];
                const float keep = upper ? v[i + cnt / 2] : v[i];
                v[i] = keep + __shfl_xor(give, off);
            }
        }
#pragma unroll
        for (; off >= 1; off >>= 1) v[0] += __shfl_xor(v[0], off);   // lanes that still hold the same value index
        {
            // halving steps done: log2(2r), capped at 6; the value index is the top bits of the lane number
            constexpr int kSteps = (2 * r >= 64) ? 6 : (2 * r == 32 ? 5 : 4);
            const int vi = lane >> (6 - kSteps);
            if ((lane & ((1 << (6 - kSteps)) - 1)) == 0) {
                if (2 * r <= 64) {
                    const int slot = vi / r, q = vi - slot * r;
                    if (slot == 0 || two) red[wave][slot0 + slot][q] = v[0];
                }
            }
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < k * r; e += kSmallThreads) {
        const int slot = e / r, q = e - slot * r;
        float h = 0.f;
#pragma unroll
        for (int wv = 0; wv < kSmallWaves; ++wv) h += red[wv][slot][q];   // fixed order
        hdense[(size_t)t * ext_stride + sel_idx[slot] * r + q] = from_float<bf16_t>(scale * sel_w[slot] * h);
    }
}

// A group of layers that share x (same T, N, r, k, number of K splits): the operands of the decode tail per member.
struct RouteGroup {
    struct Member {
        const float* gpart;   // [S][T][rows of Wcat]
        const float* bias;
        int32_t* idx;
        float* w;
    } m[kMaxDecodeGroup];
};
struct FinishGroup {
    struct Member {
        const float* partial;   // [S][T][d_out]
        const bf16_t* B;        // [N, r, d_out]
        bf16_t* out;            // [T, d_out]
        int d_out;
    } m[kMaxDecodeGroup];
    int nsplit, chunks;         // K splits; stretches of kTailThreads * 8 columns per row of the widest member
};

// ------------------------------------------------------------------------------------------------------------
// Decode tail: everything of a decode-sized layer call after the one launch that streams W.  That launch computes,
// as fp32 K-split tiles, x * W^T and x * Wcat^T, the latter being the gate terms (Sec. 3.1) AND the shrink x * A_i
// of EVERY adapter (N * r columns: 4% more rows to stream than W alone at N = 28, r = 8, 5120 -> 5120).  What is
// left per token is a chain of two memory round trips, taken here by independent wavefronts with no LDS and no
// barrier: (1) the gate tiles -> logits, top-k, softmax (Eq. 3); (2) the selected adapters' shrink tiles and rows
// of B -> out = bf16( sum of the projection's split tiles + sum_slot sum_q (scale * w * h) * B ), Eq. 2 with one
// rounding.  A wavefront owns 64 x 8 consecutive output columns of one token and repeats the token's routing
// (a few hundred bytes) instead of waiting for another wavefront.  The routing is the routine every path shares.
// ------------------------------------------------------------------------------------------------------------

// one wavefront per workgroup (measured: 64, 128 and 256 threads per workgroup time the same)
constexpr int kTailThreads = 64;

template <int R8>   // r = 8 * R8
__global__ __launch_bounds__(kTailThreads) void decode_tail_kernel(int T, int N, int CR, int k, float inv_temperature,
                                                                   float scale, const RouteGroup rg,
                                                                   const FinishGroup fg) {
    constexpr int r = R8 * 8, NP = 32;
    constexpr int SLOTS = 64 / r;   // slots whose shrink values a wavefront holds at a time, one value per lane
    const int lane = threadIdx.x & 63;
    const int chunk = blockIdx.x % fg.chunks;
    int t = blockIdx.x / fg.chunks;
    const int member = t / T;
    t -= member * T;
    const int d_out = fg.m[member].d_out, c8 = d_out / 8, nsplit = fg.nsplit;
    if (chunk * kTailThreads >= c8) return;   // a narrower member of the group: nothing in this stretch
    const int gi = chunk * kTailThreads + threadIdx.x;
    const bool active = gi < c8;              // lanes past the row's end work on its last columns and do not store
    const int c = (active ? gi : c8 - 1) * 8;
    const float* __restrict__ gpart = rg.m[member].gpart;
    const bf16_t* __restrict__ B = fg.m[member].B;
    const float* partial = fg.m[member].partial + (size_t)t * d_out + c;
    const size_t pstride = (size_t)T * d_out;

    // the projection's split tiles do not depend on the routing: the first 8 go out first
    f32x4 pre0[8], pre1[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const float* src = partial + (size_t)min(u, nsplit - 1) * pstride;
        pre0[u] = *reinterpret_cast<const f32x4*>(src);
        pre1[u] = *reinterpret_cast<const f32x4*>(src + 4);
    }
    float g[1];
    const int lt[1] = {0};
    dense_logits<NP, 1, 8>(gpart, nsplit, CR, rg.m[member].bias, T, N, t, lt, lane & (NP - 1), g);
    int sel_i[1];
    float sel_w[1];
    wave_topk_softmax<NP, 1>(g, lane, N, k, inv_temperature, sel_i, sel_w);   // lane s < k: the s-th choice
    if (chunk == 0 && threadIdx.x < k) {   // the wavefronts of a token compute the same routing: one reports it
        rg.m[member].idx[(size_t)t * k + lane] = sel_i[0];
        rg.m[member].w[(size_t)t * k + lane] = sel_w[0];
    }
    f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 8; ++u)
        if (u < nsplit) { lo += pre0[u]; hi += pre1[u]; }
    for (int s0 = 8; s0 < nsplit; s0 += 8) {   // tiles in order, 8 tiles' loads in flight
        f32x4 v0[8], v1[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float* src = partial + (size_t)min(s0 + u, nsplit - 1) * pstride;
            v0[u] = *reinterpret_cast<const f32x4*>(src);
            v1[u] = *reinterpret_cast<const f32x4*>(src + 4);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (s0 + u < nsplit) { lo += v0[u]; hi += v1[u]; }
    }

    auto load_rows = [&](int slot, int q0, u32x4 (&b)[8]) {   // 8 rows of B of the slot's adapter, this lane's columns
        const int a = __builtin_amdgcn_readlane(sel_i[0], slot);
        const bf16_t* Ba = B + ((size_t)a * r + q0) * d_out + c;
#pragma unroll
        for (int u = 0; u < 8; ++u) b[u] = *reinterpret_cast<const u32x4*>(Ba + (size_t)u * d_out);
    };
    for (int s0 = 0; s0 < k; s0 += SLOTS) {
        const int ns = min(SLOTS, k - s0);
        // lane e holds scale * w * h of slot s0 + e / r, component e % r: the shrink tiles of that adapter's columns
        // of Wcat, added in split order
        const int my_slot = min(s0 + lane / r, k - 1);
        const int a_e = __shfl(sel_i[0], my_slot);
        const float w_e = __shfl(sel_w[0], my_slot);
        const float* hsrc = gpart + (size_t)t * CR + 3 * NP + a_e * r + (lane & (r - 1));
        float hv8[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) hv8[u] = hsrc[(size_t)min(u, nsplit - 1) * T * CR];
        u32x4 bcur[8];
        load_rows(s0, 0, bcur);   // the first rows of B are under way while the shrink tiles arrive
        float h = 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (u < nsplit) h += hv8[u];
        for (int p0 = 8; p0 < nsplit; p0 += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = hsrc[(size_t)min(p0 + u, nsplit - 1) * T * CR];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (p0 + u < nsplit) h += v[u];
        }
        const float hv = scale * w_e * h;
        const int ngroups = ns * R8;
        for (int j = 0; j < ngroups; ++j) {   // (slot, 8 rows) pieces; the next piece's loads go out before this one's FMAs
            u32x4 bnext[8];
            const bool more = j + 1 < ngroups;
            if (more) load_rows(s0 + (j + 1) / R8, ((j + 1) % R8) * 8, bnext);
            const int e0 = (j / R8) * r + (j % R8) * 8;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float hq = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(hv), e0 + u));
                lo[0] = fmaf(hq, bf16_bits_to_float(bcur[u][0] & 0xffffu), lo[0]);
                lo[1] = fmaf(hq, bf16_bits_to_float(bcur[u][0] >> 16), lo[1]);
                lo[2] = fmaf(hq, bf16_bits_to_float(bcur[u][1] & 0xffffu), lo[2]);
                lo[3] = fmaf(hq, bf16_bits_to_float(bcur[u][1] >> 16), lo[3]);
                hi[0] = fmaf(hq, bf16_bits_to_float(bcur[u][2] & 0xffffu), hi[0]);
                hi[1] = fmaf(hq, bf16_bits_to_float(bcur[u][2] >> 16), hi[1]);
                hi[2] = fmaf(hq, bf16_bits_to_float(bcur[u][3] & 0xffffu), hi[2]);
                hi[3] = fmaf(hq, bf16_bits_to_float(bcur[u][3] >> 16), hi[3]);
            }
            if (more) {
#pragma unroll
                for (int u = 0; u < 8; ++u) bcur[u] = bnext[u];
            }
        }
    }
    if (active) {
        u32x4 pk;
        pk[0] = pack_bf16x2(lo[0], lo[1]); pk[1] = pack_bf16x2(lo[2], lo[3]);
        pk[2] = pack_bf16x2(hi[0], hi[1]); pk[3] = pack_bf16x2(hi[2], hi[3]);
        *reinterpret_cast<u32x4*>(fg.m[member].out + (size_t)t * d_out + c) = pk;
    }
}

bool decode_tail_applies(int r) { return r == 8 || r == 16 || r == 32; }

// gate_rows = every row of Wcat: the split tiles mem[g].gpartial hold the gate terms and all adapters' shrink.
hipError_t launch_decode_tail_group(const DecodeMember* mem, int G, int S, int T, int N, int r, int k, int gate_rows,
                                    float inv_temperature, float scale, hipStream_t stream) {
    if (G < 1 || G > kMaxDecodeGroup || S < 1 || padded_adapters(N) != 32 || gate_rows != prep_wcat_rows(N, r))
        return hipErrorInvalidValue;
    RouteGroup rg{};
    FinishGroup fg{};
    int widest = 0;
    for (int g = 0; g < G; ++g) {
        if (mem[g].d_out % 8 != 0 || mem[g].d_out < 8) return hipErrorInvalidValue;
        rg.m[g] = {mem[g].gpartial, mem[g].bias, mem[g].idx, mem[g].w};
        fg.m[g] = {mem[g].partial, (const bf16_t*)mem[g].B, (bf16_t*)mem[g].out, mem[g].d_out};
        widest = mem[g].d_out > widest ? mem[g].d_out : widest;
    }
    fg.nsplit = S;
    fg.chunks = ceil_div(widest / 8, kTailThreads);
    const unsigned grid = (unsigned)G * T * fg.chunks;
    auto go = [&](auto kern) {
        kern<<<grid, kTailThreads, 0, stream>>>(T, N, gate_rows, k, inv_temperature, scale, rg, fg);
        return hipGetLastError();
    };
    if (r == 8) return go(decode_tail_kernel<1>);
    if (r == 16) return go(decode_tail_kernel<2>);
    if (r == 32) return go(decode_tail_kernel<4>);
    return hipErrorInvalidValue;
}

bool route_small_applies(int T, int r, bool bf16) { return bf16 && T <= 64 && (r == 8 || r == 16 || r == 32); }

hipError_t launch_route_shrink_small(const void* x, const float* partials, int KS, const float* bias, const void* A,
                                     int T, int d_in, int N, int r, int k, float inv_temperature, float scale,
                                     int32_t* topk_idx, float* topk_w, void* hdense, int ext_stride,
                                     hipStream_t stream) {
    const int NP = padded_adapters(N);
    auto go = [&](auto kern) {
        kern<<<T, kSmallThreads, 0, stream>>>((const bf16_t*)x, partials, KS, bias, (const bf16_t*)A, T, d_in, N, NP, k,
                                              inv_temperature, scale, topk_idx, topk_w, (bf16_t*)hdense, ext_stride);
        return hipGetLastError();
    };
    if (r == 8) return go(route_shrink_small_kernel<1>);
    if (r == 16) return go(route_shrink_small_kernel<2>);
    if (r == 32) return go(route_shrink_small_kernel<4>);
    return hipErrorInvalidValue;
}

}  // namespace meteora
