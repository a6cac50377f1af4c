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

namespace meteora {

constexpr int kSmallThreads = 1024;   // 16 wavefronts per token: the shrink is latency-bound, so many short loops
constexpr int kSmallWaves = kSmallThreads / 64;

// A group of layers that share x (same T, d_in, N, r, k): workgroup b serves token b % T of member b / T.
struct RouteGroup {
    struct Member {
        const float* gpart;
        const float* bias;
        const bf16_t* A;
        int32_t* idx;
        float* w;
        float* hs;
    } m[kMaxDecodeGroup];
    int G;   // 0: the kernel's own pointer arguments describe the one layer
};

template <int R8>   // R8 = r / 8: 16-byte pieces per row of A_a
__global__ __launch_bounds__(kSmallThreads) void route_shrink_small_kernel(
    const bf16_t* __restrict__ x, const float* __restrict__ partials, int KS, const float* bias_in,
    const bf16_t* A_in, int T, int d_in, int N, int NP, int k, float inv_temperature, float scale,
    int32_t* idx_in, float* w_in, bf16_t* __restrict__ hdense, int ext_stride,
    const float* gpart_in, int GS, float* hs_in, const RouteGroup rg) {
    constexpr int r = R8 * 8;
    constexpr int ROWS = 8 / R8;   // rows of A_a per slot whose loads are in flight together
    __shared__ int sel_idx[kMaxTopK];
    __shared__ float sel_w[kMaxTopK];
    __shared__ float red[kSmallWaves][kMaxTopK][r];
    __shared__ float gsum[2][kSmallWaves][kMaxAdapters];   // per-split logit terms, double-buffered over rounds
    float glog = 0.f;
    int t = blockIdx.x;
    const float* __restrict__ bias = bias_in;
    const bf16_t* __restrict__ A = A_in;
    int32_t* __restrict__ topk_idx = idx_in;
    float* __restrict__ topk_w = w_in;
    const float* __restrict__ gpart = gpart_in;
    float* __restrict__ hs = hs_in;
    if (rg.G > 0) {   // uniform
        const int g = blockIdx.x / T;
        t = blockIdx.x - g * T;
        bias = rg.m[g].bias; A = rg.m[g].A; topk_idx = rg.m[g].idx; topk_w = rg.m[g].w;
        gpart = rg.m[g].gpart; hs = rg.m[g].hs;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    // this token's row of the dense expand operand starts as zeros
    if (hdense != nullptr) {
        u32x4* row = reinterpret_cast<u32x4*>(hdense + (size_t)t * ext_stride);
        for (int i = threadIdx.x; i < ext_stride / 8; i += kSmallThreads) row[i] = u32x4{0u, 0u, 0u, 0u};
    }
    // Logits from the split-K tiles of the gate-term rows: wavefront w fetches split w, w + 16, ... (every wavefront
    // has its loads out at once), (lo + mid) + hi within a split; wavefront 0 then adds the splits in order.
    if (gpart != nullptr) {
        const int GR = 3 * NP;
        for (int s0 = 0; s0 < GS; s0 += kSmallWaves) {
            const int sp = s0 + wave;
            float v = 0.f;
            if (sp < GS && lane < N) {
                const float* src = gpart + ((size_t)sp * T + t) * GR + lane;
                const float hi = src[0], mid = src[NP], lo = src[2 * NP];
                v = (lo + mid) + hi;
            }
            if (lane < kMaxAdapters) gsum[s0 / kSmallWaves & 1][wave][lane] = v;
            __syncthreads();
            if (wave == 0) {
                const int n = min(kSmallWaves, GS - s0);
                for (int u = 0; u < n; ++u) glog += gsum[s0 / kSmallWaves & 1][u][lane];
            }
        }
    }
    if (wave == 0) {   // top-k and softmax: lane = adapter
        float g = 0.f;
        if (lane < N && gpart != nullptr) {
            g = glog + (bias != nullptr ? bias[lane] : 0.f);
            if (g == 0.f) g = 0.f;
        } else if (lane < N) {
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
        if (hs != nullptr) hs[((size_t)t * k + slot) * r + q] = scale * sel_w[slot] * h;
        else hdense[(size_t)t * ext_stride + sel_idx[slot] * r + q] = from_float<bf16_t>(scale * sel_w[slot] * h);
    }
}

bool route_small_applies(int T, int r, bool bf16) { return bf16 && T <= 64 && (r == 8 || r == 16 || r == 32); }

hipError_t launch_route_shrink_small(const void* x, const float* partials, int KS, const float* bias, const void* A,
                                     int T, int d_in, int N, int r, int k, float inv_temperature, float scale,
                                     int32_t* topk_idx, float* topk_w, void* hdense, int ext_stride,
                                     hipStream_t stream, const float* gpart, int GS, float* hs) {
    const int NP = padded_adapters(N);
    auto go = [&](auto kern) {
        kern<<<T, kSmallThreads, 0, stream>>>((const bf16_t*)x, partials, KS, bias, (const bf16_t*)A, T, d_in, N, NP, k,
                                    inv_temperature, scale, topk_idx, topk_w, (bf16_t*)hdense, ext_stride, gpart,
                                    GS, hs, RouteGroup{});
        return hipGetLastError();
    };
    if (r == 8) return go(route_shrink_small_kernel<1>);
    if (r == 16) return go(route_shrink_small_kernel<2>);
    if (r == 32) return go(route_shrink_small_kernel<4>);
    return hipErrorInvalidValue;
}

hipError_t launch_route_shrink_small_group(const void* x, const DecodeMember* mem, int G, int S, int T, int d_in, int N,
                                           int r, int k, float inv_temperature, float scale, hipStream_t stream) {
    if (G < 1 || G > kMaxDecodeGroup) return hipErrorInvalidValue;
    const int NP = padded_adapters(N);
    RouteGroup rg{};
    for (int g = 0; g < G; ++g)
        rg.m[g] = {mem[g].gpartial, mem[g].bias, (const bf16_t*)mem[g].A, mem[g].idx, mem[g].w, mem[g].hs};
    rg.G = G;
    auto go = [&](auto kern) {
        kern<<<G * T, kSmallThreads, 0, stream>>>((const bf16_t*)x, nullptr, 0, nullptr, nullptr, T, d_in, N, NP, k,
                                                  inv_temperature, scale, nullptr, nullptr, nullptr, 0, nullptr, S,
                                                  nullptr, rg);
        return hipGetLastError();
    };
    if (r == 8) return go(route_shrink_small_kernel<1>);
    if (r == 16) return go(route_shrink_small_kernel<2>);
    if (r == 32) return go(route_shrink_small_kernel<4>);
    return hipErrorInvalidValue;
}

}  // namespace meteora
