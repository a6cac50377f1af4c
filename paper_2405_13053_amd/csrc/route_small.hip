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

// The rest of a decode-sized layer call in the same launch (FINISH): once a token's shrink values are known its
// workgroup also adds the K-split tiles of the base projection for a stretch of the token's output row, in split
// order, adds the expand of Eq. 2 from the shrink values it holds in LDS, and rounds once:
//   out[t, c] = bf16( sum_s partial[s][t][c] + sum_slot sum_q (scale * w * h)[slot][q] * B[a_slot][q][c] ).
// A token's row is cut into `chunks` stretches, one workgroup each (blockIdx = (member * T + token) * chunks +
// chunk), so that the launch fills the chip; the workgroups of a token repeat its routing and shrink (a few hundred
// KB from L2 each) instead of waiting for one another.  Arithmetic and order are those of
// gemm_splitk_reduce_expand_kernel.
struct FinishGroup {
    struct Member {
        const float* partial;   // [S][T][d_out]
        const bf16_t* B;        // [N, r, d_out]
        bf16_t* out;            // [T, d_out]
        int d_out;
    } m[kMaxDecodeGroup];
    int nsplit, chunks;         // chunks == 0: no finish stage
};

template <int R8, bool FINISH = false>   // R8 = r / 8: 16-byte pieces per row of A_a
__global__ __launch_bounds__(kSmallThreads) void route_shrink_small_kernel(
    const bf16_t* __restrict__ x, const float* __restrict__ partials, int KS, const float* bias_in,
    const bf16_t* A_in, int T, int d_in, int N, int NP, int k, float inv_temperature, float scale,
    int32_t* idx_in, float* w_in, bf16_t* __restrict__ hdense, int ext_stride,
    const float* gpart_in, int GS, float* hs_in, const RouteGroup rg, const FinishGroup fg) {
    constexpr int r = R8 * 8;
    constexpr int ROWS = 8 / R8;   // rows of A_a per slot whose loads are in flight together
    __shared__ int sel_idx[kMaxTopK];
    __shared__ float sel_w[kMaxTopK];
    __shared__ float red[kSmallWaves][kMaxTopK][r];
    __shared__ float gsum[2][kSmallWaves][kMaxAdapters];   // per-split logit terms, double-buffered over rounds
    float glog = 0.f;
    int t = blockIdx.x, member = 0, chunk = 0;
    if constexpr (FINISH) {
        chunk = blockIdx.x % fg.chunks;
        t = blockIdx.x / fg.chunks;
    }
    const float* __restrict__ bias = bias_in;
    const bf16_t* __restrict__ A = A_in;
    int32_t* __restrict__ topk_idx = idx_in;
    float* __restrict__ topk_w = w_in;
    const float* __restrict__ gpart = gpart_in;
    float* __restrict__ hs = hs_in;
    if (rg.G > 0) {   // uniform
        const int g = t / T;
        t = t - g * T;
        member = g;
        bias = rg.m[g].bias; A = rg.m[g].A; topk_idx = rg.m[g].idx; topk_w = rg.m[g].w;
        gpart = rg.m[g].gpart; hs = rg.m[g].hs;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    // FINISH: the K-split tiles of this thread's first 8 output columns do not depend on the routing: their loads
    // (the first 8 splits) go out now and are added, in split order, once the top-k is done, so that their latency
    // hides behind the logit fetch and the ranking
    f32x4 pre0[8], pre1[8];
    f32x4 pre_lo = {0.f, 0.f, 0.f, 0.f}, pre_hi = {0.f, 0.f, 0.f, 0.f};
    int fin_first = 0, fin_end = 0;
    if constexpr (FINISH) {
        const int c8 = fg.m[member].d_out / 8, per = (c8 + fg.chunks - 1) / fg.chunks;
        fin_first = chunk * per + threadIdx.x;
        fin_end = min(c8, (chunk + 1) * per);
        if (fin_first < fin_end) {
            const float* base = fg.m[member].partial + (size_t)t * fg.m[member].d_out + fin_first * 8;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float* src = base + (size_t)min(u, fg.nsplit - 1) * T * fg.m[member].d_out;
                pre0[u] = *reinterpret_cast<const f32x4*>(src);
                pre1[u] = *reinterpret_cast<const f32x4*>(src + 4);
            }
        }
    }

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
            if (chunk == 0) {   // the workgroups of a token compute the same routing: one of them reports it
                topk_idx[(size_t)t * k + lane] = my_i[0];
                topk_w[(size_t)t * k + lane] = my_w[0];
            }
        }
    }
    __syncthreads();
    if constexpr (FINISH) {
        if (fin_first < fin_end) {
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (u < fg.nsplit) { pre_lo += pre0[u]; pre_hi += pre1[u]; }
        }
    }

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
    __shared__ float hsl[kMaxTopK * r];   // scale * w * h of this token (FINISH)
    for (int e = threadIdx.x; e < k * r; e += kSmallThreads) {
        const int slot = e / r, q = e - slot * r;
        float h = 0.f;
#pragma unroll
        for (int wv = 0; wv < kSmallWaves; ++wv) h += red[wv][slot][q];   // fixed order
        const float v = scale * sel_w[slot] * h;
        if constexpr (FINISH) {
            hsl[e] = v;
            if (hs != nullptr && chunk == 0) hs[((size_t)t * k + slot) * r + q] = v;
        } else {
            if (hs != nullptr) hs[((size_t)t * k + slot) * r + q] = v;
            else hdense[(size_t)t * ext_stride + sel_idx[slot] * r + q] = from_float<bf16_t>(v);
        }
    }
    if constexpr (FINISH) {
        __syncthreads();
        const float* __restrict__ partial = fg.m[member].partial;
        const bf16_t* __restrict__ B = fg.m[member].B;
        bf16_t* __restrict__ out = fg.m[member].out;
        const int d_out = fg.m[member].d_out, nsplit = fg.nsplit;
        for (int gi = fin_first; gi < fin_end; gi += kSmallThreads) {   // 8 consecutive columns
            const int c = gi * 8;
            // the first stretch of this thread starts from the sums of the splits fetched at the top
            const bool first = gi == fin_first;
            f32x4 lo = first ? pre_lo : f32x4{0.f, 0.f, 0.f, 0.f}, hi = first ? pre_hi : f32x4{0.f, 0.f, 0.f, 0.f};
            for (int s0 = first ? 8 : 0; s0 < nsplit; s0 += 8) {   // tiles in order, 8 tiles' loads in flight
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
                const bf16_t* Ba = B + (size_t)sel_idx[slot] * r * d_out + c;
                const float* h = hsl + slot * r;
#pragma unroll
                for (int q0 = 0; q0 < r; q0 += 8) {   // 8 rows of B in flight
                    u32x4 b[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) b[u] = *reinterpret_cast<const u32x4*>(Ba + (size_t)(q0 + u) * d_out);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const float hv = h[q0 + u];
                        lo[0] = fmaf(hv, bf16_bits_to_float(b[u][0] & 0xffffu), lo[0]);
                        lo[1] = fmaf(hv, bf16_bits_to_float(b[u][0] >> 16), lo[1]);
                        lo[2] = fmaf(hv, bf16_bits_to_float(b[u][1] & 0xffffu), lo[2]);
                        lo[3] = fmaf(hv, bf16_bits_to_float(b[u][1] >> 16), lo[3]);
                        hi[0] = fmaf(hv, bf16_bits_to_float(b[u][2] & 0xffffu), hi[0]);
                        hi[1] = fmaf(hv, bf16_bits_to_float(b[u][2] >> 16), hi[1]);
                        hi[2] = fmaf(hv, bf16_bits_to_float(b[u][3] & 0xffffu), hi[2]);
                        hi[3] = fmaf(hv, bf16_bits_to_float(b[u][3] >> 16), hi[3]);
                    }
                }
            }
            u32x4 pk;
            pk[0] = pack_bf16x2(lo[0], lo[1]); pk[1] = pack_bf16x2(lo[2], lo[3]);
            pk[2] = pack_bf16x2(hi[0], hi[1]); pk[3] = pack_bf16x2(hi[2], hi[3]);
            *reinterpret_cast<u32x4*>(out + (size_t)t * d_out + c) = pk;
        }
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
                                    GS, hs, RouteGroup{}, FinishGroup{});
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
                                                  nullptr, rg, FinishGroup{});
        return hipGetLastError();
    };
    if (r == 8) return go(route_shrink_small_kernel<1>);
    if (r == 16) return go(route_shrink_small_kernel<2>);
    if (r == 32) return go(route_shrink_small_kernel<4>);
    return hipErrorInvalidValue;
}

// Routing, shrink, split-K reduction and expand of decode-sized calls in one launch (the FINISH form of the kernel):
// replaces launch_route_shrink_small_group followed by launch_gemm_decode_finish, with the same results bit for bit.
int decode_finish_chunks(int T, int G) {
    // about one workgroup per CU (a workgroup is 16 wavefronts): 256 / (G * T), at least 1, at most 16
    int ch = 256 / (G * T > 0 ? G * T : 1);
    return ch < 1 ? 1 : (ch > 16 ? 16 : ch);
}

hipError_t launch_route_shrink_finish_group(const void* x, const DecodeMember* mem, int G, int S, int T, int d_in, int N,
                                            int r, int k, float inv_temperature, float scale, hipStream_t stream) {
    if (G < 1 || G > kMaxDecodeGroup || S < 1) return hipErrorInvalidValue;
    const int NP = padded_adapters(N);
    RouteGroup rg{};
    FinishGroup fg{};
    for (int g = 0; g < G; ++g) {
        if (mem[g].d_out % 8 != 0) return hipErrorInvalidValue;
        rg.m[g] = {mem[g].gpartial, mem[g].bias, (const bf16_t*)mem[g].A, mem[g].idx, mem[g].w, nullptr};
        fg.m[g] = {mem[g].partial, (const bf16_t*)mem[g].B, (bf16_t*)mem[g].out, mem[g].d_out};
    }
    rg.G = G;
    fg.nsplit = S;
    fg.chunks = decode_finish_chunks(T, G);
    auto go = [&](auto kern) {
        kern<<<G * T * fg.chunks, kSmallThreads, 0, stream>>>((const bf16_t*)x, nullptr, 0, nullptr, nullptr, T, d_in, N,
                                                              NP, k, inv_temperature, scale, nullptr, nullptr, nullptr, 0,
                                                              nullptr, S, nullptr, rg, fg);
        return hipGetLastError();
    };
    if (r == 8) return go(route_shrink_small_kernel<1, true>);
    if (r == 16) return go(route_shrink_small_kernel<2, true>);
    if (r == 32) return go(route_shrink_small_kernel<4, true>);
    return hipErrorInvalidValue;
}

}  // namespace meteora
