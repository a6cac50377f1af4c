// Gradients of the gate of a MeteoRA module (Sec. 3.2, Eq. 4; App. "Top-k strategy"): W, A_i, B_i are
// frozen, only W_gate and its bias are trained.
//
// With dy = dL_lm/do, v_j = scale * (x A_{a_j}) B_{a_j} the contribution of the j-th selected adapter and w the
// Eq. 3 weights, the language-model loss reaches the selected logits as
//     dL/dw_j = <dy, v_j> = scale * sum_q (x A_{a_j})_q * (B_{a_j} dy)_q,      dL/dg_{a_j} = w_j (dL/dw_j - sum_i w_i dL/dw_i)
// and the LoRA-classification loss (cross entropy of the softmax over all N logits against the token's
// label, weight beta) adds beta * (softmax(g) - onehot(label)) to every logit's gradient.  Then
//     dW_gate = x^T d_logits,   dbias = sum_t d_logits[t].
//
// Launches: the two r-vectors come from dense MFMA products, as in the mid-batch forward path:
// x * Wcat^T gives the logits and x A_i of EVERY adapter (the forward's own first launch, so the logits and with
// them the top-k are bit-identical to that path's), dy * Bflat^T with Bflat = B viewed as [N*r, d_out] gives
// B_i dy of every adapter; both as fp32 K-split partials.  gate_bwd_dlogits_kernel (this file) turns them
// into d_logits per token, gate_bwd_wgrad_kernel accumulates x^T d_logits over token slices with fp32 MFMAs
// (a [d_in, T] x [T, 32] product whose x operand is not K-contiguous), and gate_bwd_reduce_kernel adds the
// slices in order.
//
// Input gradient (optional): dx = dy W + scale * sum_j w_j (B_{a_j} dy) A_{a_j}^T + d_logits W_gate^T is the
// forward's fused GEMM with the roles swapped: dy times W^T's storage (the caller's transposed copy
// W_t[d_in, d_out]) with the K loop continued over an extension operand hx[T, E] against Xt[d_in, E]:
//   columns a*r + q:        hx = scale * w * (B_a dy)_q for the selected adapters, else 0;   Xt[c] = A[a][c][q]
//   next 3 blocks of 32:    hx = hi(d_logits) | hi(d_logits) | lo(d_logits);  Xt[c] = hi(W_gate[c]) | lo(W_gate[c]) | hi(W_gate[c])
// (two-term bf16 splits, the lo * lo product dropped: the gate term to about 2^-16 of its size).
// gate_bwd_dlogits_kernel writes hx, gate_bwd_pack_kernel writes Xt (W_gate changes with every optimizer step).
#include <type_traits>
#include "common.hpp"
#include "kernels.hpp"
#include "topk_key.hpp"
#include "dense_logits.hpp"

namespace meteora {

constexpr int kBwdTokens = 16;          // tokens per workgroup of the d_logits kernel
constexpr int kBwdTokensPerWave = 4;
constexpr int kBwdThreads = kBwdTokens / kBwdTokensPerWave * 64;
constexpr int kBwdNP = 32;              // logit columns (N <= 32, as the dense products require)

struct DlogitsArgs {
    const float* part_x;     // [S1][T][CR]  x * Wcat^T
    const float* part_dy;    // [S2][T][NR]  dy * Bflat^T
    const float* bias;       // [N] or NULL
    const int32_t* idx_in;   // [T,k] routing of the forward call, or NULL: rank again here
    const float* w_in;       // [T,k]
    const int32_t* labels;   // [T] or NULL
    float* dg;               // [T][32], columns >= N zero
    float* d_logits;         // [T,N] or NULL
    bf16_t* hx;              // [T][ext] extension operand of the input-gradient GEMM, or NULL
    int ext;                 // columns of hx: N*r + 96 rounded up to 64
    int S1, S2, CR, NR, T, N, r, k;
    float scale, beta;
};

__global__ __launch_bounds__(kBwdThreads) void gate_bwd_dlogits_kernel(const DlogitsArgs a) {
    constexpr int NP = kBwdNP;
    constexpr int TPP = 64 / NP;
    constexpr int G = kBwdTokensPerWave / TPP;
    constexpr int kChunks = kMaxRank / 8;
    __shared__ int s_idx[kBwdTokens][kMaxTopK];
    __shared__ float s_w[kBwdTokens][kMaxTopK];
    __shared__ float s_dot[kBwdTokens][kMaxTopK][kChunks];
    __shared__ float s_dg[kBwdTokens][NP];
    extern __shared__ __attribute__((aligned(16))) float s_u[];   // [kBwdTokens][k][r]: B_a dy, only when hx is written
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & (NP - 1), sub = lane / NP;
    const int t0 = blockIdx.x * kBwdTokens;
    const int T = a.T, N = a.N, r = a.r, k = a.k;

    float g[G];
    int lt[G];
#pragma unroll
    for (int i = 0; i < G; ++i) lt[i] = wave * kBwdTokensPerWave + i * TPP + sub;
    dense_logits<NP, G>(a.part_x, a.S1, a.CR, a.bias, T, N, t0, lt, col, g);

    int sel_i[G];
    float sel_w[G];
    if (a.idx_in != nullptr) {
#pragma unroll
        for (int i = 0; i < G; ++i) {
            const int t = min(t0 + lt[i], T - 1);
            sel_i[i] = col < k ? min(max(a.idx_in[(size_t)t * k + col], 0), N - 1) : 0;   // stay inside the partials
            sel_w[i] = col < k ? a.w_in[(size_t)t * k + col] : 0.f;
        }
    } else {
        wave_topk_softmax<NP, G>(g, lane, N, k, 1.0f, sel_i, sel_w);
    }
#pragma unroll
    for (int i = 0; i < G; ++i) {
        if (col < k) { s_idx[lt[i]][col] = sel_i[i]; s_w[lt[i]][col] = sel_w[i]; }
        // classification part: beta * (softmax over the N logits - onehot(label)); labels outside [0, N) carry none
        float ce = 0.f;
        const int t = min(t0 + lt[i], T - 1);
        const int label = a.labels != nullptr ? a.labels[t] : -1;
        float gmax = col < N ? g[i] : -INFINITY;
#pragma unroll
        for (int off = NP / 2; off >= 1; off >>= 1) gmax = fmaxf(gmax, __shfl_xor(gmax, off));
        const float e = col < N ? expf(g[i] - gmax) : 0.f;
        float sum = e;
#pragma unroll
        for (int off = NP / 2; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
        if (label >= 0 && label < N && col < N) ce = a.beta * (e / sum - (col == label ? 1.f : 0.f));
        s_dg[lt[i]][col] = ce;
    }
    __syncthreads();

    // ---- dL/dw of every (token, slot): a thread takes 8 of the r products, splits added in order ----
    const int R8 = r / 8;
    for (int e = threadIdx.x; e < kBwdTokens * k * R8; e += kBwdThreads) {
        const int tl = e / (k * R8), rem = e - tl * (k * R8);
        const int s = rem / R8, c = rem - s * R8;
        const int t = min(t0 + tl, T - 1);
        const int ad = s_idx[tl][s];
        const float* ph = a.part_x + (size_t)t * a.CR + 3 * NP + ad * r + c * 8;
        const float* pu = a.part_dy + (size_t)t * a.NR + ad * r + c * 8;
        f32x4 h0 = {0.f, 0.f, 0.f, 0.f}, h1 = h0, u0 = h0, u1 = h0;
        for (int s0 = 0; s0 < a.S1; s0 += 4) {
            f32x4 v0[4], v1[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float* p = ph + (size_t)min(s0 + u, a.S1 - 1) * T * a.CR;
                v0[u] = *reinterpret_cast<const f32x4*>(p);
                v1[u] = *reinterpret_cast<const f32x4*>(p + 4);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (s0 + u < a.S1) { h0 += v0[u]; h1 += v1[u]; }
        }
        for (int s0 = 0; s0 < a.S2; s0 += 4) {
            f32x4 v0[4], v1[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float* p = pu + (size_t)min(s0 + u, a.S2 - 1) * T * a.NR;
                v0[u] = *reinterpret_cast<const f32x4*>(p);
                v1[u] = *reinterpret_cast<const f32x4*>(p + 4);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (s0 + u < a.S2) { u0 += v0[u]; u1 += v1[u]; }
        }
        float d = 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q) d += h0[q] * u0[q];
#pragma unroll
        for (int q = 0; q < 4; ++q) d += h1[q] * u1[q];
        s_dot[tl][s][c] = d;
        if (a.hx != nullptr) {
            float* su = s_u + ((size_t)tl * k + s) * r + c * 8;
            *reinterpret_cast<f32x4*>(su) = u0;
            *reinterpret_cast<f32x4*>(su + 4) = u1;
        }
    }
    __syncthreads();

    // ---- softmax backward over the k selected, scattered onto the token's logit row ----
#pragma unroll
    for (int i = 0; i < G; ++i) {
        float dw = 0.f;
        if (col < k) {
            for (int c = 0; c < R8; ++c) dw += s_dot[lt[i]][col][c];
            dw *= a.scale;
        }
        float mean = col < k ? sel_w[i] * dw : 0.f;
#pragma unroll
        for (int off = 1; off < kMaxTopK; off <<= 1) mean += __shfl_xor(mean, off);
        // the k selected adapters of a token are distinct: no two lanes add to the same entry
        if (col < k) s_dg[lt[i]][sel_i[i]] += sel_w[i] * (dw - mean);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < G; ++i) {
        const int t = t0 + lt[i];
        if (t >= T) continue;
        const float v = col < N ? s_dg[lt[i]][col] : 0.f;
        a.dg[(size_t)t * NP + col] = v;
        if (a.d_logits != nullptr && col < N) a.d_logits[(size_t)t * N + col] = v;
    }
    if (a.hx == nullptr) return;

    // ---- rows of hx: a thread owns 8 columns of one token ----
    const int C8 = a.ext / 8, NR = N * r;
    for (int e = threadIdx.x; e < kBwdTokens * C8; e += kBwdThreads) {
        const int tl = e / C8, c0 = (e - tl * C8) * 8;
        const int t = t0 + tl;
        if (t >= T) continue;
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = 0.f;
        if (c0 < NR) {                                       // the adapter part: scale * w * (B_a dy)
            const int ad = c0 / r;
            for (int sl = 0; sl < k; ++sl)
                if (s_idx[tl][sl] == ad) {
                    const float sw = a.scale * s_w[tl][sl];
                    const float* su = s_u + ((size_t)tl * k + sl) * r + (c0 - ad * r);
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[i] = sw * su[i];
                }
        } else if (c0 < NR + 3 * NP) {                       // the gate part: hi | hi | lo of d_logits
            const int term = (c0 - NR) / NP, n0 = (c0 - NR) - term * NP;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float d = s_dg[tl][n0 + i];            // columns >= N are not written above and hold 0 or the
                const float dz = n0 + i < N ? d : 0.f;       // classification part of a padding lane: masked here
                const float hi = static_cast<float>(static_cast<bf16_t>(dz));
                v[i] = term == 2 ? dz - hi : hi;
            }
        }
        u32x4 pk;
        pk[0] = pack_bf16x2(v[0], v[1]); pk[1] = pack_bf16x2(v[2], v[3]);
        pk[2] = pack_bf16x2(v[4], v[5]); pk[3] = pack_bf16x2(v[6], v[7]);
        *reinterpret_cast<u32x4*>(a.hx + (size_t)t * a.ext + c0) = pk;
    }
}

// Xt[c][ext] for the input-gradient GEMM: A[a][c][:] at columns a*r.., then hi | lo | hi of W_gate[c][:] in blocks
// of 32 columns, zero elsewhere.  A thread owns 8 columns of one row c.
__global__ __launch_bounds__(256) void gate_bwd_pack_kernel(const uint16_t* __restrict__ A,
                                                             const float* __restrict__ W_gate, int d_in, int N, int r,
                                                             int ext, uint16_t* __restrict__ Xt) {
    const int C8 = ext / 8, NR = N * r;
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (size_t)d_in * C8) return;
    const int c = (int)(e / C8), c0 = (int)(e - (size_t)c * C8) * 8;
    u32x4 pk = {0u, 0u, 0u, 0u};
    if (c0 < NR) {
        const int ad = c0 / r, q0 = c0 - ad * r;
        pk = *reinterpret_cast<const u32x4*>(A + ((size_t)ad * d_in + c) * r + q0);
    } else if (c0 < NR + 3 * kBwdNP) {
        const int term = (c0 - NR) / kBwdNP, n0 = (c0 - NR) - term * kBwdNP;
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float w = n0 + i < N ? W_gate[(size_t)c * N + n0 + i] : 0.f;
            const float hi = static_cast<float>(static_cast<bf16_t>(w));
            v[i] = term == 1 ? w - hi : hi;
        }
        pk[0] = pack_bf16x2(v[0], v[1]); pk[1] = pack_bf16x2(v[2], v[3]);
        pk[2] = pack_bf16x2(v[4], v[5]); pk[3] = pack_bf16x2(v[6], v[7]);
    }
    *reinterpret_cast<u32x4*>(Xt + (size_t)c * ext + c0) = pk;
}

// ---- dW_gate partials: wpart[slice][c][32] = sum over the slice's tokens of x[t][c] * dg[t][:] ----
// The contraction runs over tokens, and x[T, d_in] is not token-contiguous, so the bf16 MFMA operand layout
// (eight consecutive K values per lane) would need a transposed copy of x.  The fp32 MFMA 32x32x2 takes ONE K
// value per lane: lane l holds A[m = l % 32][k = l / 32] and B[k = l / 32][n = l % 32].  With m = adapter,
// k = token and n = column slot, both operands are plain coalesced loads and the product keeps full fp32
// accuracy.  The kernel is bound by the number of vector loads it issues (a CU takes a 4-byte-per-lane load
// every ~6 cycles, a 2-, 8- or 16-byte one every 15 to 29), so a lane loads one dword of x, two adjacent
// columns, per token pair and feeds two MFMAs with column slots c0 + 2n and c0 + 2n + 1: one x load and one dg
// load per two MFMAs.  A wavefront covers 64 columns; the four wavefronts of a workgroup are 2 column halves
// x 2 token halves of a 128-column slice, the token halves added through LDS in a fixed order.
// Workgroups of column tile 0 also add up dg for dbias.
constexpr int kWgCols = 128;
constexpr int kWgRing = 16;      // token pairs whose loads are in flight per wavefront
constexpr int kWgChunk = 2 * kWgRing;

__global__ __launch_bounds__(256, 2) void gate_bwd_wgrad_kernel(const uint16_t* __restrict__ x,
                                                                 const float* __restrict__ dg, int T, int d_in,
                                                                 int slice_tokens, float* __restrict__ wpart,
                                                                 float* __restrict__ bpart) {
    constexpr int R = kWgRing;
    __shared__ float red[2][32][64];                         // [column half][acc entry][lane] of the second token half
    __shared__ float s_b[kBwdNP];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, kh = lane >> 5;
    const int chalf = wave & 1, thalf = wave >> 1;
    const int c = blockIdx.x * kWgCols + chalf * 64 + 2 * n; // d_in is even: both columns inside or both outside
    const int cc = min(c, d_in - 2);
    const int slice = blockIdx.y;
    const int s_begin = slice * slice_tokens, s_end = min(T, s_begin + slice_tokens);
    const int half_tokens = slice_tokens / 2;                // a multiple of kWgChunk
    const int t_begin = s_begin + thalf * half_tokens, t_end = min(s_end, t_begin + half_tokens);
    f32x16 acc0, acc1;
#pragma unroll
    for (int i = 0; i < 16; ++i) { acc0[i] = 0.f; acc1[i] = 0.f; }
    float bsum = 0.f;
    uint32_t xv[R];
    float dv[R];
    const uint32_t* xw = reinterpret_cast<const uint32_t*>(x);
    // lane part of the addresses (in dwords); the token part is uniform, so a full pair needs no per-lane arithmetic
    const int lane_x = (kh * d_in + cc) >> 1;
    const int row_dwords = d_in >> 1;
    // pair p of this wavefront = tokens t_begin + 2p (lanes 0..31) and t_begin + 2p + 1 (lanes 32..63)
    auto load_pair = [&](int slot, int pair, bool inside) {
        const int t0 = t_begin + 2 * pair;
        if (inside) {                                        // both tokens lie in [t_begin, t_end)
            xv[slot] = xw[(size_t)t0 * row_dwords + lane_x];
            dv[slot] = dg[(size_t)t0 * kBwdNP + lane];
        } else {
            const int t = t0 + kh;
            const int tc = min(t, T - 1);
            xv[slot] = xw[((size_t)tc * d_in + cc) >> 1];
            const float d = dg[(size_t)tc * kBwdNP + n];
            dv[slot] = t < t_end ? d : 0.f;                  // tokens past the range contribute nothing
        }
    };
    const int pairs = (max(t_end - t_begin, 0) + 1) / 2;
    // The loads of R pairs are in flight; each step consumes one pair (two MFMAs) and then requests the pair R
    // steps ahead into the same registers, so the load unit and the matrix cores work side by side instead of in
    // bursts.  The scheduling barriers keep the compiler from gathering the loads of a round at its top.
    // The operands of a step are converted one step ahead, while the matrix cores run the step before (a conversion
    // placed right in front of its MFMA holds the MFMA back by about 20 cycles).
    float cur_d = 0.f, cur_a0 = 0.f, cur_a1 = 0.f;
    auto convert = [&](int slot) {
        cur_d = dv[slot];
        cur_a0 = __uint_as_float(xv[slot] << 16);
        cur_a1 = __uint_as_float(xv[slot] & 0xffff0000u);
    };
    auto round = [&](auto mode, int p) {                     // mode 0: refill inside, 1: refill at the ragged end, 2: none
#pragma unroll
        for (int u = 0; u < R; ++u) {
            acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(cur_d, cur_a0, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(cur_d, cur_a1, acc1, 0, 0, 0);
            bsum += cur_d;
            if constexpr (decltype(mode)::value != 2) load_pair(u, p + R + u, decltype(mode)::value == 0);
            convert((u + 1) % R);                            // slot 0 at the end of a round: refilled at its first step
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (pairs > 0) {
#pragma unroll
        for (int u = 0; u < R; ++u) load_pair(u, u, false);
        convert(0);
        for (int p = 0; p < pairs; p += R) {
            if (t_begin + 2 * (p + 2 * R) <= t_end) round(std::integral_constant<int, 0>{}, p);
            else if (p + R < pairs) round(std::integral_constant<int, 1>{}, p);
            else round(std::integral_constant<int, 2>{}, p);
        }
    }
    // ---- second token half into LDS, first half adds it ----
    bsum += __shfl_xor(bsum, 32);
    if (thalf == 1) {
#pragma unroll
        for (int i = 0; i < 16; ++i) { red[chalf][i][lane] = acc0[i]; red[chalf][16 + i][lane] = acc1[i]; }
        if (chalf == 0 && kh == 0) s_b[n] = bsum;
    }
    __syncthreads();
    if (thalf == 1) return;
#pragma unroll
    for (int i = 0; i < 16; ++i) { acc0[i] += red[chalf][i][lane]; acc1[i] += red[chalf][16 + i][lane]; }
    // accumulator entry i of lane l: adapter 8*(i/4) + 4*(l/32) + i%4, column slot l%32
    if (c < d_in) {
        float* p = wpart + ((size_t)slice * d_in + c) * kBwdNP + kh * 4;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            *reinterpret_cast<f32x4*>(p + q * 8) = f32x4{acc0[4 * q], acc0[4 * q + 1], acc0[4 * q + 2], acc0[4 * q + 3]};
            *reinterpret_cast<f32x4*>(p + kBwdNP + q * 8) =
                f32x4{acc1[4 * q], acc1[4 * q + 1], acc1[4 * q + 2], acc1[4 * q + 3]};
        }
    }
    if (blockIdx.x == 0 && chalf == 0 && kh == 0) bpart[slice * kBwdNP + n] = bsum + s_b[n];
}

// dW_gate[c][n] = sum of the slices in order (thread per (c, padded n)); the last workgroup does dbias.
__global__ __launch_bounds__(256) void gate_bwd_reduce_kernel(const float* __restrict__ wpart,
                                                               const float* __restrict__ bpart, int slices, int d_in,
                                                               int N, float* __restrict__ dW_gate,
                                                               float* __restrict__ dbias) {
    const size_t total = (size_t)d_in * kBwdNP;
    if (blockIdx.x == gridDim.x - 1) {
        if (dbias != nullptr && threadIdx.x < N) {
            float s = 0.f;
            for (int sl = 0; sl < slices; ++sl) s += bpart[sl * kBwdNP + threadIdx.x];
            dbias[threadIdx.x] = s;
        }
        return;
    }
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int n = (int)(e % kBwdNP);
    const size_t cidx = e / kBwdNP;
    float s = 0.f;
    for (int s0 = 0; s0 < slices; s0 += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = wpart[(size_t)min(s0 + u, slices - 1) * total + e];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (s0 + u < slices) s += v[u];
    }
    if (n < N) dW_gate[cidx * N + n] = s;
}

// ---- host side ----
bool gate_backward_applies(int T, int d_in, int d_out, int N, int r, bool bf16) {
    return route_dense_possible(d_in, N, r, bf16) && T >= 1 && T <= kGateBackwardMaxTokens && r <= kMaxRank &&
           gemm_dense_splitk_ok(T, d_in, prep_wcat_rows(N, r)) && gemm_dense_splitk_ok(T, d_out, N * r);
}

static int wgrad_slices(int T, int d_in) {
    const int col_tiles = ceil_div(d_in, kWgCols);
    int slices = ceil_div(512, col_tiles);   // two workgroups per CU (measured: 256 to 2048 workgroups tried)
    const int most = ceil_div(T, 2 * kWgChunk);
    if (slices > most) slices = most;
    return slices < 1 ? 1 : slices;
}
static int wgrad_slice_tokens(int T, int d_in) {   // a multiple of one chunk per token half
    constexpr int step = 2 * kWgChunk;
    return ceil_div(ceil_div(T, wgrad_slices(T, d_in)), step) * step;
}

GateBackwardLayout gate_backward_layout(int T, int d_in, int d_out, int N, int r) {
    GateBackwardLayout L{};
    const int CR = prep_wcat_rows(N, r), NR = N * r;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off = align_up(off + bytes, 256); return o; };
    L.part_x = take((size_t)gemm_dense_splits(T, d_in, CR) * T * CR * sizeof(float));
    L.part_dy = take((size_t)gemm_dense_splits(T, d_out, NR) * T * NR * sizeof(float));
    L.dg = take((size_t)T * kBwdNP * sizeof(float));
    const int slices = ceil_div(T, wgrad_slice_tokens(T, d_in));
    L.wpart = take((size_t)slices * d_in * kBwdNP * sizeof(float));
    L.bpart = take((size_t)slices * kBwdNP * sizeof(float));
    L.ext = (int)align_up((size_t)NR + 3 * kBwdNP, 64);
    L.hx = take((size_t)T * L.ext * sizeof(uint16_t));
    L.xt = take((size_t)d_in * L.ext * sizeof(uint16_t));
    L.total = off;
    return L;
}

hipError_t launch_gate_backward(const void* x, const void* dy, const void* wcat, const void* B, const float* bias,
                                const int32_t* idx_in, const float* w_in, const int32_t* labels, float beta, int T,
                                int d_in, int d_out, int N, int r, int k, float scale, float* dW_gate, float* dbias,
                                float* d_logits, const float* part_x_given, int part_x_splits, const void* A,
                                const float* W_gate, const void* W_t, void* dx, char* ws, hipStream_t stream) {
    if ((dx != nullptr) && (!A || !W_gate || !W_t)) return hipErrorInvalidValue;
    if (!gate_backward_applies(T, d_in, d_out, N, r, true) || k < 1 || k > kMaxTopK || k > N)
        return hipErrorInvalidValue;
    const GateBackwardLayout L = gate_backward_layout(T, d_in, d_out, N, r);
    const int CR = prep_wcat_rows(N, r), NR = N * r;
    const float* part_x = part_x_given != nullptr ? part_x_given : reinterpret_cast<float*>(ws + L.part_x);
    float* part_dy = reinterpret_cast<float*>(ws + L.part_dy);
    float* dg = reinterpret_cast<float*>(ws + L.dg);
    float* wpart = reinterpret_cast<float*>(ws + L.wpart);
    float* bpart = reinterpret_cast<float*>(ws + L.bpart);
    hipError_t e = hipSuccess;
    if (part_x_given == nullptr) e = launch_gemm_dense_splitk(x, wcat, T, d_in, CR, reinterpret_cast<float*>(ws + L.part_x), stream);
    if (e != hipSuccess) return e;
    e = launch_gemm_dense_splitk(dy, B, T, d_out, NR, part_dy, stream);
    if (e != hipSuccess) return e;
    DlogitsArgs a{};
    a.part_x = part_x; a.part_dy = part_dy; a.bias = bias; a.idx_in = idx_in; a.w_in = w_in; a.labels = labels;
    a.dg = dg; a.d_logits = d_logits;
    a.hx = dx != nullptr ? reinterpret_cast<bf16_t*>(ws + L.hx) : nullptr;
    a.ext = L.ext;
    a.S1 = (part_x_given != nullptr && part_x_splits > 0) ? part_x_splits : gemm_dense_splits(T, d_in, CR);
    a.S2 = gemm_dense_splits(T, d_out, NR);
    a.CR = CR; a.NR = NR; a.T = T; a.N = N; a.r = r; a.k = k; a.scale = scale; a.beta = beta;
    const size_t u_bytes = dx != nullptr ? (size_t)kBwdTokens * k * r * sizeof(float) : 0;   // at most 32 KB
    gate_bwd_dlogits_kernel<<<ceil_div(T, kBwdTokens), kBwdThreads, u_bytes, stream>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (dx != nullptr) {
        uint16_t* xt = reinterpret_cast<uint16_t*>(ws + L.xt);
        const int64_t chunks = (int64_t)d_in * (L.ext / 8);
        gate_bwd_pack_kernel<<<(unsigned)ceil_div64(chunks, 256), 256, 0, stream>>>((const uint16_t*)A, W_gate, d_in, N,
                                                                                    r, L.ext, xt);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        // dx = dy * W_t^T continued over hx * Xt^T: the forward's GEMM with d_in and d_out swapped
        e = launch_gemm(dy, W_t, T, d_out, d_in, true, ws + L.hx, L.ext, xt, L.ext, dx, 0, nullptr, stream);
        if (e != hipSuccess) return e;
    }
    const int slice_tokens = wgrad_slice_tokens(T, d_in);
    const int slices = ceil_div(T, slice_tokens);
    gate_bwd_wgrad_kernel<<<dim3(ceil_div(d_in, kWgCols), slices), 256, 0, stream>>>(
        (const uint16_t*)x, dg, T, d_in, slice_tokens, wpart, bpart);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int blocks = (int)ceil_div64((int64_t)d_in * kBwdNP, 256) + 1;
    gate_bwd_reduce_kernel<<<blocks, 256, 0, stream>>>(wpart, bpart, slices, d_in, N, dW_gate, dbias);
    return hipGetLastError();
}

}  // namespace meteora
