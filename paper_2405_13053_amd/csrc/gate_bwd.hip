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
// into d_logits per token, gate_bwd_wgrad_kernel accumulates x^T d_logits over token slices with plain fp32
// FMAs (a [d_in, T] x [T, 32] product whose x operand is not K-contiguous; 1 GFLOP at T = d_in = 4096, below
// what re-tiling x for MFMA would cost), and gate_bwd_reduce_kernel adds the slices in order.
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
}

// ---- dW_gate partials: wpart[slice][c][32] = sum over the slice's tokens of x[t][c] * dg[t][:] ----
// A workgroup takes 128 columns of x (a lane two adjacent ones) and one token slice; its four wavefronts take
// eight adapters each.  dg of 64 tokens at a time sits in LDS (read as broadcasts); x streams with eight
// tokens' loads in flight.  Workgroups of column tile 0 also add up dg itself for the bias gradient.
constexpr int kWgCols = 128;
constexpr int kWgChunk = 64;

__global__ __launch_bounds__(256) void gate_bwd_wgrad_kernel(const bf16_t* __restrict__ x, const float* __restrict__ dg,
                                                              int T, int d_in, int slice_tokens,
                                                              float* __restrict__ wpart, float* __restrict__ bpart) {
    __shared__ __attribute__((aligned(16))) float s_dg[kWgChunk][kBwdNP];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = blockIdx.x * kWgCols + 2 * lane;
    const int cc = min(c, d_in - 2);                         // d_in is even; clamped lanes do not store
    const int slice = blockIdx.y;
    const int t_begin = slice * slice_tokens, t_end = min(T, t_begin + slice_tokens);
    float acc0[8], acc1[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { acc0[j] = 0.f; acc1[j] = 0.f; }
    float bsum = 0.f;
    for (int tc = t_begin; tc < t_end; tc += kWgChunk) {
        __syncthreads();
        {   // 64 x 32 floats: a thread copies 8 of them; rows past the slice are zero
            const int row = threadIdx.x >> 2, q = (threadIdx.x & 3) * 8;
            f32x4 v0 = {0.f, 0.f, 0.f, 0.f}, v1 = v0;
            if (tc + row < t_end) {
                const float* p = dg + (size_t)(tc + row) * kBwdNP + q;
                v0 = *reinterpret_cast<const f32x4*>(p);
                v1 = *reinterpret_cast<const f32x4*>(p + 4);
            }
            *reinterpret_cast<f32x4*>(&s_dg[row][q]) = v0;
            *reinterpret_cast<f32x4*>(&s_dg[row][q + 4]) = v1;
        }
        __syncthreads();
        if (blockIdx.x == 0 && threadIdx.x < kBwdNP)
            for (int tt = 0; tt < kWgChunk; ++tt) bsum += s_dg[tt][threadIdx.x];
        for (int tt0 = 0; tt0 < kWgChunk; tt0 += 8) {
            uint32_t xv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int t = min(tc + tt0 + u, T - 1);      // rows past the slice meet zero dg
                xv[u] = *reinterpret_cast<const uint32_t*>(x + (size_t)t * d_in + cc);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float x0 = bf16_bits_to_float(xv[u] & 0xffffu), x1 = bf16_bits_to_float(xv[u] >> 16);
                const f32x4 d0 = *reinterpret_cast<const f32x4*>(&s_dg[tt0 + u][wave * 8]);
                const f32x4 d1 = *reinterpret_cast<const f32x4*>(&s_dg[tt0 + u][wave * 8 + 4]);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc0[j] += x0 * d0[j]; acc0[4 + j] += x0 * d1[j];
                    acc1[j] += x1 * d0[j]; acc1[4 + j] += x1 * d1[j];
                }
            }
        }
    }
    if (c < d_in) {
        float* p = wpart + ((size_t)slice * d_in + c) * kBwdNP + wave * 8;
        *reinterpret_cast<f32x4*>(p) = f32x4{acc0[0], acc0[1], acc0[2], acc0[3]};
        *reinterpret_cast<f32x4*>(p + 4) = f32x4{acc0[4], acc0[5], acc0[6], acc0[7]};
        *reinterpret_cast<f32x4*>(p + kBwdNP) = f32x4{acc1[0], acc1[1], acc1[2], acc1[3]};
        *reinterpret_cast<f32x4*>(p + kBwdNP + 4) = f32x4{acc1[4], acc1[5], acc1[6], acc1[7]};
    }
    if (blockIdx.x == 0 && threadIdx.x < kBwdNP) bpart[slice * kBwdNP + threadIdx.x] = bsum;
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
    int slices = ceil_div(1024, col_tiles);                   // about four workgroups per CU
    const int most = ceil_div(T, kWgChunk);
    if (slices > most) slices = most;
    return slices < 1 ? 1 : slices;
}
static int wgrad_slice_tokens(int T, int d_in) {
    return ceil_div(ceil_div(T, wgrad_slices(T, d_in)), kWgChunk) * kWgChunk;
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
    L.total = off;
    return L;
}

hipError_t launch_gate_backward(const void* x, const void* dy, const void* wcat, const void* B, const float* bias,
                                const int32_t* idx_in, const float* w_in, const int32_t* labels, float beta, int T,
                                int d_in, int d_out, int N, int r, int k, float scale, float* dW_gate, float* dbias,
                                float* d_logits, char* ws, hipStream_t stream) {
    if (!gate_backward_applies(T, d_in, d_out, N, r, true) || k < 1 || k > kMaxTopK || k > N)
        return hipErrorInvalidValue;
    const GateBackwardLayout L = gate_backward_layout(T, d_in, d_out, N, r);
    const int CR = prep_wcat_rows(N, r), NR = N * r;
    float* part_x = reinterpret_cast<float*>(ws + L.part_x);
    float* part_dy = reinterpret_cast<float*>(ws + L.part_dy);
    float* dg = reinterpret_cast<float*>(ws + L.dg);
    float* wpart = reinterpret_cast<float*>(ws + L.wpart);
    float* bpart = reinterpret_cast<float*>(ws + L.bpart);
    hipError_t e = launch_gemm_dense_splitk(x, wcat, T, d_in, CR, part_x, stream);
    if (e != hipSuccess) return e;
    e = launch_gemm_dense_splitk(dy, B, T, d_out, NR, part_dy, stream);
    if (e != hipSuccess) return e;
    DlogitsArgs a{};
    a.part_x = part_x; a.part_dy = part_dy; a.bias = bias; a.idx_in = idx_in; a.w_in = w_in; a.labels = labels;
    a.dg = dg; a.d_logits = d_logits;
    a.S1 = gemm_dense_splits(T, d_in, CR); a.S2 = gemm_dense_splits(T, d_out, NR);
    a.CR = CR; a.NR = NR; a.T = T; a.N = N; a.r = r; a.k = k; a.scale = scale; a.beta = beta;
    gate_bwd_dlogits_kernel<<<ceil_div(T, kBwdTokens), kBwdThreads, 0, stream>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int slice_tokens = wgrad_slice_tokens(T, d_in);
    const int slices = ceil_div(T, slice_tokens);
    gate_bwd_wgrad_kernel<<<dim3(ceil_div(d_in, kWgCols), slices), 256, 0, stream>>>(
        (const bf16_t*)x, dg, T, d_in, slice_tokens, wpart, bpart);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int blocks = (int)ceil_div64((int64_t)d_in * kBwdNP, 256) + 1;
    gate_bwd_reduce_kernel<<<blocks, 256, 0, stream>>>(wpart, bpart, slices, d_in, N, dW_gate, dbias);
    return hipGetLastError();
}

}  // namespace meteora
