// The paper's own ways of evaluating Eq. 2 (Sec. 3.3), as measured baselines on the same GPU, built from this
// library's kernels plus the few plain kernels below.  They exist to restate the paper's ratios (Sec. 3.3, Sec. 5,
// App. A.7) beside the bucketed/fused path; nothing in the layer calls them.
//
//   loop-original   for every adapter i in turn: gather the tokens routed to it into X_i, (X_i A_i) B_i as two
//                   GEMMs, weighted scatter-add into the output.  The per-adapter row counts decide the launch
//                   shapes, so they come back to the host first (one stream synchronisation per call), as the
//                   data-dependent shapes of the PyTorch loop do.
//   bmm-gather      Eq. 5 ("bmm-torch"): copy A_{I(t)_j}, B_{I(t)_j} for every (token, slot) pair into gathered
//                   tensors of T*k entries (T*k/N times the stacked adapters, the memory cost Sec. 3.3 names),
//                   then two batched products over the pairs and the weighted sum over the k slots.
// Both take the routing from the library's gate (meteora_gate_topk) and the base projection from its GEMM, so
// they differ from the layer only in how the LoRA term is scheduled.
#include "../../include/meteora.h"
#include "common.hpp"
#include "kernels.hpp"

namespace meteora {
namespace {

// ---- loop-original ------------------------------------------------------------------------------------------
// At[a][q][i] = A[a][i][q], Btr[a][c][q] = B[a][q][c]: both GEMMs of an iteration then read K-contiguous operands.
template <typename TX>
__global__ __launch_bounds__(256) void transpose_adapters_kernel(const TX* __restrict__ A, const TX* __restrict__ B,
                                                                 int N, int d_in, int d_out, int r,
                                                                 TX* __restrict__ At, TX* __restrict__ Btr) {
    const size_t nA = (size_t)N * d_in * r, nB = (size_t)N * r * d_out;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < nA + nB; e += (size_t)gridDim.x * 256) {
        if (e < nA) {   // e indexes At: (a, q, i)
            const int i = (int)(e % d_in), q = (int)((e / d_in) % r), a = (int)(e / ((size_t)d_in * r));
            At[e] = A[((size_t)a * d_in + i) * r + q];
        } else {        // e - nA indexes Btr: (a, c, q)
            const size_t f = e - nA;
            const int q = (int)(f % r), c = (int)((f / r) % d_out), a = (int)(f / ((size_t)r * d_out));
            Btr[f] = B[((size_t)a * r + q) * d_out + c];
        }
    }
}

// X_i[p, :] = x[tok[p], :], 16-byte pieces (row bytes are a multiple of 16)
__global__ __launch_bounds__(256) void gather_rows_kernel(const u32x4* __restrict__ x, const int32_t* __restrict__ tok,
                                                          int rows, int row16, u32x4* __restrict__ Xi) {
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < (size_t)rows * row16; e += (size_t)gridDim.x * 256) {
        const int p = (int)(e / row16), c = (int)(e % row16);
        Xi[e] = x[(size_t)tok[p] * row16 + c];
    }
}

// out[tok[p], :] += scale * w[tok[p], slot[p]] * D_i[p, :].  A token is routed to an adapter at most once, so
// the rows of one launch are distinct: plain read-modify-write, no atomics.
template <typename TX>
__global__ __launch_bounds__(256) void scatter_add_kernel(const TX* __restrict__ Di, const int32_t* __restrict__ tok,
                                                          const int32_t* __restrict__ slot,
                                                          const float* __restrict__ topk_w, int rows, int d_out, int k,
                                                          float scale, TX* __restrict__ out) {
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < (size_t)rows * d_out; e += (size_t)gridDim.x * 256) {
        const int p = (int)(e / d_out), c = (int)(e % d_out);
        const int t = tok[p];
        const float sw = scale * topk_w[(size_t)t * k + slot[p]];
        TX* o = out + (size_t)t * d_out + c;
        *o = from_float<TX>(to_float(*o) + sw * to_float(Di[e]));
    }
}

// ---- bmm-gather (Eq. 5) -------------------------------------------------------------------------------------
// Asel[p] = A[idx[p]], Bsel[p] = B[idx[p]] for every pair p = t*k + slot: the materialised copies.
__global__ __launch_bounds__(256) void gather_adapters_kernel(const u32x4* __restrict__ A, const u32x4* __restrict__ B,
                                                              const int32_t* __restrict__ idx, int a16, int b16,
                                                              u32x4* __restrict__ Asel, u32x4* __restrict__ Bsel) {
    const int p = blockIdx.x;
    const int a = idx[p];
    const u32x4* As = A + (size_t)a * a16;
    const u32x4* Bs = B + (size_t)a * b16;
    for (int e = threadIdx.x; e < a16; e += 256) Asel[(size_t)p * a16 + e] = As[e];
    for (int e = threadIdx.x; e < b16; e += 256) Bsel[(size_t)p * b16 + e] = Bs[e];
}

// first batched product: h[p, :] = x[t(p), :] * Asel[p]  ([1, d_in] x [d_in, r]), one workgroup per pair.
// A thread takes rows i, i + 256, ... of Asel[p] (r values each, read as 16-byte pieces, r % 8 == 0).
template <typename TX>
__global__ __launch_bounds__(256) void bmm_shrink_kernel(const TX* __restrict__ x, const TX* __restrict__ Asel,
                                                         int d_in, int r, int k, TX* __restrict__ h) {
    __shared__ float red[4][kMaxRank];
    const int p = blockIdx.x, t = p / k;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const TX* xt = x + (size_t)t * d_in;
    const TX* Ap = Asel + (size_t)p * d_in * r;
    for (int q0 = 0; q0 < r; q0 += 8) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int i = threadIdx.x; i < d_in; i += 256) {
            const float xv = to_float(xt[i]);
            const TX* row = Ap + (size_t)i * r + q0;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = fmaf(xv, to_float(row[j]), acc[j]);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float v = acc[j];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
            if (lane == 0) red[wave][q0 + j] = v;
        }
    }
    __syncthreads();
    if (threadIdx.x < r)
        h[(size_t)p * r + threadIdx.x] =
            from_float<TX>((red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]));
}

// second batched product, the weighted sum over the k slots and the base term:
// out[t, :] += scale * sum_slot w[t,slot] * (h[p, :] * Bsel[p]);  out holds x W on entry.  One workgroup per token.
template <typename TX>
__global__ __launch_bounds__(256) void bmm_expand_sum_kernel(const TX* __restrict__ h, const TX* __restrict__ Bsel,
                                                             const float* __restrict__ topk_w, int d_out, int r, int k,
                                                             float scale, TX* __restrict__ out) {
    __shared__ float hs[kMaxTopK * kMaxRank];
    const int t = blockIdx.x;
    for (int i = threadIdx.x; i < k * r; i += 256)
        hs[i] = scale * topk_w[(size_t)t * k + i / r] * to_float(h[(size_t)t * k * r + i]);
    __syncthreads();
    for (int c = threadIdx.x; c < d_out; c += 256) {
        float acc = to_float(out[(size_t)t * d_out + c]);
        for (int slot = 0; slot < k; ++slot) {
            const TX* Bp = Bsel + ((size_t)t * k + slot) * r * d_out + c;
            float d = 0.f;
            for (int q = 0; q < r; ++q) d = fmaf(hs[slot * r + q], to_float(Bp[(size_t)q * d_out]), d);
            acc += d;
        }
        out[(size_t)t * d_out + c] = from_float<TX>(acc);
    }
}

struct VariantLayout {
    size_t gate_ws, idx, w, counts, offsets, btok, bslot, bucket_ws, At, Btr, Xi, Hi, Di, Asel, Bsel, h, total;
};

VariantLayout variant_layout(int variant, int T, int d_in, int d_out, int N, int r, int k, meteora_dtype dt) {
    VariantLayout L{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const size_t e = dt == METEORA_BF16 ? 2 : 4, pairs = (size_t)T * k;
    L.gate_ws = take(meteora_workspace_bytes(T, d_in, 8, N, 1, k, dt));
    L.idx = take(pairs * sizeof(int32_t));
    L.w = take(pairs * sizeof(float));
    if (variant == METEORA_VARIANT_LOOP_ORIGINAL) {
        L.counts = take((size_t)N * sizeof(int32_t));
        L.offsets = take((size_t)(N + 1) * sizeof(int32_t));
        L.btok = take(pairs * sizeof(int32_t));
        L.bslot = take(pairs * sizeof(int32_t));
        L.bucket_ws = take((size_t)bucket_chunks(T) * N * sizeof(int32_t));
        L.At = take((size_t)N * r * d_in * e);
        L.Btr = take((size_t)N * d_out * r * e);
        L.Xi = take((size_t)T * d_in * e);    // an adapter gets at most T rows
        L.Hi = take((size_t)T * r * e);
        L.Di = take((size_t)T * d_out * e);
    } else {
        L.Asel = take(pairs * d_in * r * e);
        L.Bsel = take(pairs * r * d_out * e);
        L.h = take(pairs * r * e);
    }
    L.total = off;
    return L;
}

template <typename T> T* at(void* ws, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(ws) + off); }

#define VARIANT_HIP(expr)                                 \
    do {                                                  \
        if ((expr) != hipSuccess) return METEORA_ERR_HIP; \
    } while (0)

template <typename TX>
meteora_status run_loop_original(const TX* x, const TX* A, const TX* B, int T, int d_in, int d_out, int N, int r, int k,
                                 float scale, bool bf16, TX* out, void* ws, const VariantLayout& L, hipStream_t st) {
    const int32_t* idx = at<int32_t>(ws, L.idx);
    const float* w = at<float>(ws, L.w);
    int32_t* counts = at<int32_t>(ws, L.counts);
    int32_t* offsets = at<int32_t>(ws, L.offsets);
    int32_t* btok = at<int32_t>(ws, L.btok);
    int32_t* bslot = at<int32_t>(ws, L.bslot);
    VARIANT_HIP(launch_bucket(idx, T, k, N, at<int32_t>(ws, L.bucket_ws), false, counts, offsets, btok, bslot, nullptr,
                              0, st));
    TX* At = at<TX>(ws, L.At);
    TX* Btr = at<TX>(ws, L.Btr);
    transpose_adapters_kernel<TX><<<1024, 256, 0, st>>>(A, B, N, d_in, d_out, r, At, Btr);
    VARIANT_HIP(hipGetLastError());
    // the loop's shapes depend on the routing: the counts come back to the host
    int32_t host_off[kMaxAdapters + 1];
    VARIANT_HIP(hipMemcpyAsync(host_off, offsets, (size_t)(N + 1) * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    VARIANT_HIP(hipStreamSynchronize(st));
    TX* Xi = at<TX>(ws, L.Xi);
    TX* Hi = at<TX>(ws, L.Hi);
    TX* Di = at<TX>(ws, L.Di);
    const int row16 = (int)((size_t)d_in * sizeof(TX) / 16);
    for (int a = 0; a < N; ++a) {
        const int p0 = host_off[a], rows = host_off[a + 1] - host_off[a];
        if (rows <= 0) continue;
        const unsigned gblocks = (unsigned)min((size_t)4096, ((size_t)rows * row16 + 255) / 256);
        gather_rows_kernel<<<gblocks, 256, 0, st>>>((const u32x4*)x, btok + p0, rows, row16, (u32x4*)Xi);
        VARIANT_HIP(hipGetLastError());
        VARIANT_HIP(launch_gemm(Xi, At + (size_t)a * r * d_in, rows, d_in, r, bf16, nullptr, 0, nullptr, 0, Hi, 0,
                                nullptr, st));
        VARIANT_HIP(launch_gemm(Hi, Btr + (size_t)a * d_out * r, rows, r, d_out, bf16, nullptr, 0, nullptr, 0, Di, 0,
                                nullptr, st));
        const unsigned sblocks = (unsigned)min((size_t)4096, ((size_t)rows * d_out + 255) / 256);
        scatter_add_kernel<TX><<<sblocks, 256, 0, st>>>(Di, btok + p0, bslot + p0, w, rows, d_out, k, scale, out);
        VARIANT_HIP(hipGetLastError());
    }
    return METEORA_OK;
}

template <typename TX>
meteora_status run_bmm_gather(const TX* x, const TX* A, const TX* B, int T, int d_in, int d_out, int N, int r, int k,
                              float scale, TX* out, void* ws, const VariantLayout& L, hipStream_t st) {
    const int32_t* idx = at<int32_t>(ws, L.idx);
    const float* w = at<float>(ws, L.w);
    TX* Asel = at<TX>(ws, L.Asel);
    TX* Bsel = at<TX>(ws, L.Bsel);
    TX* h = at<TX>(ws, L.h);
    const int a16 = (int)((size_t)d_in * r * sizeof(TX) / 16), b16 = (int)((size_t)r * d_out * sizeof(TX) / 16);
    const unsigned pairs = (unsigned)((size_t)T * k);
    gather_adapters_kernel<<<pairs, 256, 0, st>>>((const u32x4*)A, (const u32x4*)B, idx, a16, b16, (u32x4*)Asel,
                                                  (u32x4*)Bsel);
    VARIANT_HIP(hipGetLastError());
    bmm_shrink_kernel<TX><<<pairs, 256, 0, st>>>(x, Asel, d_in, r, k, h);
    VARIANT_HIP(hipGetLastError());
    bmm_expand_sum_kernel<TX><<<T, 256, 0, st>>>(h, Bsel, w, d_out, r, k, scale, out);
    VARIANT_HIP(hipGetLastError());
    (void)N;
    return METEORA_OK;
}

}  // namespace
}  // namespace meteora

using namespace meteora;

extern "C" {

size_t meteora_variant_workspace_bytes(meteora_variant variant, int T, int d_in, int d_out, int N, int r, int k,
                                       meteora_dtype dt) {
    if (variant != METEORA_VARIANT_LOOP_ORIGINAL && variant != METEORA_VARIANT_BMM_GATHER) return 0;
    if (meteora_workspace_bytes(T, d_in, d_out, N, r, k, dt) == 0) return 0;   // the layer's own argument limits
    if (r % 8 != 0) return 0;   // rows of the gathered operands are moved in 16-byte pieces
    return variant_layout(variant, T, d_in, d_out, N, r, k, dt).total + 256;
}

meteora_status meteora_variant_forward(meteora_variant variant, const void* x, const void* W, const float* W_gate,
                                       const float* gate_bias, const void* A, const void* B, int T, int d_in, int d_out,
                                       int N, int r, int k, float scale, meteora_dtype dt, void* out,
                                       int32_t* topk_idx_out, float* topk_w_out, void* ws, size_t ws_bytes,
                                       meteora_stream stream) {
    if (variant != METEORA_VARIANT_LOOP_ORIGINAL && variant != METEORA_VARIANT_BMM_GATHER)
        return METEORA_ERR_INVALID_ARG;
    if (!x || !W || !W_gate || !A || !B || !out) return METEORA_ERR_INVALID_ARG;
    const size_t need = meteora_variant_workspace_bytes(variant, T, d_in, d_out, N, r, k, dt);
    if (need == 0) {
        // tell bad arguments from unsupported ones the way the layer call does
        if (T < 0 || d_in < 1 || d_out < 1 || N < 1 || r < 1 || k < 1 || k > N) return METEORA_ERR_INVALID_ARG;
        return METEORA_ERR_UNSUPPORTED;
    }
    if (!(scale == scale) || scale - scale != 0.f) return METEORA_ERR_INVALID_ARG;   // NaN or infinite
    auto aligned = [](const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; };
    if (!aligned(x, 16) || !aligned(W, 16) || !aligned(W_gate, 16) || !aligned(A, 16) || !aligned(B, 16) ||
        !aligned(out, 16) || (gate_bias && !aligned(gate_bias, 4)) || (topk_idx_out && !aligned(topk_idx_out, 16)) ||
        (topk_w_out && !aligned(topk_w_out, 16)))
        return METEORA_ERR_UNSUPPORTED;
    if (!ws || !aligned(ws, 256) || ws_bytes < need) return METEORA_ERR_WORKSPACE;
    if (T == 0) return METEORA_OK;
    const bool bf16 = dt == METEORA_BF16;
    const VariantLayout L = variant_layout(variant, T, d_in, d_out, N, r, k, dt);
    hipStream_t st = static_cast<hipStream_t>(stream);
    int32_t* idx = at<int32_t>(ws, L.idx);
    float* w = at<float>(ws, L.w);
    // routing from the library's gate, base projection from its GEMM
    meteora_status s = meteora_gate_topk(x, W_gate, gate_bias, T, d_in, N, k, dt, 1.0f, idx, w, nullptr,
                                         at<void>(ws, L.gate_ws), meteora_workspace_bytes(T, d_in, 8, N, 1, k, dt),
                                         stream);
    if (s != METEORA_OK) return s;
    VARIANT_HIP(launch_gemm(x, W, T, d_in, d_out, bf16, nullptr, 0, nullptr, 0, out, 0, nullptr, st));
    if (variant == METEORA_VARIANT_LOOP_ORIGINAL) {
        s = bf16 ? run_loop_original<bf16_t>((const bf16_t*)x, (const bf16_t*)A, (const bf16_t*)B, T, d_in, d_out, N, r,
                                             k, scale, true, (bf16_t*)out, ws, L, st)
                 : run_loop_original<float>((const float*)x, (const float*)A, (const float*)B, T, d_in, d_out, N, r, k,
                                            scale, false, (float*)out, ws, L, st);
    } else {
        s = bf16 ? run_bmm_gather<bf16_t>((const bf16_t*)x, (const bf16_t*)A, (const bf16_t*)B, T, d_in, d_out, N, r, k,
                                          scale, (bf16_t*)out, ws, L, st)
                 : run_bmm_gather<float>((const float*)x, (const float*)A, (const float*)B, T, d_in, d_out, N, r, k,
                                         scale, (float*)out, ws, L, st);
    }
    if (s != METEORA_OK) return s;
    if (topk_idx_out)
        VARIANT_HIP(hipMemcpyAsync(topk_idx_out, idx, (size_t)T * k * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    if (topk_w_out)
        VARIANT_HIP(hipMemcpyAsync(topk_w_out, w, (size_t)T * k * sizeof(float), hipMemcpyDeviceToDevice, st));
    return METEORA_OK;
}

}  // extern "C"
