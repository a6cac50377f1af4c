// Host-side launchers of the gfx950 kernels.  Every launcher only enqueues work
// on `stream`; none allocates or synchronises.  Shapes have been validated by
// the C-ABI layer before a launcher is called.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace meteora {

// ---- process state (runtime.hip): raise a kernel's dynamic-LDS limit once per device (thread-safe), and the
// set-up of every kernel of the library ahead of its first launch, for the current device (meteora_init)
hipError_t ensure_lds_limit(const void* kernel, int bytes);
hipError_t init_kernels();
hipError_t gemm_init_kernels();
hipError_t gate_init_kernels();
hipError_t shrink_init_kernels();
hipError_t bucket_init_scratch();

// ---- weight repacking, one launch: W_gate -> split bf16 fragments (bf16 gate), A -> MFMA fragments,
// stacked B -> its transpose Bt[d_out, N*r rounded up to 64] (zero-padded) for the GEMM's K-extension.
// Any pair (W_gate, wsplit) / (A, apack) / (B, btrans) may be NULL to skip it; sizes are gate_wsplit_bytes,
// shrink_apack_bytes and prep_btrans_bytes (0 = that operand is not packed for this dtype/rank: pass NULL).
// wcat (optional, needs W_gate and A, d_in % 64 == 0, r % 8 == 0): Wcat[prep_wcat_rows, d_in] bf16 for the dense routing path,
// rows = hi | mid | lo terms of the gate columns (padded_adapters(N) rows each), then column q of A_a as row a*r+q.
size_t prep_btrans_bytes(int d_out, int N, int r, bool bf16);
int prep_wcat_rows(int N, int r);
size_t prep_wcat_bytes(int d_in, int N, int r, bool bf16);
hipError_t launch_prep(const float* W_gate, void* wsplit, const void* A, void* apack, const void* B, void* btrans,
                       void* wcat, int d_in, int d_out, int N, int r, hipStream_t stream);

// ---- gate (Sec. 3.1: G(x), I(x), Eq. 3) ------------------------------------------------
// Number of K-slices the logit kernel splits d_in into (partials[KS][T][NP]).
int gate_kslices(int d_in, bool bf16);
// bytes of the split-bf16 copy of W_gate the MFMA logit kernel reads (0 for fp32 inputs)
size_t gate_wsplit_bytes(int d_in, int N, bool bf16);
hipError_t launch_gate_logits(const void* x, const float* W_gate, int T, int d_in, int N, bool bf16,
                              void* wsplit, float* partials, hipStream_t stream);
// chunk_counts (optional): per-chunk adapter histograms [bucket_chunks(T)][N] for launch_bucket_scatter
hipError_t launch_gate_topk(const float* partials, int KS, const float* bias, int T, int N, int k,
                            float inv_temperature, int32_t* topk_idx, float* topk_w, float* logits,
                            int32_t* chunk_counts, hipStream_t stream);

// ---- small batches (T <= 64, bf16, r in {8, 16, 32}): top-k + softmax and the shrink of the selected
// adapters in one launch, one workgroup per token; consumes launch_gate_logits' partials and writes
// topk_idx, topk_w and every column of the token's row of hdense.  Replaces launch_gate_topk,
// launch_bucket and launch_shrink for the whole-layer call (shapes the two-launch decode form below does not take).
bool route_small_applies(int T, int r, bool bf16);
hipError_t launch_route_shrink_small(const void* x, const float* partials, int KS, const float* bias, const void* A,
                                     int T, int d_in, int N, int r, int k, float inv_temperature, float scale,
                                     int32_t* topk_idx, float* topk_w, void* hdense, int ext_stride,
                                     hipStream_t stream);

// ---- batches of more than 64 tokens (bf16, r % 8 == 0, d_in % 64 == 0, at most 640 rows of Wcat): one MFMA launch
// computes the split-bf16 gate logits and x * A_i of every adapter as fp32 K-split partials
// part[splits][T][prep_wcat_rows], then a launch of independent wavefronts adds the splits, ranks (Sec. 3.1, Eq. 3)
// and writes topk_idx, topk_w and every column of the tokens' rows of hdense.  Replaces launch_gate_logits,
// launch_gate_topk, launch_bucket and launch_shrink for the whole-layer call.  Up to kRouteDenseMaxTokens always;
// beyond, with up to 320 rows of Wcat always, with more where the products' tiles fill the CUs
// (route_dense_applies).
constexpr int kRouteDenseMaxTokens = 8192;
bool route_dense_possible(int d_in, int N, int r, bool bf16);            // whatever T: is Wcat worth packing
bool route_dense_applies(int T, int d_in, int N, int r, bool bf16);
size_t route_dense_part_bytes(int T, int d_in, int N, int r, bool bf16);  // 0 if the path does not apply
hipError_t launch_route_dense_products(const void* x, const void* wcat, int T, int d_in, int N, int r, float* part,
                                       hipStream_t stream);
hipError_t launch_route_dense_select(const float* part, const float* bias, int T, int d_in, int N, int r, int k,
                                     float inv_temperature, float scale, int32_t* topk_idx, float* topk_w,
                                     void* hdense, int ext_stride, hipStream_t stream, float* hs = nullptr,
                                     int splits = 0);
// hs (optional): also write hs[T,k,r] = scale * w * h in fp32 (the operand of launch_gemm_decode_finish); hdense may
// then be NULL.  splits (optional): the number of K splits in `part` if it is not launch_route_dense_products' own.
// the GEMM behind launch_route_dense_products: partial[split][T][rows] = x * Wcat^T over the split's K range
bool gemm_dense_splitk_ok(int T, int d_in, int rows);
int gemm_dense_splits(int T, int d_in, int rows);
// few-tile split-K launches over several matrices: S capped to one workgroup per CU where the tiles are 256 rows high
// (col_tiles: the 128-column tiles of all the matrices of the launch)
int gemm_multi_cap_splits(int T, int col_tiles, int S);
hipError_t launch_gemm_dense_splitk(const void* x, const void* Wcat, int T, int d_in, int rows, float* partial,
                                    hipStream_t stream);

// the same for several matrices in one launch of 128 x 128 tiles, all with S splits (at most 8 matrices)
struct DenseOperand { const void* W; int rows; float* partial; };
hipError_t launch_gemm_dense_splitk_multi(const void* x, const DenseOperand* ops, int n_ops, int S, int T, int d_in,
                                          hipStream_t stream);

// ---- bucketing (Sec. 3.3: per-adapter token sets as index lists) --------------------------
constexpr int kBucketChunkTokens = 64;   // tokens (k pairs each) whose pairs one workgroup histograms and scatters
inline int bucket_chunks(int T) { return (T + kBucketChunkTokens - 1) / kBucketChunkTokens; }
// The library's own histogram scratch (a file-scope device array, one copy per GPU) for the entry point that takes
// no workspace: room for kStaticBucketMaxTokens tokens and any supported N; the pointer is the current device's.
constexpr int kStaticBucketMaxTokens = 65536;
hipError_t bucket_static_scratch(int32_t** ptr);
// have_hist: chunk_counts already holds the histograms (written by launch_gate_topk)
// clear_rows (optional): a [T][clear_row_bytes] array (row bytes a multiple of 16) that the scatter zeroes,
// every chunk its own rows: the dense expand operand that launch_shrink then fills in (shrink_clears_hdense)
hipError_t launch_bucket(const int32_t* topk_idx, int T, int k, int N, int32_t* chunk_counts, bool have_hist,
                         int32_t* counts, int32_t* offsets, int32_t* bucket_tok, int32_t* bucket_slot,
                         void* clear_rows, int clear_row_bytes, hipStream_t stream);

// ---- grouped LoRA shrink: h[t,slot,:] = x[t,:] * A[idx[t,slot]] ---------------------------
// h32 ([T,k,r] fp32) and/or hdense (bf16 [T, ext_stride], column idx*r+q = scale*w*h, other
// columns zero) are written; either may be NULL.
// apack / hpart: scratch of shrink_apack_bytes / shrink_hpart_bytes (A in MFMA operand order,
// per-K-slice partial sums); both sizes are 0 when the plain-FMA kernel is used.
// false: launch_shrink writes only the selected columns of hdense, so the caller has its rows cleared
// first (launch_bucket's clear_rows); true: launch_shrink writes every column itself
bool shrink_clears_hdense(bool bf16, int r, int T, int k);
size_t shrink_apack_bytes(int d_in, int N, int r, bool bf16);
size_t shrink_hpart_bytes(int T, int d_in, int r, int k, bool bf16);
hipError_t launch_shrink(const void* x, const void* A, const int32_t* topk_idx, const float* topk_w,
                         const int32_t* offsets, const int32_t* bucket_tok, const int32_t* bucket_slot,
                         int T, int d_in, int N, int r, int k, float scale, bool bf16,
                         void* apack, float* hpart, float* h32, void* hdense, int ext_stride,
                         hipStream_t stream);

// ---- grouped LoRA expand: out (+)= scale * sum_slot w * h[t,slot,:] * B[idx[t,slot]] ------
hipError_t launch_expand(const float* h32, const void* B, const int32_t* topk_idx, const float* topk_w,
                         int T, int d_out, int N, int r, int k, float scale, bool bf16, void* out,
                         int accumulate, hipStream_t stream);

// ---- decode-sized batches in two launches (T <= 64, bf16, r in {8, 16, 32}, Wcat packed), for one layer or for a
// group of up to kMaxDecodeGroup layers that share x (q/k/v, gate/up):
// launch_gemm_decode_main: the main K splits of x * W_g^T as fp32 tiles partial_g[S][T][d_out_g], and in the same
//   launch x * Wcat_g^T (gate_rows = prep_wcat_rows(N, r): the gate terms and every adapter's shrink columns) as
//   gpartial_g[S][T][gate_rows]; S = gemm_group_splits(...) for every member;
// launch_decode_tail_group (route_small.hip): top-k, softmax -> idx_g, w_g, and
//   out_g = bf16(sum of the S tiles in order + sum_slot (scale * w * h from the shrink tiles) * B_g[idx_g]).
// launch_gemm_decode_finish: the reduction with the expand alone, from hs_g[T,k,r] = scale * w * h (the few-tile
//   form of mid-sized batches below).
constexpr int kMaxDecodeGroup = 4;
struct DecodeMember {
    const void* W;        // [d_out, d_in]
    const void* wg3;      // Wcat
    const float* bias;    // gate bias or NULL
    const void* A;        // [N, d_in, r]
    const void* B;        // [N, r, d_out]
    int d_out;
    float* partial;       // [S][T][d_out]
    float* gpartial;      // [S][T][gate_rows]
    float* hs;            // [T,k,r]
    int32_t* idx;         // [T,k]
    float* w;             // [T,k]
    void* out;            // [T,d_out]
};
int gemm_splitk_splits(int T, int d_in, int d_out, bool bf16);
int gemm_group_splits(int T, int d_in, const int* d_out, int G, int gate_rows);   // 0: the shapes are not split
hipError_t launch_gemm_decode_main(const void* x, const DecodeMember* mem, int G, int gate_rows, int S, int T,
                                   int d_in, hipStream_t stream);
hipError_t launch_gemm_decode_finish(const DecodeMember* mem, int G, int S, int T, int k, int r, hipStream_t stream);
bool decode_tail_applies(int r);   // ranks the tail's kernel is built for
hipError_t launch_decode_tail_group(const DecodeMember* mem, int G, int S, int T, int N, int r, int k, int gate_rows,
                                    float inv_temperature, float scale, hipStream_t stream);
// The same three launches for batches of a few hundred tokens with few output tiles: launch_gemm_dense_splitk_multi over
// every W_g and Wcat_g (gpartial_g then holds [S][T][prep_wcat_rows]), this selection for all members, the finish above.
hipError_t launch_route_dense_select_group(const DecodeMember* mem, int G, int S, int T, int N, int r, int k,
                                           float inv_temperature, float scale, hipStream_t stream);

// ---- gate gradients (Sec. 3.2, Eq. 4): dW_gate[d_in,N], dbias[N] (optional) and d_logits[T,N] (optional) from
// x, dy = dL/do, the packed Wcat and B; bf16 shapes of the dense routing path with d_out % 64 == 0.
// idx_in / w_in (optional, both or neither): the routing of the forward call; NULL ranks again from the same
// logits.  labels (optional): per-token adapter label of the classification loss, weight beta; values outside
// [0, N) give that token no classification part.  ws: gate_backward_layout(...).total bytes.
// part_x_given (optional): the K-split products x * Wcat^T that launch_route_dense_products left for this x
// (same T, d_in, N, r) in part_x_splits K splits (0 = that launcher's own count); NULL computes them here.
// dx (optional, bf16 [T, d_in]): the input gradient; needs A, W_gate and W_t = the base weight transposed,
// [d_in, d_out].
constexpr int kGateBackwardMaxTokens = 65536;
struct GateBackwardLayout { size_t part_x, part_dy, dg, wpart, bpart, hx, xt, total; int ext; };
bool gate_backward_applies(int T, int d_in, int d_out, int N, int r, bool bf16);
GateBackwardLayout gate_backward_layout(int T, int d_in, int d_out, int N, int r);
hipError_t launch_gate_backward(const void* x, const void* dy, const void* wcat, const void* B, const float* bias,
                                const int32_t* idx_in, const float* w_in, const int32_t* labels, float beta, int T,
                                int d_in, int d_out, int N, int r, int k, float scale, float* dW_gate, float* dbias,
                                float* d_logits, const float* part_x_given, int part_x_splits, const void* A,
                                const float* W_gate, const void* W_t, void* dx, char* ws, hipStream_t stream);

// ---- base projection out = x * W^T (W stored [d_out, d_in]), optional fused LoRA expand ---
// If hdense != NULL the contraction is extended by the columns of hdense against the stacked B
// (out += hdense * B viewed as [N*r, d_out]), i.e. the LoRA expand runs in the same accumulators;
// the kernel takes B transposed and zero-padded, Bt[d_out, ext_stride] as launch_prep writes it,
// and ext_stride must be a multiple of 64.
// d_in may be 0 (expand only); accumulate=1 adds the previous contents of out.
// true if launch_gemm applies the hdense/B extension for this dtype (else run launch_expand after it)
bool gemm_fuses_expand(bool bf16);
// splitk_ws: scratch of gemm_splitk_bytes (0 = this shape is not split) or NULL to forbid splitting.
size_t gemm_splitk_bytes(int T, int d_in, int d_out, bool bf16);
hipError_t launch_gemm(const void* x, const void* W, int T, int d_in, int d_out, bool bf16,
                       const void* hdense, int ext_stride, const void* Bt, int ext_k,
                       void* out, int accumulate, float* splitk_ws, hipStream_t stream);

}  // namespace meteora
