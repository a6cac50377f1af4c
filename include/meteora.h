/*
 * meteora.h - C ABI of the MI355X (gfx950) MeteoRA linear-layer forward.
 *
 * The layer (paper Sec. 3.1, Eq. 2 and Eq. 3; row-vector convention of Eq. 1):
 *
 *     G(x) = x * W_gate (+ bias)                      gate logits, fp32
 *     I(x) = top-k adapters by logit (ties -> lower index)
 *     w_i  = softmax over the k selected logits       Eq. 3
 *     o    = x * W_base + scale * sum_{i in I(x)} w_i * ((x * A_i) * B_i)   Eq. 2
 *
 * with the n LoRA pairs stacked contiguously as in Sec. 3.3:
 * A[N, d_in, r], B[N, r, d_out].
 *
 * Conventions common to every entry point
 *  - Every pointer is a DEVICE pointer (HBM of the current HIP device) unless
 *    it is marked "host".  All arrays are dense, row-major, 16-byte aligned.
 *  - `dt` is the storage type of x, W, A, B and out: METEORA_BF16 (bfloat16,
 *    fp32 accumulation) or METEORA_F32.  W_gate, gate_bias, logits and topk_w
 *    are always fp32; indices are int32.
 *  - Storage: x[T, d_in]; W[d_out, d_in] (o[t,c] = sum_i x[t,i] * W[c,i]);
 *    W_gate[d_in, N]; gate_bias[N] or NULL; A[N, d_in, r]; B[N, r, d_out];
 *    out[T, d_out].
 *  - Ownership: the caller owns all memory.  The library never allocates,
 *    frees or keeps device memory; scratch space is the caller's `ws`
 *    (at least meteora_workspace_bytes(...) bytes, 256-byte aligned).
 *    Inputs are only read; outputs are fully overwritten (except
 *    accumulate=1).  Outputs must not alias inputs.
 *  - Execution: all work is enqueued on `stream` (a hipStream_t passed as
 *    void*; NULL = the default stream).  No call synchronises with the host.
 *    Results are deterministic: same inputs -> bit-identical outputs.
 *    Calls that share a workspace must be ordered on one stream.
 *  - Errors: a status code is returned, nothing is thrown.  Arguments are
 *    validated on the host before any launch, so an error status means that
 *    nothing was enqueued.  T == 0 returns METEORA_OK without a launch.
 *  - Limits: 1 <= k <= N <= 64, k <= 8, 1 <= r <= 64; d_in % 8 == 0 and
 *    d_out % 8 == 0; T * k < 2^31.  Inputs must be finite.
 */
#ifndef METEORA_H
#define METEORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    METEORA_OK = 0,
    METEORA_ERR_INVALID_ARG = 1, /* null required pointer, negative size, k<1, k>N, non-finite scale */
    METEORA_ERR_UNSUPPORTED = 2, /* shape/dtype/alignment outside the limits above */
    METEORA_ERR_WORKSPACE = 3,   /* ws is NULL or ws_bytes too small */
    METEORA_ERR_HIP = 4,         /* a HIP launch reported an error */
    METEORA_ERR_TOO_LARGE = 5    /* beyond the fixed scratch of an entry point that takes no workspace */
} meteora_status;

typedef enum { METEORA_F32 = 0, METEORA_BF16 = 1 } meteora_dtype;

/* A hipStream_t, passed as an opaque pointer so that this header needs no HIP include. */
typedef void* meteora_stream;

/* Library version (major*10000 + minor*100 + patch).  Host only. */
int meteora_version(void);

/* Text for a status code.  Host only; returns a static string. */
const char* meteora_status_string(meteora_status s);

/*
 * Optional set-up of HIP device `device` (-1 = the current device): everything that a kernel's first
 * launch on a device otherwise does by itself, which is one host-side function attribute per kernel
 * that uses more than 64 KB of LDS.  Setting that attribute is not a stream operation and is not
 * allowed while the stream is being captured into a HIP graph: a caller that captures its first call
 * of an entry point runs meteora_init (or one eager call of the same entry point at the same kind of
 * batch size) beforehand.  Cheap to repeat; thread-safe.  Returns METEORA_ERR_HIP without a usable
 * device, METEORA_ERR_INVALID_ARG if `device` cannot be selected.  Leaves the current device unchanged.
 */
meteora_status meteora_init(int device);

/*
 * Scratch bytes needed by meteora_gate_topk, meteora_bucket_tokens,
 * meteora_lora_forward and meteora_linear_forward for this problem size (the
 * maximum over the four; entry points that take no d_out or r accept the
 * value computed with any legal d_out, r, e.g. 8 and 1).
 * Host only, no HIP call.  Returns 0 for arguments outside the limits.
 */
size_t meteora_workspace_bytes(int T, int d_in, int d_out, int N, int r, int k, meteora_dtype dt);

/*
 * Audit of the workspace carving of meteora_linear_forward (with_packed = 0) or
 * meteora_linear_forward_packed with a blob (with_packed = 1), for tests.  Host only, no HIP call.
 * Entry i of the host arrays (each may be NULL) receives region i's name (static string), its
 * byte offset in ws, the bytes reserved for it, and the bytes that the launch sequence this
 * shape selects writes there (from that sequence's own tile and K-split counts).  Returns the
 * number of regions (at most max_regions entries are filled), or -1 for arguments outside the
 * limits.  Every written extent must fit its reservation, and offset + reserved must stay inside
 * meteora_workspace_bytes.
 */
int meteora_workspace_regions(int T, int d_in, int d_out, int N, int r, int k, meteora_dtype dt,
                              int with_packed, const char** names /*host*/, size_t* offset /*host*/,
                              size_t* reserved /*host*/, size_t* written /*host*/, int max_regions);

/*
 * Gate network and top-k routing (Sec. 3.1: G(x), I(x); Eq. 3).
 *   logits[t,j]  = sum_i x[t,i] * W_gate[i,j] (+ gate_bias[j]), fp32 accumulation
 *   topk_idx[t,:] = the k adapters with the largest logits, listed by descending
 *                   logit, equal logits by ascending adapter index
 *   topk_w[t,:]   = exp(g - g_max) / sum over the k selected (Eq. 3), fp32
 * `logits` ([T,N] fp32) may be NULL if the caller does not want them.
 * inv_temperature scales the selected logits inside the softmax only
 * (1.0f = Eq. 3 as printed; 1/tau for the temperature of App. A.6).
 */
meteora_status meteora_gate_topk(const void* x, const float* W_gate, const float* gate_bias,
                                 int T, int d_in, int N, int k, meteora_dtype dt,
                                 float inv_temperature,
                                 int32_t* topk_idx /*[T,k]*/, float* topk_w /*[T,k]*/,
                                 float* logits /*[T,N] or NULL*/,
                                 void* ws, size_t ws_bytes, meteora_stream stream);

/*
 * Token-to-adapter bucketing: the per-adapter token sets {x | i in I(x)} of
 * Sec. 3.3 as index lists instead of gathered copies.
 *   counts[j]  = number of (token, slot) pairs routed to adapter j
 *   offsets    = exclusive prefix sum of counts, offsets[N] = T*k
 *   bucket_tok / bucket_slot [offsets[j] .. offsets[j+1]) = the pairs of adapter
 *                j, ordered by ascending token, then ascending slot (stable)
 * topk_idx values must lie in [0, N).
 */
meteora_status meteora_bucket_tokens(const int32_t* topk_idx /*[T,k]*/, int T, int k, int N,
                                     int32_t* counts /*[N]*/, int32_t* offsets /*[N+1]*/,
                                     int32_t* bucket_tok /*[T*k]*/, int32_t* bucket_slot /*[T*k]*/,
                                     void* ws, size_t ws_bytes, meteora_stream stream);

/*
 * meteora_bucket_tokens for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs,
 * outputs, order and bit-exact results; the per-chunk histograms that the other entry point keeps in
 * `ws` live in a fixed 256 KiB device array inside the library (one copy per GPU, held until the
 * process ends), so the call allocates nothing and frees nothing.
 *   Limit: T <= 65536 tokens (any k <= 8, N <= 64); beyond that METEORA_ERR_TOO_LARGE, nothing is launched.
 *   The array's device address is looked up on the first call on each device (or by meteora_init).
 *   All calls on one GPU share the array: calls that can overlap on one GPU (different streams with
 *   no ordering between them, or several host threads) race on it and must be serialised by the
 *   caller.  Nothing in it needs clearing between calls: the histogram pass overwrites every entry
 *   the scatter pass reads, so a call may follow a larger one.
 * Other errors as for meteora_bucket_tokens.
 */
meteora_status meteora_bucket_tokens_noalloc(const int32_t* topk_idx /*[T,k]*/, int T, int k, int N,
                                             int32_t* counts /*[N]*/, int32_t* offsets /*[N+1]*/,
                                             int32_t* bucket_tok /*[T*k]*/, int32_t* bucket_slot /*[T*k]*/,
                                             meteora_stream stream);

/*
 * LoRA term of Eq. 2 for a given routing:
 *   delta[t,:] = scale * sum_j topk_w[t,j] * ((x[t,:] * A[a]) * B[a]),  a = topk_idx[t,j]
 *   accumulate = 0: out = delta;  accumulate = 1: out = out + delta.
 * Runs bucketing, the grouped shrink (h = x*A_a, fp32) and the grouped expand.
 */
meteora_status meteora_lora_forward(const void* x, const void* A, const void* B,
                                    const int32_t* topk_idx, const float* topk_w,
                                    int T, int d_in, int d_out, int N, int r, int k,
                                    float scale, meteora_dtype dt,
                                    void* out /*[T,d_out]*/, int accumulate,
                                    void* ws, size_t ws_bytes, meteora_stream stream);

/*
 * Whole layer, Eq. 2: out = x*W + scale * sum_{i in I(x)} w_i * ((x*A_i)*B_i),
 * with I(x), w from the gate as in meteora_gate_topk.  inv_temperature as there:
 * 1.0f is Eq. 3 as printed, 1/tau the softmax temperature that App. A.6 uses for the
 * composite tasks (tau = 15, 20, 30); it changes the weights, never the selection.
 * With k = 1 (the top-1 strategy of App. A.1) the weight is exactly 1: no exponential is
 * evaluated, and the per-token work of the shrink and expand is that of one adapter.
 * If topk_idx_out / topk_w_out are not NULL they receive the routing used.
 * Errors: a non-finite scale or inv_temperature is METEORA_ERR_INVALID_ARG.
 */
meteora_status meteora_linear_forward(const void* x, const void* W, const float* W_gate,
                                      const float* gate_bias, const void* A, const void* B,
                                      int T, int d_in, int d_out, int N, int r, int k,
                                      float scale, float inv_temperature, meteora_dtype dt,
                                      void* out /*[T,d_out]*/,
                                      int32_t* topk_idx_out /*[T,k] or NULL*/,
                                      float* topk_w_out /*[T,k] or NULL*/,
                                      void* ws, size_t ws_bytes, meteora_stream stream);

/*
 * Weight packing, done once when the adapters are loaded: the stacked adapter
 * tensors of Sec. 3.3 and the gate weight are static during inference, so their
 * kernel-side layouts (W_gate split into three bf16 terms in matrix-core operand
 * order, A in operand order, B transposed, and the gate terms with every column of
 * every A_i as the rows of one matrix for the mid-sized-batch routing kernel) need
 * not be rebuilt for every batch.
 *   meteora_packed_bytes   size of the packed blob for these shapes (0 if this dtype
 *                          uses no packed operands, e.g. METEORA_F32).  Host only.
 *   meteora_pack_weights   fills `packed` (device, 256-byte aligned, caller-owned) from
 *                          W_gate[d_in,N] fp32, A[N,d_in,r], B[N,r,d_out]; enqueued on
 *                          `stream`.  The blob is valid for exactly these tensors and
 *                          shapes; repack after changing any of them.
 *   meteora_linear_forward_packed   meteora_linear_forward that reads the blob instead
 *                          of repacking into the workspace.  `packed` = NULL behaves as
 *                          meteora_linear_forward.  The results are bit-identical.
 *                          W_gate, A and B are still required and must be the tensors the
 *                          blob was packed from: some paths (fp32, decode-sized batches)
 *                          read them directly.
 * Errors: METEORA_ERR_WORKSPACE if packed_bytes is smaller than meteora_packed_bytes.
 */
size_t meteora_packed_bytes(int d_in, int d_out, int N, int r, meteora_dtype dt);

meteora_status meteora_pack_weights(const float* W_gate, const void* A, const void* B,
                                    int d_in, int d_out, int N, int r, meteora_dtype dt,
                                    void* packed, size_t packed_bytes, meteora_stream stream);

meteora_status meteora_linear_forward_packed(const void* x, const void* W, const float* W_gate,
                                             const float* gate_bias, const void* A, const void* B,
                                             const void* packed, size_t packed_bytes,
                                             int T, int d_in, int d_out, int N, int r, int k,
                                             float scale, float inv_temperature, meteora_dtype dt,
                                             void* out /*[T,d_out]*/,
                                             int32_t* topk_idx_out /*[T,k] or NULL*/,
                                             float* topk_w_out /*[T,k] or NULL*/,
                                             void* ws, size_t ws_bytes, meteora_stream stream);

/*
 * Several MeteoRA layers on the same input: the layers of a decoder block that share x (q/k/v, and
 * gate/up; Sec. 4.1 embeds the adapters in all seven linear layers) each have their own base weight,
 * gate and adapters but the same T, d_in, N, r, k, scale and inv_temperature.  The result is that of one
 * meteora_linear_forward_packed call per member (same routing; outputs equal to bf16 accuracy, the
 * split-K sums may run in another order).  For decode-sized batches (T <= 64) and for batches of a few
 * hundred tokens whose members have few output tiles in all (at most 320 tiles of 128 x 128, routing
 * products included), with bf16, packed weights and at most 4 members, the whole group runs in two
 * (decode) or three launches instead of that many per layer; otherwise the members run one after the other.
 *   members  host array of G descriptors; every pointer in it is a device pointer with the meaning and
 *            alignment it has in meteora_linear_forward_packed (packed may be NULL: that member is then
 *            repacked into the workspace on every call, and the group runs member by member).
 *   ws       at least meteora_group_workspace_bytes(d_out[0..G), ...) bytes, 256-byte aligned.
 * Errors as for meteora_linear_forward_packed; G < 1 or G > 64 is METEORA_ERR_INVALID_ARG.
 */
typedef struct {
    const void* W;            /* [d_out, d_in] */
    const float* W_gate;      /* [d_in, N] */
    const float* gate_bias;   /* [N] or NULL */
    const void* A;            /* [N, d_in, r] */
    const void* B;            /* [N, r, d_out] */
    const void* packed;       /* blob of meteora_pack_weights for this member, or NULL */
    size_t packed_bytes;
    int d_out;
    void* out;                /* [T, d_out] */
    int32_t* topk_idx_out;    /* [T,k] or NULL */
    float* topk_w_out;        /* [T,k] or NULL */
} meteora_group_member;

size_t meteora_group_workspace_bytes(const int* d_out /*host, [G]*/, int G, int T, int d_in, int N, int r, int k,
                                     meteora_dtype dt);

meteora_status meteora_linear_forward_group(const void* x, const meteora_group_member* members /*host*/, int G,
                                            int T, int d_in, int N, int r, int k, float scale,
                                            float inv_temperature, meteora_dtype dt,
                                            void* ws, size_t ws_bytes, meteora_stream stream);

/*
 * Gradients of the gate of one module for its training (Sec. 3.2, Eq. 4; App. "Top-k strategy"): W, A and B
 * stay fixed, the loss reaches W_gate and gate_bias
 *   - through the output: dy[T,d_out] = dL_lm/do (storage type dt).  With v_j = scale * (x*A_a)*B_a,
 *     a = topk_idx[t,j]:  dL/dw_j = <dy[t], v_j>,  dL/dg_a = w_j * (dL/dw_j - sum_i w_i * dL/dw_i)
 *     (softmax of Eq. 3 over the k selected; the selection itself carries no gradient; zero for k = 1);
 *   - through the LoRA-classification loss of the module, beta * sum_t CE(softmax over all N logits of token
 *     t, labels[t]):  dL/dg_n += beta * (softmax(g)_n - [n == labels[t]]).  labels[t] outside [0, N) gives
 *     token t no classification part; labels == NULL or beta == 0 leaves the term out.
 * Outputs (fp32, overwritten):  d_logits[T,N] (may be NULL),  dW_gate[d_in,N] = x^T * d_logits,
 * dbias[N] = sum_t d_logits[t] (may be NULL).
 * The logits are recomputed from x and the packed weights with the forward call's arithmetic (three-term bf16
 * split of W_gate, fp32 sums over K splits; the number of splits, and with it the last bits, can differ from the
 * forward call's).  topk_idx / topk_w (both or neither): the routing the forward call returned, to be used
 * as it is; NULL ranks again from the recomputed logits (the same routing unless two logits tie to fp32 accuracy).
 * dx[T,d_in] (storage type dt, optional): the gradient with respect to the module's input, for the modules
 * in front of this one:  dx = dy*W + scale * sum_j w_j * ((dy*B_a^T)*A_a^T) + d_logits*W_gate^T  (base projection,
 * selected adapters, gate).  It needs A[N,d_in,r], W_gate[d_in,N] and W_t = the base weight TRANSPOSED, stored
 * [d_in,d_out] (the frozen base weight is kept in both orientations by a caller that trains); with dx == NULL
 * these three may be NULL.  The gate term is computed from two-term bf16 splits (about 2^-16 of its size).
 * `packed` is the blob of meteora_pack_weights for these adapters; B is the stacked [N,r,d_out] tensor.
 * forward_ws (optional): the workspace in which meteora_linear_forward(_packed) ran on this same x, these
 * adapters and the same T, d_in, d_out, N, r, k, dt, not written to since.  For 64 < T <= 8192 that call leaves
 * its products of x with the packed gate and A operands there and they are read instead of being computed
 * again (one launch less); for other T the argument is ignored.  The caller vouches for the contents.
 * Limits: dt == METEORA_BF16, N <= 32, r % 8 == 0, d_in % 64 == 0, d_out % 64 == 0, 3*32 + N*r <= 640,
 * T <= 65536; otherwise METEORA_ERR_UNSUPPORTED (meteora_gate_backward_workspace_bytes returns 0).
 * All pointers but the host-side scalars are device memory; ws as for the other entry points.
 */
size_t meteora_gate_backward_workspace_bytes(int T, int d_in, int d_out, int N, int r, int k, meteora_dtype dt);

meteora_status meteora_gate_backward(const void* x /*[T,d_in]*/, const void* dy /*[T,d_out]*/,
                                     const float* gate_bias /*[N] or NULL*/, const void* B /*[N,r,d_out]*/,
                                     const void* packed, size_t packed_bytes,
                                     const int32_t* topk_idx /*[T,k] or NULL*/, const float* topk_w /*[T,k] or NULL*/,
                                     const int32_t* labels /*[T] or NULL*/, float beta,
                                     int T, int d_in, int d_out, int N, int r, int k, float scale, meteora_dtype dt,
                                     float* dW_gate /*[d_in,N]*/, float* dbias /*[N] or NULL*/,
                                     float* d_logits /*[T,N] or NULL*/,
                                     const void* A /*[N,d_in,r] or NULL*/, const float* W_gate /*[d_in,N] or NULL*/,
                                     const void* W_t /*[d_in,d_out] or NULL*/, void* dx /*[T,d_in] or NULL*/,
                                     const void* forward_ws /*or NULL*/, size_t forward_ws_bytes,
                                     void* ws, size_t ws_bytes, meteora_stream stream);

/*
 * The paper's own schedules of Eq. 2 (Sec. 3.3), as baselines to measure against on the same GPU.  Same
 * arguments, result and routing as meteora_linear_forward (inv_temperature = 1); only the LoRA term is
 * scheduled differently, from this library's gate, bucketing and GEMM kernels plus plain gather / scatter /
 * batched-product kernels.  Not part of the layer's own path.
 *   METEORA_VARIANT_LOOP_ORIGINAL  "loop-original": for each adapter i in turn, gather the tokens routed to it
 *       (X_i), two GEMMs (X_i A_i) B_i, weighted scatter-add into out.  The launch shapes depend on the
 *       routing, so the call SYNCHRONISES `stream` once to read the per-adapter counts on the host (it cannot
 *       be captured into a HIP graph); up to 4 launches per non-empty adapter.
 *   METEORA_VARIANT_BMM_GATHER     Eq. 5 ("bmm-torch"): A_{I(t)_j} and B_{I(t)_j} are copied for every
 *       (token, slot) pair (T*k/N times the size of the stacked adapters, the cost Sec. 3.3 names), then two
 *       batched products over the T*k pairs and the weighted sum over the k slots.
 * Intermediates are stored in dt (X_i A_i, (X_i A_i) B_i and the running output are rounded to bf16 for
 * METEORA_BF16, as a framework-level implementation does), so outputs agree with the layer call to a few
 * bf16 roundings, not bit for bit.
 * Limits: as meteora_linear_forward, and r % 8 == 0.  ws: meteora_variant_workspace_bytes (bmm-gather:
 * about T*k*r*(d_in+d_out) elements).  Errors as for meteora_linear_forward.
 */
typedef enum { METEORA_VARIANT_LOOP_ORIGINAL = 0, METEORA_VARIANT_BMM_GATHER = 1 } meteora_variant;

size_t meteora_variant_workspace_bytes(meteora_variant variant, int T, int d_in, int d_out, int N, int r, int k,
                                       meteora_dtype dt);

meteora_status meteora_variant_forward(meteora_variant variant, const void* x, const void* W, const float* W_gate,
                                       const float* gate_bias, const void* A, const void* B,
                                       int T, int d_in, int d_out, int N, int r, int k, float scale, meteora_dtype dt,
                                       void* out /*[T,d_out]*/, int32_t* topk_idx_out /*[T,k] or NULL*/,
                                       float* topk_w_out /*[T,k] or NULL*/,
                                       void* ws, size_t ws_bytes, meteora_stream stream);

/*
 * Base projection alone, first term of Eq. 1 / Eq. 2: out = x * W
 * (W stored [d_out, d_in]).  Exposed so the dense contraction can be checked
 * and timed on its own.
 */
meteora_status meteora_base_gemm(const void* x, const void* W, int T, int d_in, int d_out,
                                 meteora_dtype dt, void* out /*[T,d_out]*/, meteora_stream stream);

/*
 * Optional per-stage timing, for benchmarks.  Host only; off by default.
 * While enabled, meteora_lora_forward and meteora_linear_forward record
 * hipEvents on `stream` around each stage (prep, gate_logits, gate_topk,
 * bucket, shrink, gemm, expand) for up to 256 calls.  A stage's reading is its kernels' time
 * plus the dispatch gap in front of them (about 2 us per launch against a kernel trace).  A stage that a batch size
 * folds into another is not reported: where the routing runs without bucket lists (bf16, T > 64) gate_logits covers
 * the gate logits and the shrink, gate_topk the top-k, softmax and selection (batches with few output tiles:
 * gemm covers the K-split projection with those products, shrink the launch after it); for
 * T <= 64 gemm covers the base projection's split-K launch (with the gate logits and every adapter's shrink),
 * shrink the launch after it (top-k, softmax, reduction, expand).  meteora_stage_timing_read waits
 * for those events, returns per stage the summed milliseconds and the number
 * of timed launches (arrays of meteora_stage_count() entries, host memory)
 * and the number of calls covered, and starts a new window.  Not thread-safe;
 * enable/disable must not race with other calls.
 */
int meteora_stage_count(void);
const char* meteora_stage_name(int stage);
meteora_status meteora_stage_timing_enable(int on);
meteora_status meteora_stage_timing_read(float* ms_sum /*host*/, int* launches /*host*/, int* calls /*host*/);

#ifdef __cplusplus
}
#endif
#endif /* METEORA_H */
