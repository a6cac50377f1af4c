// C ABI of the library (declared in include/meteora.h): argument validation, workspace
// carving and the launch sequence of each entry point.  No device memory is allocated here
// and nothing synchronises with the host.
#include <math.h>
#include <string.h>

#include "../../include/meteora.h"
#include "common.hpp"
#include "kernels.hpp"

using namespace meteora;

namespace {

struct WsLayout {
    size_t wsplit, partials, chunk_counts, counts, offsets, bucket_tok, bucket_slot, topk_idx, topk_w, h32,
        hdense, apack, hpart, splitk, btrans, wcat, dpart, gpart, spart, total;
    int ext_stride;   // columns of hdense: N*r rounded up to 64 (one K tile of the GEMM)
};

bool shape_ok(int T, int d_in, int d_out, int N, int r, int k) {
    return T >= 0 && d_in >= 1 && d_out >= 1 && N >= 1 && r >= 1 && k >= 1 && k <= N;
}

// Decode in two launches (gate logits and every adapter's shrink inside the GEMM's launch, then routing + reduce +
// expand): the split-K shapes whose adapters also have the Wcat operand.
bool decode_fused_applies(int T, int d_in, int d_out, int N, int r, bool bf16) {
    return route_small_applies(T, r, bf16) && gemm_splitk_splits(T, d_in, d_out, bf16) > 0 &&
           route_dense_possible(d_in, N, r, bf16);
}

// Mid-sized batches whose 128 x 128 output tiles would leave most CUs idle (a few hundred tokens): the base
// projection is split along K over workgroups like the routing products (fp32 tiles), and the reduction adds the
// LoRA expand, as for decode.  Returns the number of K splits, 0 = the fused GEMM runs instead.
int dense_midsplit_splits(int T, int d_in, int d_out, int N, int r, bool bf16) {
    // measured on 4096 -> 4096, 4096 -> 14336 and 14336 -> 4096, T = 65 ... 2048: the split form wins as long as the
    // projection can still be cut into at least two K splits of at most one workgroup per CU (19.0 against 56.1 us
    // at T = 65, 36.1 against 60.1 at T = 512, 45.6 against 48.7 at T = 704, 47.6 against 48.8 at T = 768 for
    // 4096 -> 4096; 43.3 against 47.6 at T = 160 for 4096 -> 14336; 107 against 131 at T = 704 for 14336 -> 4096);
    // up to 128 tokens, where the tiles are 128 rows high, up to about 160 output tiles
    const int64_t tiles = (int64_t)ceil_div(T, 128) * ceil_div(d_out, 128);
    if (!route_dense_applies(T, d_in, N, r, bf16) || (T <= 128 && tiles > 160) || d_out % 8 != 0 ||
        !gemm_dense_splitk_ok(T, d_in, d_out))
        return 0;
    const int S = gemm_multi_cap_splits(T, ceil_div(d_out, 128) + ceil_div(prep_wcat_rows(N, r), 128),
                                        gemm_dense_splits(T, d_in, d_out));
    return S >= 2 ? S : 0;
}

bool shape_supported(int T, int d_in, int d_out, int N, int r, int k) {
    return N <= kMaxAdapters && k <= kMaxTopK && r <= kMaxRank && d_in % 8 == 0 && d_out % 8 == 0 &&
           (int64_t)T * k < (int64_t)INT32_MAX && (int64_t)T * (int64_t)(d_in > d_out ? d_in : d_out) < ((int64_t)1 << 40);
}

WsLayout ws_layout(int T, int d_in, int d_out, int N, int r, int k, bool bf16) {
    WsLayout L{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const int NP = padded_adapters(N);
    const size_t pairs = (size_t)T * k;
    L.ext_stride = (int)align_up((size_t)N * r, 64);
    L.wsplit = take(gate_wsplit_bytes(d_in, N, bf16));
    L.partials = take((size_t)gate_kslices(d_in, bf16) * T * NP * sizeof(float));
    L.chunk_counts = take((size_t)bucket_chunks(T) * N * sizeof(int32_t));
    L.counts = take((size_t)N * sizeof(int32_t));
    L.offsets = take((size_t)(N + 1) * sizeof(int32_t));
    L.bucket_tok = take(pairs * sizeof(int32_t));
    L.bucket_slot = take(pairs * sizeof(int32_t));
    L.topk_idx = take(pairs * sizeof(int32_t));
    L.topk_w = take(pairs * sizeof(float));
    L.h32 = take(pairs * r * sizeof(float));
    L.hdense = take((size_t)T * L.ext_stride * sizeof(uint16_t));
    L.apack = take(shrink_apack_bytes(d_in, N, r, bf16));
    L.hpart = take(shrink_hpart_bytes(T, d_in, r, k, bf16));
    L.splitk = take(gemm_splitk_bytes(T, d_in, d_out, bf16));
    L.btrans = take(prep_btrans_bytes(d_out, N, r, bf16));
    const bool dense = route_dense_applies(T, d_in, N, r, bf16);
    const bool decode3 = decode_fused_applies(T, d_in, d_out, N, r, bf16);
    L.wcat = take(dense || decode3 ? prep_wcat_bytes(d_in, N, r, bf16) : 0);
    // the routing products come in the K splits of the launch that writes them: the products launch's own count, or
    // that of the split base projection when both share one launch (which may be the larger of the two)
    const int S_mid = dense_midsplit_splits(T, d_in, d_out, N, r, bf16);
    L.dpart = take(S_mid > 0 ? (size_t)S_mid * T * prep_wcat_rows(N, r) * sizeof(float)
                             : route_dense_part_bytes(T, d_in, N, r, bf16));
    L.gpart = take(decode3 ? (size_t)gemm_splitk_splits(T, d_in, d_out, bf16) * T * prep_wcat_rows(N, r) * sizeof(float) : 0);
    L.spart = take((size_t)S_mid * T * d_out * sizeof(float));
    L.total = off;
    return L;
}

// Packed weights (meteora_pack_weights): the three operand layouts, each 256-byte aligned.
struct PackLayout { size_t wsplit, apack, btrans, wcat, total; };

PackLayout pack_layout(int d_in, int d_out, int N, int r, bool bf16) {
    PackLayout P{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    P.wsplit = take(gate_wsplit_bytes(d_in, N, bf16));
    P.apack = take(shrink_apack_bytes(d_in, N, r, bf16));
    P.btrans = take(prep_btrans_bytes(d_out, N, r, bf16));
    P.wcat = take(route_dense_possible(d_in, N, r, bf16) ? prep_wcat_bytes(d_in, N, r, bf16) : 0);
    P.total = off;
    return P;
}

// Where the kernels find the packed operands: in the caller's blob, or in the workspace after a prep launch.
struct PackedPtrs { void* wsplit; void* apack; void* btrans; void* wcat; };

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }
inline bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }
template <typename T> T* at(void* ws, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(ws) + off); }

#define METEORA_HIP(expr)                              \
    do {                                               \
        if ((expr) != hipSuccess) return METEORA_ERR_HIP; \
    } while (0)

// ---- optional per-stage timing (off by default; hipEvents recorded between the launches) ----
enum Stage { ST_PREP = 0, ST_GATE_LOGITS, ST_GATE_TOPK, ST_BUCKET, ST_SHRINK, ST_GEMM, ST_EXPAND, ST_COUNT };
constexpr int kTimingRing = 256;
struct StageTiming {
    bool on = false;
    int calls = 0;
    hipEvent_t ev[kTimingRing][ST_COUNT][2];
    bool used[kTimingRing][ST_COUNT];
} g_timing;

struct StageScope {
    int stage;
    hipStream_t st;
    int slot;
    StageScope(int stage_, hipStream_t st_, int slot_) : stage(stage_), st(st_), slot(slot_) {
        if (slot >= 0) { (void)hipEventRecord(g_timing.ev[slot][stage][0], st); }
    }
    ~StageScope() {
        if (slot >= 0) { (void)hipEventRecord(g_timing.ev[slot][stage][1], st); g_timing.used[slot][stage] = true; }
    }
};

int timing_begin_call(hipStream_t) {
    if (!g_timing.on || g_timing.calls >= kTimingRing) return -1;
    return g_timing.calls++;
}

}  // namespace

extern "C" {

int meteora_stage_count(void) { return ST_COUNT; }

const char* meteora_stage_name(int stage) {
    static const char* names[ST_COUNT] = {"prep", "gate_logits", "gate_topk", "bucket", "shrink", "gemm", "expand"};
    return (stage >= 0 && stage < ST_COUNT) ? names[stage] : "";
}

meteora_status meteora_stage_timing_enable(int on) {
    if (on && !g_timing.on) {
        for (int c = 0; c < kTimingRing; ++c)
            for (int s = 0; s < ST_COUNT; ++s) {
                METEORA_HIP(hipEventCreate(&g_timing.ev[c][s][0]));
                METEORA_HIP(hipEventCreate(&g_timing.ev[c][s][1]));
                g_timing.used[c][s] = false;
            }
        g_timing.calls = 0;
        g_timing.on = true;
    } else if (!on && g_timing.on) {
        for (int c = 0; c < kTimingRing; ++c)
            for (int s = 0; s < ST_COUNT; ++s) {
                (void)hipEventDestroy(g_timing.ev[c][s][0]);
                (void)hipEventDestroy(g_timing.ev[c][s][1]);
            }
        g_timing.on = false;
    }
    return METEORA_OK;
}

meteora_status meteora_stage_timing_read(float* ms_sum, int* launches, int* calls) {
    if (!ms_sum || !launches || !calls) return METEORA_ERR_INVALID_ARG;
    if (!g_timing.on) return METEORA_ERR_INVALID_ARG;
    for (int s = 0; s < ST_COUNT; ++s) { ms_sum[s] = 0.f; launches[s] = 0; }
    for (int c = 0; c < g_timing.calls; ++c)
        for (int s = 0; s < ST_COUNT; ++s) {
            if (!g_timing.used[c][s]) continue;
            METEORA_HIP(hipEventSynchronize(g_timing.ev[c][s][1]));
            float ms = 0.f;
            METEORA_HIP(hipEventElapsedTime(&ms, g_timing.ev[c][s][0], g_timing.ev[c][s][1]));
            ms_sum[s] += ms;
            launches[s] += 1;
            g_timing.used[c][s] = false;
        }
    *calls = g_timing.calls;
    g_timing.calls = 0;
    return METEORA_OK;
}

int meteora_version(void) { return 200; }

meteora_status meteora_init(int device) {
    int cur = 0;
    if (hipGetDevice(&cur) != hipSuccess) return METEORA_ERR_HIP;
    const bool other = device >= 0 && device != cur;
    if (other && hipSetDevice(device) != hipSuccess) return METEORA_ERR_INVALID_ARG;
    const hipError_t e = init_kernels();
    if (other) (void)hipSetDevice(cur);
    return e == hipSuccess ? METEORA_OK : METEORA_ERR_HIP;
}

const char* meteora_status_string(meteora_status s) {
    switch (s) {
        case METEORA_OK: return "ok";
        case METEORA_ERR_INVALID_ARG: return "invalid argument";
        case METEORA_ERR_UNSUPPORTED: return "unsupported shape, dtype or alignment";
        case METEORA_ERR_WORKSPACE: return "workspace missing or too small";
        case METEORA_ERR_HIP: return "HIP launch error";
        case METEORA_ERR_TOO_LARGE: return "problem larger than the fixed scratch of a call that takes no workspace";
    }
    return "unknown status";
}

size_t meteora_workspace_bytes(int T, int d_in, int d_out, int N, int r, int k, meteora_dtype dt) {
    if (!shape_ok(T, d_in, d_out, N, r, k) || !shape_supported(T, d_in, d_out, N, r, k)) return 0;
    if (dt != METEORA_F32 && dt != METEORA_BF16) return 0;
    return ws_layout(T, d_in, d_out, N, r, k, dt == METEORA_BF16).total + 256;
}

// Host-only audit of the workspace carving of meteora_linear_forward(_packed): for every region, where it starts,
// how many bytes the layout reserves and how many bytes the launch sequence that this shape selects writes there.
// The written extents are derived from the launch decisions (which path, how many K splits), not from the layout's
// own size formulas, so that a region sized for another split count than the one that writes it shows up.
int meteora_workspace_regions(int T, int d_in, int d_out, int N, int r, int k, meteora_dtype dt, int with_packed,
                              const char** names, size_t* offset, size_t* reserved, size_t* written, int max_regions) {
    if (!shape_ok(T, d_in, d_out, N, r, k) || !shape_supported(T, d_in, d_out, N, r, k)) return -1;
    if (dt != METEORA_F32 && dt != METEORA_BF16) return -1;
    const bool bf16 = dt == METEORA_BF16;
    const WsLayout L = ws_layout(T, d_in, d_out, N, r, k, bf16);
    struct Region { const char* name; size_t off, written; };
    Region R[19] = {{"wsplit", L.wsplit, 0}, {"partials", L.partials, 0}, {"chunk_counts", L.chunk_counts, 0},
                    {"counts", L.counts, 0}, {"offsets", L.offsets, 0}, {"bucket_tok", L.bucket_tok, 0},
                    {"bucket_slot", L.bucket_slot, 0}, {"topk_idx", L.topk_idx, 0}, {"topk_w", L.topk_w, 0},
                    {"h32", L.h32, 0}, {"hdense", L.hdense, 0}, {"apack", L.apack, 0}, {"hpart", L.hpart, 0},
                    {"splitk", L.splitk, 0}, {"btrans", L.btrans, 0}, {"wcat", L.wcat, 0}, {"dpart", L.dpart, 0},
                    {"gpart", L.gpart, 0}, {"spart", L.spart, 0}};
    auto wr = [&](const char* name, size_t bytes) {
        for (Region& g : R)
            if (strcmp(g.name, name) == 0 && bytes > g.written) g.written = bytes;
    };
    const int NP = padded_adapters(N);
    const size_t pairs = (size_t)T * k;
    const int CR = prep_wcat_rows(N, r);
    const bool dense = route_dense_applies(T, d_in, N, r, bf16);
    const bool decode3 = decode_fused_applies(T, d_in, d_out, N, r, bf16);
    wr("topk_idx", pairs * sizeof(int32_t));
    wr("topk_w", pairs * sizeof(float));
    if (!with_packed) {
        if (!dense && !decode3) { wr("wsplit", gate_wsplit_bytes(d_in, N, bf16)); wr("apack", shrink_apack_bytes(d_in, N, r, bf16)); }
        if (!decode3) wr("btrans", prep_btrans_bytes(d_out, N, r, bf16));
        if (dense || decode3) wr("wcat", prep_wcat_bytes(d_in, N, r, bf16));
    }
    if (decode3) {
        const int S = gemm_group_splits(T, d_in, &d_out, 1, CR);
        wr("splitk", (size_t)S * T * d_out * sizeof(float));
        wr("gpart", (size_t)S * T * CR * sizeof(float));
    } else if (dense) {
        if (const int S = dense_midsplit_splits(T, d_in, d_out, N, r, bf16)) {
            wr("spart", (size_t)S * T * d_out * sizeof(float));
            wr("dpart", (size_t)S * T * CR * sizeof(float));
            if (!decode_tail_applies(r)) wr("h32", pairs * r * sizeof(float));
        } else {
            wr("dpart", (size_t)gemm_dense_splits(T, d_in, CR) * T * CR * sizeof(float));
            wr("hdense", (size_t)T * L.ext_stride * sizeof(uint16_t));
        }
    } else {
        wr("partials", (size_t)gate_kslices(d_in, bf16) * T * NP * sizeof(float));
        const bool fused = gemm_fuses_expand(bf16);
        if (fused) wr("hdense", (size_t)T * L.ext_stride * sizeof(uint16_t));
        if (route_small_applies(T, r, bf16)) {
            const int S = gemm_splitk_splits(T, d_in, d_out, bf16);
            if (S > 0) wr("splitk", (size_t)(S + 1) * T * d_out * sizeof(float));
        } else {
            wr("chunk_counts", (size_t)bucket_chunks(T) * N * sizeof(int32_t));
            wr("counts", (size_t)N * sizeof(int32_t));
            wr("offsets", (size_t)(N + 1) * sizeof(int32_t));
            wr("bucket_tok", pairs * sizeof(int32_t));
            wr("bucket_slot", pairs * sizeof(int32_t));
            wr("hpart", shrink_hpart_bytes(T, d_in, r, k, bf16));
            if (!fused) wr("h32", pairs * r * sizeof(float));
            const int S = gemm_splitk_splits(T, d_in, d_out, bf16);
            if (fused && S > 0) wr("splitk", (size_t)(S + 1) * T * d_out * sizeof(float));
        }
    }
    const int n = (int)(sizeof(R) / sizeof(R[0]));
    for (int i = 0; i < n && i < max_regions; ++i) {
        const size_t end = i + 1 < n ? R[i + 1].off : L.total;
        if (names) names[i] = R[i].name;
        if (offset) offset[i] = R[i].off;
        if (reserved) reserved[i] = end - R[i].off;
        if (written) written[i] = R[i].written;
    }
    return n;
}

meteora_status meteora_gate_topk(const void* x, const float* W_gate, const float* gate_bias, int T, int d_in,
                                 int N, int k, meteora_dtype dt, float inv_temperature, int32_t* topk_idx,
                                 float* topk_w, float* logits, void* ws, size_t ws_bytes,
                                 meteora_stream stream) {
    if (!x || !W_gate || !topk_idx || !topk_w) return METEORA_ERR_INVALID_ARG;
    if (!shape_ok(T, d_in, 8, N, 1, k) || !isfinite(inv_temperature)) return METEORA_ERR_INVALID_ARG;
    if (dt != METEORA_F32 && dt != METEORA_BF16) return METEORA_ERR_UNSUPPORTED;
    if (!shape_supported(T, d_in, 8, N, 1, k)) return METEORA_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(W_gate) || !aligned16(topk_idx) || !aligned16(topk_w) ||
        (logits && !aligned16(logits)) || (gate_bias && !aligned4(gate_bias)))
        return METEORA_ERR_UNSUPPORTED;
    const bool bf16 = dt == METEORA_BF16;
    const WsLayout L = ws_layout(T, d_in, 8, N, 1, k, bf16);
    if (!ws || !aligned256(ws) || ws_bytes < L.chunk_counts) return METEORA_ERR_WORKSPACE;
    if (T == 0) return METEORA_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float* partials = at<float>(ws, L.partials);
    if (gate_wsplit_bytes(d_in, N, bf16) > 0)
        METEORA_HIP(launch_prep(W_gate, at<void>(ws, L.wsplit), nullptr, nullptr, nullptr, nullptr, nullptr, d_in, 8, N,
                                1, st));
    METEORA_HIP(launch_gate_logits(x, W_gate, T, d_in, N, bf16, at<void>(ws, L.wsplit), partials, st));
    METEORA_HIP(launch_gate_topk(partials, gate_kslices(d_in, bf16), gate_bias, T, N, k, inv_temperature,
                                 topk_idx, topk_w, logits, nullptr, st));
    return METEORA_OK;
}

meteora_status meteora_bucket_tokens(const int32_t* topk_idx, int T, int k, int N, int32_t* counts,
                                     int32_t* offsets, int32_t* bucket_tok, int32_t* bucket_slot, void* ws,
                                     size_t ws_bytes, meteora_stream stream) {
    if (!topk_idx || !counts || !offsets || !bucket_tok || !bucket_slot) return METEORA_ERR_INVALID_ARG;
    if (!shape_ok(T, 8, 8, N, 1, k)) return METEORA_ERR_INVALID_ARG;
    if (!shape_supported(T, 8, 8, N, 1, k)) return METEORA_ERR_UNSUPPORTED;
    if (!aligned16(topk_idx) || !aligned4(counts) || !aligned4(offsets) || !aligned16(bucket_tok) ||
        !aligned16(bucket_slot))
        return METEORA_ERR_UNSUPPORTED;
    // only the chunk histograms live in the workspace; they sit at offset 0 for this entry point
    const size_t need = (size_t)bucket_chunks(T) * N * sizeof(int32_t);
    if (!ws || !aligned256(ws) || ws_bytes < need) return METEORA_ERR_WORKSPACE;
    if (T == 0) {
        // nothing to enqueue; counts/offsets of an empty batch are left to the caller
        return METEORA_OK;
    }
    METEORA_HIP(launch_bucket(topk_idx, T, k, N, static_cast<int32_t*>(ws), false, counts, offsets, bucket_tok,
                              bucket_slot, nullptr, 0, static_cast<hipStream_t>(stream)));
    return METEORA_OK;
}

meteora_status meteora_bucket_tokens_noalloc(const int32_t* topk_idx, int T, int k, int N, int32_t* counts,
                                             int32_t* offsets, int32_t* bucket_tok, int32_t* bucket_slot,
                                             meteora_stream stream) {
    if (!topk_idx || !counts || !offsets || !bucket_tok || !bucket_slot) return METEORA_ERR_INVALID_ARG;
    if (!shape_ok(T, 8, 8, N, 1, k)) return METEORA_ERR_INVALID_ARG;
    if (!shape_supported(T, 8, 8, N, 1, k)) return METEORA_ERR_UNSUPPORTED;
    if (T > kStaticBucketMaxTokens) return METEORA_ERR_TOO_LARGE;   // beyond the library's fixed scratch
    if (!aligned16(topk_idx) || !aligned4(counts) || !aligned4(offsets) || !aligned16(bucket_tok) ||
        !aligned16(bucket_slot))
        return METEORA_ERR_UNSUPPORTED;
    if (T == 0) return METEORA_OK;
    int32_t* chunk_counts = nullptr;   // the current device's copy of the library's scratch array
    METEORA_HIP(bucket_static_scratch(&chunk_counts));
    METEORA_HIP(launch_bucket(topk_idx, T, k, N, chunk_counts, false, counts, offsets, bucket_tok, bucket_slot, nullptr,
                              0, static_cast<hipStream_t>(stream)));
    return METEORA_OK;
}

static meteora_status check_lora_args(const void* x, const void* A, const void* B, int T, int d_in, int d_out,
                                      int N, int r, int k, float scale, meteora_dtype dt, const void* out) {
    if (!x || !A || !B || !out) return METEORA_ERR_INVALID_ARG;
    if (!shape_ok(T, d_in, d_out, N, r, k) || !isfinite(scale)) return METEORA_ERR_INVALID_ARG;
    if (dt != METEORA_F32 && dt != METEORA_BF16) return METEORA_ERR_UNSUPPORTED;
    if (!shape_supported(T, d_in, d_out, N, r, k)) return METEORA_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(A) || !aligned16(B) || !aligned16(out)) return METEORA_ERR_UNSUPPORTED;
    return METEORA_OK;
}

// bucketing + shrink + (base projection if W != NULL) + expand on a given routing;
// shared by lora_forward (W == NULL) and linear_forward
static meteora_status run_lora(const void* x, const void* W, const void* A, const void* B, const int32_t* topk_idx,
                               const float* topk_w, int T, int d_in, int d_out, int N, int r, int k, float scale,
                               bool bf16, void* out, int accumulate, void* ws, const WsLayout& L,
                               const PackedPtrs& pk, hipStream_t st, int tslot, bool have_hist) {
    int32_t* offsets = at<int32_t>(ws, L.offsets);
    int32_t* btok = at<int32_t>(ws, L.bucket_tok);
    int32_t* bslot = at<int32_t>(ws, L.bucket_slot);
    float* h32 = at<float>(ws, L.h32);
    const bool fused = gemm_fuses_expand(bf16);
    {
        StageScope sc(ST_BUCKET, st, tslot);
        const bool clear = fused && !shrink_clears_hdense(bf16, r, T, k);
        METEORA_HIP(launch_bucket(topk_idx, T, k, N, at<int32_t>(ws, L.chunk_counts), have_hist,
                                  at<int32_t>(ws, L.counts), offsets, btok, bslot,
                                  clear ? at<void>(ws, L.hdense) : nullptr, L.ext_stride * (int)sizeof(uint16_t), st));
    }
    {
        StageScope sc(ST_SHRINK, st, tslot);
        METEORA_HIP(launch_shrink(x, A, topk_idx, topk_w, offsets, btok, bslot, T, d_in, N, r, k, scale, bf16,
                                  pk.apack, at<float>(ws, L.hpart), fused ? nullptr : h32,
                                  fused ? at<void>(ws, L.hdense) : nullptr, L.ext_stride, st));
    }
    if (fused) {
        // base projection (if W is given) and LoRA expand in one MFMA kernel, one rounding of the output
        StageScope sc(ST_GEMM, st, tslot);
        METEORA_HIP(launch_gemm(x, W, T, W ? d_in : 0, d_out, bf16, at<void>(ws, L.hdense), L.ext_stride,
                                pk.btrans, N * r, out, accumulate,
                                gemm_splitk_bytes(T, d_in, d_out, bf16) > 0 ? at<float>(ws, L.splitk) : nullptr, st));
    } else {
        if (W) {
            StageScope sc(ST_GEMM, st, tslot);
            METEORA_HIP(launch_gemm(x, W, T, d_in, d_out, bf16, nullptr, 0, nullptr, 0, out, accumulate, nullptr, st));
        }
        StageScope sc(ST_EXPAND, st, tslot);
        METEORA_HIP(launch_expand(h32, B, topk_idx, topk_w, T, d_out, N, r, k, scale, bf16, out,
                                  W ? 1 : accumulate, st));
    }
    return METEORA_OK;
}

meteora_status meteora_lora_forward(const void* x, const void* A, const void* B, const int32_t* topk_idx,
                                    const float* topk_w, int T, int d_in, int d_out, int N, int r, int k,
                                    float scale, meteora_dtype dt, void* out, int accumulate, void* ws,
                                    size_t ws_bytes, meteora_stream stream) {
    if (!topk_idx || !topk_w) return METEORA_ERR_INVALID_ARG;
    if (accumulate != 0 && accumulate != 1) return METEORA_ERR_INVALID_ARG;
    meteora_status s = check_lora_args(x, A, B, T, d_in, d_out, N, r, k, scale, dt, out);
    if (s != METEORA_OK) return s;
    if (!aligned16(topk_idx) || !aligned16(topk_w)) return METEORA_ERR_UNSUPPORTED;
    const bool bf16 = dt == METEORA_BF16;
    const WsLayout L = ws_layout(T, d_in, d_out, N, r, k, bf16);
    if (!ws || !aligned256(ws) || ws_bytes < L.total) return METEORA_ERR_WORKSPACE;
    if (T == 0) return METEORA_OK;
    {
        const bool pa = shrink_apack_bytes(d_in, N, r, bf16) > 0, pb = prep_btrans_bytes(d_out, N, r, bf16) > 0;
        METEORA_HIP(launch_prep(nullptr, nullptr, pa ? A : nullptr, pa ? at<void>(ws, L.apack) : nullptr,
                                pb ? B : nullptr, pb ? at<void>(ws, L.btrans) : nullptr, nullptr, d_in, d_out, N, r,
                                static_cast<hipStream_t>(stream)));
    }
    const PackedPtrs pk{nullptr, at<void>(ws, L.apack), at<void>(ws, L.btrans), nullptr};
    return run_lora(x, nullptr, A, B, topk_idx, topk_w, T, d_in, d_out, N, r, k, scale, bf16, out, accumulate, ws, L,
                    pk, static_cast<hipStream_t>(stream), timing_begin_call(static_cast<hipStream_t>(stream)), false);
}

meteora_status meteora_base_gemm(const void* x, const void* W, int T, int d_in, int d_out, meteora_dtype dt,
                                 void* out, meteora_stream stream) {
    if (!x || !W || !out) return METEORA_ERR_INVALID_ARG;
    if (!shape_ok(T, d_in, d_out, 1, 1, 1)) return METEORA_ERR_INVALID_ARG;
    if (dt != METEORA_F32 && dt != METEORA_BF16) return METEORA_ERR_UNSUPPORTED;
    if (!shape_supported(T, d_in, d_out, 1, 1, 1)) return METEORA_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(W) || !aligned16(out)) return METEORA_ERR_UNSUPPORTED;
    if (T == 0) return METEORA_OK;
    METEORA_HIP(launch_gemm(x, W, T, d_in, d_out, dt == METEORA_BF16, nullptr, 0, nullptr, 0, out, 0, nullptr,
                            static_cast<hipStream_t>(stream)));
    return METEORA_OK;
}

size_t meteora_packed_bytes(int d_in, int d_out, int N, int r, meteora_dtype dt) {
    if (!shape_ok(0, d_in, d_out, N, r, 1) || !shape_supported(0, d_in, d_out, N, r, 1)) return 0;
    if (dt != METEORA_F32 && dt != METEORA_BF16) return 0;
    return pack_layout(d_in, d_out, N, r, dt == METEORA_BF16).total;
}

meteora_status meteora_pack_weights(const float* W_gate, const void* A, const void* B, int d_in, int d_out, int N,
                                    int r, meteora_dtype dt, void* packed, size_t packed_bytes,
                                    meteora_stream stream) {
    if (!W_gate || !A || !B) return METEORA_ERR_INVALID_ARG;
    if (!shape_ok(0, d_in, d_out, N, r, 1)) return METEORA_ERR_INVALID_ARG;
    if (dt != METEORA_F32 && dt != METEORA_BF16) return METEORA_ERR_UNSUPPORTED;
    if (!shape_supported(0, d_in, d_out, N, r, 1)) return METEORA_ERR_UNSUPPORTED;
    if (!aligned16(W_gate) || !aligned16(A) || !aligned16(B)) return METEORA_ERR_UNSUPPORTED;
    const bool bf16 = dt == METEORA_BF16;
    const PackLayout P = pack_layout(d_in, d_out, N, r, bf16);
    if (P.total == 0) return METEORA_OK;   // this dtype reads the tensors as they are
    if (!packed || !aligned256(packed) || packed_bytes < P.total) return METEORA_ERR_WORKSPACE;
    const bool pw = gate_wsplit_bytes(d_in, N, bf16) > 0, pa = shrink_apack_bytes(d_in, N, r, bf16) > 0;
    const bool pb = prep_btrans_bytes(d_out, N, r, bf16) > 0, pc = route_dense_possible(d_in, N, r, bf16);
    METEORA_HIP(launch_prep(W_gate, pw ? at<void>(packed, P.wsplit) : nullptr, A,
                            pa ? at<void>(packed, P.apack) : nullptr, pb ? B : nullptr,
                            pb ? at<void>(packed, P.btrans) : nullptr, pc ? at<void>(packed, P.wcat) : nullptr, d_in,
                            d_out, N, r, static_cast<hipStream_t>(stream)));
    return METEORA_OK;
}

meteora_status meteora_linear_forward_packed(const void* x, const void* W, const float* W_gate,
                                             const float* gate_bias, const void* A, const void* B,
                                             const void* packed, size_t packed_bytes, int T, int d_in, int d_out,
                                             int N, int r, int k, float scale, float inv_temperature,
                                             meteora_dtype dt, void* out, int32_t* topk_idx_out, float* topk_w_out,
                                             void* ws, size_t ws_bytes, meteora_stream stream) {
    if (!W || !W_gate || !isfinite(inv_temperature)) return METEORA_ERR_INVALID_ARG;
    meteora_status s = check_lora_args(x, A, B, T, d_in, d_out, N, r, k, scale, dt, out);
    if (s != METEORA_OK) return s;
    if (!aligned16(W) || !aligned16(W_gate) || (gate_bias && !aligned4(gate_bias)) ||
        (topk_idx_out && !aligned16(topk_idx_out)) || (topk_w_out && !aligned16(topk_w_out)))
        return METEORA_ERR_UNSUPPORTED;
    const bool bf16 = dt == METEORA_BF16;
    const WsLayout L = ws_layout(T, d_in, d_out, N, r, k, bf16);
    if (!ws || !aligned256(ws) || ws_bytes < L.total) return METEORA_ERR_WORKSPACE;
    const PackLayout P = pack_layout(d_in, d_out, N, r, bf16);
    const bool use_packed = packed != nullptr && P.total > 0;
    if (use_packed && (!aligned256(packed) || packed_bytes < P.total)) return METEORA_ERR_WORKSPACE;
    if (T == 0) return METEORA_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int32_t* idx = topk_idx_out ? topk_idx_out : at<int32_t>(ws, L.topk_idx);
    float* w = topk_w_out ? topk_w_out : at<float>(ws, L.topk_w);
    float* partials = at<float>(ws, L.partials);
    const int tslot = timing_begin_call(st);
    // mid-sized batch: gate logits and the shrink of every adapter in one MFMA launch, selection afterwards
    const bool dense = route_dense_applies(T, d_in, N, r, bf16);
    const bool decode3 = decode_fused_applies(T, d_in, d_out, N, r, bf16);
    PackedPtrs pk{at<void>(ws, L.wsplit), at<void>(ws, L.apack), at<void>(ws, L.btrans), at<void>(ws, L.wcat)};
    if (use_packed) {
        void* blob = const_cast<void*>(packed);   // read only from here on
        pk = PackedPtrs{at<void>(blob, P.wsplit), at<void>(blob, P.apack), at<void>(blob, P.btrans),
                        at<void>(blob, P.wcat)};
    } else {
        // only the operands this batch size reads are packed
        StageScope sc(ST_PREP, st, tslot);
        const bool pw = !dense && !decode3 && gate_wsplit_bytes(d_in, N, bf16) > 0;
        const bool pa = !dense && !decode3 && shrink_apack_bytes(d_in, N, r, bf16) > 0;
        const bool pb = !decode3 && prep_btrans_bytes(d_out, N, r, bf16) > 0;
        METEORA_HIP(launch_prep(W_gate, pw ? pk.wsplit : nullptr, A, pa ? pk.apack : nullptr, pb ? B : nullptr,
                                pb ? pk.btrans : nullptr, dense || decode3 ? pk.wcat : nullptr, d_in, d_out, N, r, st));
    }
    if (decode3) {
        // decode-sized batch: the launch that streams W also computes the gate logits; then top-k, softmax and the
        // shrink of the selected adapters token by token; then the split-K reduction, which adds the expand
        const DecodeMember mem{W, pk.wcat, gate_bias, A, B, d_out, at<float>(ws, L.splitk), at<float>(ws, L.gpart),
                               at<float>(ws, L.h32), idx, w, out};
        const int gate_rows = prep_wcat_rows(N, r);   // the gate terms and every adapter's shrink columns
        const int S = gemm_group_splits(T, d_in, &d_out, 1, gate_rows);
        {
            StageScope sc(ST_GEMM, st, tslot);
            METEORA_HIP(launch_gemm_decode_main(x, &mem, 1, gate_rows, S, T, d_in, st));
        }
        // top-k, softmax, then the split-K reduction with the expand from the selected adapters' shrink tiles: one launch
        StageScope sc(ST_SHRINK, st, tslot);
        METEORA_HIP(launch_decode_tail_group(&mem, 1, S, T, N, r, k, gate_rows, inv_temperature, scale, st));
        return METEORA_OK;
    }
    if (dense) {
        float* dpart = at<float>(ws, L.dpart);
        if (const int S = dense_midsplit_splits(T, d_in, d_out, N, r, bf16)) {
            // few output tiles: x * W^T and x * Wcat^T as fp32 K-split tiles of one launch, selection, then the
            // reduction with the expand (the decode sequence with 128 x 128 tiles and the dense selection)
            float* hs = at<float>(ws, L.h32);
            DecodeMember mem{W, nullptr, gate_bias, A, B, d_out, at<float>(ws, L.spart), dpart, hs, idx, w, out};
            {
                StageScope sc(ST_GEMM, st, tslot);
                const DenseOperand two[2] = {{W, d_out, mem.partial}, {pk.wcat, prep_wcat_rows(N, r), dpart}};
                METEORA_HIP(launch_gemm_dense_splitk_multi(x, two, 2, S, T, d_in, st));
            }
            if (decode_tail_applies(r)) {   // selection, reduction and expand in one launch, as for decode
                StageScope sc(ST_SHRINK, st, tslot);
                METEORA_HIP(launch_decode_tail_group(&mem, 1, S, T, N, r, k, prep_wcat_rows(N, r), inv_temperature, scale, st));
                return METEORA_OK;
            }
            {
                StageScope sc(ST_GATE_TOPK, st, tslot);
                METEORA_HIP(launch_route_dense_select(dpart, gate_bias, T, d_in, N, r, k, inv_temperature, scale, idx, w, nullptr,
                                                      L.ext_stride, st, hs, S));
            }
            StageScope sc(ST_EXPAND, st, tslot);
            METEORA_HIP(launch_gemm_decode_finish(&mem, 1, S, T, k, r, st));
            return METEORA_OK;
        }
        {
            StageScope sc(ST_GATE_LOGITS, st, tslot);
            METEORA_HIP(launch_route_dense_products(x, pk.wcat, T, d_in, N, r, dpart, st));
        }
        {
            StageScope sc(ST_GATE_TOPK, st, tslot);
            METEORA_HIP(launch_route_dense_select(dpart, gate_bias, T, d_in, N, r, k, inv_temperature, scale, idx, w,
                                                  at<void>(ws, L.hdense), L.ext_stride, st));
        }
        StageScope sc(ST_GEMM, st, tslot);
        METEORA_HIP(launch_gemm(x, W, T, d_in, d_out, bf16, at<void>(ws, L.hdense), L.ext_stride, pk.btrans, N * r,
                                out, 0, nullptr, st));
        return METEORA_OK;
    }
    {
        StageScope sc(ST_GATE_LOGITS, st, tslot);
        METEORA_HIP(launch_gate_logits(x, W_gate, T, d_in, N, bf16, pk.wsplit, partials, st));
    }
    if (route_small_applies(T, r, bf16)) {
        // decode-sized batch: top-k, softmax and the shrink of the selected adapters in one launch, then the GEMM
        {
            StageScope sc(ST_SHRINK, st, tslot);
            METEORA_HIP(launch_route_shrink_small(x, partials, gate_kslices(d_in, bf16), gate_bias, A, T, d_in, N, r,
                                                  k, inv_temperature, scale, idx, w, at<void>(ws, L.hdense), L.ext_stride, st));
        }
        StageScope sc(ST_GEMM, st, tslot);
        METEORA_HIP(launch_gemm(x, W, T, d_in, d_out, bf16, at<void>(ws, L.hdense), L.ext_stride, pk.btrans, N * r,
                                out, 0, gemm_splitk_bytes(T, d_in, d_out, bf16) > 0 ? at<float>(ws, L.splitk) : nullptr,
                                st));
        return METEORA_OK;
    }
    {
        StageScope sc(ST_GATE_TOPK, st, tslot);
        METEORA_HIP(launch_gate_topk(partials, gate_kslices(d_in, bf16), gate_bias, T, N, k, inv_temperature, idx, w,
                                     nullptr, at<int32_t>(ws, L.chunk_counts), st));
    }
    return run_lora(x, W, A, B, idx, w, T, d_in, d_out, N, r, k, scale, bf16, out, 0, ws, L, pk, st, tslot, true);
}

}  // extern "C"

// ---- a group of layers that share x ----------------------------------------------------------------------------
namespace {

// Fused form: decode-sized batch, every member on the two-launch path with packed weights.
bool group_fused(const meteora_group_member* m, int G, int T, int d_in, int N, int r, bool bf16) {
    if (G < 2 || G > kMaxDecodeGroup) return false;
    for (int g = 0; g < G; ++g)
        if (!m[g].packed || !decode_fused_applies(T, d_in, m[g].d_out, N, r, bf16)) return false;
    return true;
}

// Second fused form: a few hundred tokens, every member on the dense routing path with packed weights, few output
// tiles in all: the projections and routing products of all members as K-split tiles of one launch, one selection
// launch, one reduction with the expands.  Returns the number of K splits, 0 = not this form.
int group_mid_splits(const int* d_out, const bool* packed, int G, int T, int d_in, int N, int r, bool bf16) {
    if (G < 2 || G > kMaxDecodeGroup || !route_dense_applies(T, d_in, N, r, bf16)) return 0;
    const int cat_rows = prep_wcat_rows(N, r);
    int64_t tiles = 0;
    for (int g = 0; g < G; ++g) {
        if (!packed[g] || d_out[g] % 8 != 0 || !gemm_dense_splitk_ok(T, d_in, d_out[g])) return 0;
        tiles += (int64_t)ceil_div(T, 128) * (ceil_div(d_out[g], 128) + ceil_div(cat_rows, 128));
    }
    if (tiles > 320) return 0;   // beyond: member by member (each on the path its own size selects)
    const int nk = d_in / 64;
    int S = (int)((384 + tiles / 2) / tiles);
    if (S > nk / 4) S = nk / 4;
    if (S > 8) S = 8;
    int col_tiles = 0;
    for (int g = 0; g < G; ++g) col_tiles += ceil_div(d_out[g], 128) + ceil_div(cat_rows, 128);
    S = gemm_multi_cap_splits(T, col_tiles, S);
    return S < 1 ? 1 : S;
}

struct GroupLayout { size_t partial[kMaxDecodeGroup], gpart[kMaxDecodeGroup], hs[kMaxDecodeGroup], idx[kMaxDecodeGroup],
                            w[kMaxDecodeGroup], total; int S; };

// gate_rows: columns of gpart per member (the gate terms for decode, every row of Wcat for the second form)
GroupLayout group_layout(const int* d_out, int G, int T, int d_in, int N, int r, int k, int S, int gate_rows) {
    GroupLayout L{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    L.S = S;
    for (int g = 0; g < G; ++g) {
        L.partial[g] = take((size_t)L.S * T * d_out[g] * sizeof(float));
        L.gpart[g] = take((size_t)L.S * T * gate_rows * sizeof(float));
        L.hs[g] = take((size_t)T * k * r * sizeof(float));
        L.idx[g] = take((size_t)T * k * sizeof(int32_t));
        L.w[g] = take((size_t)T * k * sizeof(float));
    }
    L.total = off;
    return L;
}

}  // namespace

extern "C" size_t meteora_group_workspace_bytes(const int* d_out, int G, int T, int d_in, int N, int r, int k,
                                                meteora_dtype dt) {
    if (!d_out || G < 1 || G > 64) return 0;
    if (dt != METEORA_F32 && dt != METEORA_BF16) return 0;
    const bool bf16 = dt == METEORA_BF16;
    size_t need = 0;
    bool fused = G >= 2 && G <= kMaxDecodeGroup;
    for (int g = 0; g < G; ++g) {
        const size_t one = meteora_workspace_bytes(T, d_in, d_out[g], N, r, k, dt);
        if (one == 0) return 0;
        need = one > need ? one : need;
        fused = fused && decode_fused_applies(T, d_in, d_out[g], N, r, bf16);
    }
    if (fused) {
        const int gate_rows = prep_wcat_rows(N, r);
        const size_t f = group_layout(d_out, G, T, d_in, N, r, k, gemm_group_splits(T, d_in, d_out, G, gate_rows),
                                      gate_rows).total + 256;
        need = f > need ? f : need;
    }
    if (G >= 2 && G <= kMaxDecodeGroup) {
        bool all_packed[kMaxDecodeGroup] = {true, true, true, true};   // sized as if packed: the larger need
        if (const int S = group_mid_splits(d_out, all_packed, G, T, d_in, N, r, bf16)) {
            const size_t f = group_layout(d_out, G, T, d_in, N, r, k, S, prep_wcat_rows(N, r)).total + 256;
            need = f > need ? f : need;
        }
    }
    return need;
}

extern "C" meteora_status meteora_linear_forward_group(const void* x, const meteora_group_member* members, int G, int T,
                                                       int d_in, int N, int r, int k, float scale,
                                                       float inv_temperature, meteora_dtype dt, void* ws,
                                                       size_t ws_bytes, meteora_stream stream) {
    if (!members || G < 1 || G > 64 || !isfinite(inv_temperature)) return METEORA_ERR_INVALID_ARG;
    if (dt != METEORA_F32 && dt != METEORA_BF16) return METEORA_ERR_UNSUPPORTED;
    const bool bf16 = dt == METEORA_BF16;
    int d_outs[64];
    for (int g = 0; g < G; ++g) {
        const meteora_group_member& m = members[g];
        if (!m.W || !m.W_gate) return METEORA_ERR_INVALID_ARG;
        const meteora_status s = check_lora_args(x, m.A, m.B, T, d_in, m.d_out, N, r, k, scale, dt, m.out);
        if (s != METEORA_OK) return s;
        if (!aligned16(m.W) || !aligned16(m.W_gate) || (m.gate_bias && !aligned4(m.gate_bias)) ||
            (m.topk_idx_out && !aligned16(m.topk_idx_out)) || (m.topk_w_out && !aligned16(m.topk_w_out)))
            return METEORA_ERR_UNSUPPORTED;
        if (m.packed && (!aligned256(m.packed) ||
                         m.packed_bytes < pack_layout(d_in, m.d_out, N, r, bf16).total))
            return METEORA_ERR_WORKSPACE;
        d_outs[g] = m.d_out;
    }
    if (!ws || !aligned256(ws) || ws_bytes < meteora_group_workspace_bytes(d_outs, G, T, d_in, N, r, k, dt))
        return METEORA_ERR_WORKSPACE;
    if (T == 0) return METEORA_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    bool is_packed[64];
    for (int g = 0; g < G; ++g) is_packed[g] = members[g].packed != nullptr;
    if (const int S = (G <= kMaxDecodeGroup ? group_mid_splits(d_outs, is_packed, G, T, d_in, N, r, bf16) : 0)) {
        const int cat_rows = prep_wcat_rows(N, r);
        const GroupLayout L = group_layout(d_outs, G, T, d_in, N, r, k, S, cat_rows);
        DecodeMember mem[kMaxDecodeGroup];
        DenseOperand ops[2 * kMaxDecodeGroup];
        for (int g = 0; g < G; ++g) {
            const meteora_group_member& m = members[g];
            const PackLayout P = pack_layout(d_in, m.d_out, N, r, bf16);
            mem[g] = DecodeMember{m.W, at<void>(const_cast<void*>(m.packed), P.wcat), m.gate_bias, m.A, m.B, m.d_out,
                                  at<float>(ws, L.partial[g]), at<float>(ws, L.gpart[g]), at<float>(ws, L.hs[g]),
                                  m.topk_idx_out ? m.topk_idx_out : at<int32_t>(ws, L.idx[g]),
                                  m.topk_w_out ? m.topk_w_out : at<float>(ws, L.w[g]), m.out};
            ops[2 * g] = {mem[g].W, m.d_out, mem[g].partial};
            ops[2 * g + 1] = {mem[g].wg3, cat_rows, mem[g].gpartial};
        }
        const int tslot = timing_begin_call(st);
        {
            StageScope sc(ST_GEMM, st, tslot);
            METEORA_HIP(launch_gemm_dense_splitk_multi(x, ops, 2 * G, S, T, d_in, st));
        }
        if (decode_tail_applies(r)) {
            StageScope sc(ST_SHRINK, st, tslot);
            METEORA_HIP(launch_decode_tail_group(mem, G, S, T, N, r, k, cat_rows, inv_temperature, scale, st));
            return METEORA_OK;
        }
        {
            StageScope sc(ST_GATE_TOPK, st, tslot);
            METEORA_HIP(launch_route_dense_select_group(mem, G, S, T, N, r, k, inv_temperature, scale, st));
        }
        StageScope sc(ST_EXPAND, st, tslot);
        METEORA_HIP(launch_gemm_decode_finish(mem, G, S, T, k, r, st));
        return METEORA_OK;
    }
    if (!group_fused(members, G, T, d_in, N, r, bf16)) {
        // the same result one layer after the other (they share the workspace, which the stream order allows)
        for (int g = 0; g < G; ++g) {
            const meteora_group_member& m = members[g];
            const meteora_status s = meteora_linear_forward_packed(
                x, m.W, m.W_gate, m.gate_bias, m.A, m.B, m.packed, m.packed_bytes, T, d_in, m.d_out, N, r, k, scale,
                inv_temperature, dt, m.out, m.topk_idx_out, m.topk_w_out, ws, ws_bytes, stream);
            if (s != METEORA_OK) return s;
        }
        return METEORA_OK;
    }
    const int gate_rows = prep_wcat_rows(N, r);
    const GroupLayout L = group_layout(d_outs, G, T, d_in, N, r, k, gemm_group_splits(T, d_in, d_outs, G, gate_rows),
                                       gate_rows);
    DecodeMember mem[kMaxDecodeGroup];
    for (int g = 0; g < G; ++g) {
        const meteora_group_member& m = members[g];
        const PackLayout P = pack_layout(d_in, m.d_out, N, r, bf16);
        mem[g] = DecodeMember{m.W, at<void>(const_cast<void*>(m.packed), P.wcat), m.gate_bias, m.A, m.B, m.d_out,
                              at<float>(ws, L.partial[g]), at<float>(ws, L.gpart[g]), at<float>(ws, L.hs[g]),
                              m.topk_idx_out ? m.topk_idx_out : at<int32_t>(ws, L.idx[g]),
                              m.topk_w_out ? m.topk_w_out : at<float>(ws, L.w[g]), m.out};
    }
    const int tslot = timing_begin_call(st);
    {
        StageScope sc(ST_GEMM, st, tslot);
        METEORA_HIP(launch_gemm_decode_main(x, mem, G, gate_rows, L.S, T, d_in, st));
    }
    StageScope sc(ST_SHRINK, st, tslot);
    METEORA_HIP(launch_decode_tail_group(mem, G, L.S, T, N, r, k, gate_rows, inv_temperature, scale, st));
    return METEORA_OK;
}

extern "C" {

meteora_status meteora_linear_forward(const void* x, const void* W, const float* W_gate, const float* gate_bias,
                                      const void* A, const void* B, int T, int d_in, int d_out, int N, int r,
                                      int k, float scale, float inv_temperature, meteora_dtype dt, void* out,
                                      int32_t* topk_idx_out, float* topk_w_out, void* ws, size_t ws_bytes,
                                      meteora_stream stream) {
    return meteora_linear_forward_packed(x, W, W_gate, gate_bias, A, B, nullptr, 0, T, d_in, d_out, N, r, k, scale,
                                         inv_temperature, dt, out, topk_idx_out, topk_w_out, ws, ws_bytes, stream);
}

size_t meteora_gate_backward_workspace_bytes(int T, int d_in, int d_out, int N, int r, int k, meteora_dtype dt) {
    if (!shape_ok(T, d_in, d_out, N, r, k) || !shape_supported(T, d_in, d_out, N, r, k) || T < 1) return 0;
    if (!gate_backward_applies(T, d_in, d_out, N, r, dt == METEORA_BF16)) return 0;
    return gate_backward_layout(T, d_in, d_out, N, r).total;
}

meteora_status meteora_gate_backward(const void* x, const void* dy, const float* gate_bias, const void* B,
                                     const void* packed, size_t packed_bytes, const int32_t* topk_idx,
                                     const float* topk_w, const int32_t* labels, float beta, int T, int d_in,
                                     int d_out, int N, int r, int k, float scale, meteora_dtype dt, float* dW_gate,
                                     float* dbias, float* d_logits, const void* A, const float* W_gate,
                                     const void* W_t, void* dx, const void* forward_ws, size_t forward_ws_bytes,
                                     void* ws, size_t ws_bytes, meteora_stream stream) {
    if (!x || !dy || !B || !packed || !dW_gate || (topk_idx == nullptr) != (topk_w == nullptr))
        return METEORA_ERR_INVALID_ARG;
    if (dx != nullptr && (!A || !W_gate || !W_t)) return METEORA_ERR_INVALID_ARG;
    if (!shape_ok(T, d_in, d_out, N, r, k) || !isfinite(scale) || !isfinite(beta)) return METEORA_ERR_INVALID_ARG;
    if (dt != METEORA_BF16 && dt != METEORA_F32) return METEORA_ERR_INVALID_ARG;
    if (T == 0) return METEORA_OK;
    const bool bf16 = dt == METEORA_BF16;
    if (!shape_supported(T, d_in, d_out, N, r, k) || !gate_backward_applies(T, d_in, d_out, N, r, bf16))
        return METEORA_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(B) || !aligned16(dW_gate) || (gate_bias && !aligned4(gate_bias)) ||
        (dbias && !aligned4(dbias)) || (d_logits && !aligned4(d_logits)) || (labels && !aligned4(labels)) ||
        (topk_idx && (!aligned4(topk_idx) || !aligned4(topk_w))) ||
        (dx && (!aligned16(dx) || !aligned16(A) || !aligned16(W_gate) || !aligned16(W_t))))
        return METEORA_ERR_UNSUPPORTED;
    const PackLayout P = pack_layout(d_in, d_out, N, r, bf16);
    if (!aligned256(packed) || packed_bytes < P.total) return METEORA_ERR_WORKSPACE;
    const GateBackwardLayout L = gate_backward_layout(T, d_in, d_out, N, r);
    if (!ws || !aligned256(ws) || ws_bytes < L.total) return METEORA_ERR_WORKSPACE;
    const void* wcat = static_cast<const char*>(packed) + P.wcat;
    // the forward call of a mid-sized batch leaves x * Wcat^T in its workspace: take it instead of computing it again
    const float* part_x = nullptr;
    int part_x_splits = 0;
    if (forward_ws != nullptr && route_dense_applies(T, d_in, N, r, bf16)) {
        const WsLayout F = ws_layout(T, d_in, d_out, N, r, k, bf16);
        if (!aligned256(forward_ws) || forward_ws_bytes < F.total) return METEORA_ERR_WORKSPACE;
        part_x = reinterpret_cast<const float*>(static_cast<const char*>(forward_ws) + F.dpart);
        part_x_splits = dense_midsplit_splits(T, d_in, d_out, N, r, bf16);   // 0: the products launch's own split count
    }
    const hipError_t e = launch_gate_backward(x, dy, wcat, B, gate_bias, topk_idx, topk_w, labels, beta, T, d_in, d_out,
                                              N, r, k, scale, dW_gate, dbias, d_logits, part_x, part_x_splits, A, W_gate, W_t, dx,
                                              static_cast<char*>(ws),
                                              static_cast<hipStream_t>(stream));
    return e == hipSuccess ? METEORA_OK : METEORA_ERR_HIP;
}

}  // extern "C"
