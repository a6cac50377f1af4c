// bf16 MFMA kernel for the base projection out = x * W^T (first term of Eq. 1 / Eq. 2), with the
// LoRA expand optionally fused as an extension of the contraction:
//
//     out[t, c] = sum_{i < d_in} x[t,i] * W[c,i]  +  sum_{j < ext_k} hd[t,j] * Bst[j,c]
//
// where hd[t, a*r+q] = scale * w * h[t,slot,q] for the adapters a the token selected (zero
// elsewhere) and Bst is the stacked B[N, r, d_out] viewed as [N*r, d_out]; the kernels read it
// transposed (Bt[c, j], rows of ext_stride elements, columns j >= ext_k zero), which makes the
// extension one more stretch of K tiles with the same operand layout as x and W.  The second sum is
// exactly scale * sum_{i in I(x)} w_i (x A_i) B_i of Eq. 2, accumulated in the same fp32
// registers as the base term, so the output is rounded once.
//
// Tiling (gfx950): a workgroup of 4 wavefronts (2x2) owns a BM x BN output tile; each wavefront
// owns (BM/2) x (BN/2) as MI x NI blocks of v_mfma_f32_32x32x16_bf16.  K advances in steps of
// 64 through a double-buffered LDS tile; rows are 128 B and their 16-B chunks are XOR-swizzled
// with the row index (see swz) so that a ds_read_b128 pass touches every bank once.
// The MFMA is issued with W as the first operand, so a lane ends up with 4 consecutive output
// columns of one token row and stores them as one 8-byte word.
#pragma once
#include <type_traits>
#include <utility>

#include "common.hpp"

namespace meteora {

constexpr int kGemmBK = 64;          // K elements per LDS tile
constexpr int kGemmChunks = 8;       // 16-byte chunks per LDS row

// LDS staging of the output tile in the pipelined kernel: a wavefront's (MI*32) x (NI*32) bf16 block,
// rows padded by 16 bytes; the dynamic LDS size is the larger of the operand ring and this stage.
template <int NI>
__host__ __device__ constexpr int gemm_epilogue_stride() { return NI * 64 + 16; }
// fp32 partial tiles (split K) are staged one block row (32 tile rows) per wavefront at a time
template <int NI>
__host__ __device__ constexpr int gemm_partial_stride() { return NI * 128 + 16; }
template <int MI, int NI>
__host__ __device__ constexpr int gemm_lds_bytes() {
    constexpr int ring = 2 * (MI * 64 + NI * 64) * kGemmBK * 2;
    constexpr int stage = 4 * (MI * 32) * gemm_epilogue_stride<NI>();
    constexpr int pstage = 4 * 32 * gemm_partial_stride<NI>();
    constexpr int m = ring > stage ? ring : stage;
    return m > pstage ? m : pstage;
}

struct GemmArgs {
    const bf16_t* x;      // [T, d_in]
    const bf16_t* W;      // [d_out, d_in]
    const bf16_t* hd;     // [T, ext_stride] or nullptr
    const bf16_t* Bt;     // [d_out, ext_stride] (stacked B transposed, zero-padded columns) or nullptr
    bf16_t* out;          // [T, d_out]
    int T, d_in, d_out;
    int ext_k;            // N*r; 0 = no extension
    int ext_stride;       // row stride of hd and Bt: ext_k rounded up to a multiple of 64
    int accumulate;       // 1: add previous contents of out
    int tiles_m, tiles_n;
    // split-K (skinny batches): blockIdx.y = split; split s < splits takes K tiles [s*tiles_per_split, ...),
    // split == splits (only if ext_k > 0) takes the expand extension; fp32 tiles go to partial[split][T][d_out]
    float* partial;       // nullptr: no split, the kernel writes `out` itself
    int splits, tiles_per_split;
    // decode (two-slot split-K kernel only): the column tiles of one launch may belong to several row-major
    // matrices that share x (the base weights of the layers of a group, and for each layer the gate-term rows of
    // its Wcat, so the gate logits ride in the launch that streams W).  Segment e owns column tiles
    // [seg[e].tile0, seg[e+1].tile0) and writes fp32 tiles seg[e].partial[split][T][seg[e].rows].  nseg = 0: off.
    struct Segment {
        const bf16_t* W;   // [rows, d_in]
        float* partial;
        int rows, tile0;
    };
    static constexpr int kMaxSegments = 8;
    Segment seg[kMaxSegments];
    int nseg;
};

// LDS position of 16-byte chunk `chunk` of a 128-byte tile row.  A ds_read_b128 pass serves 16 lanes =
// 16 consecutive rows of one chunk; rows alternate between the two halves of the 64 banks, so rows 2m and
// 2m+1 may share a position and the 8 row pairs need 8 different ones: the pass then touches every bank
// once.  (chunk ^ (row & 7) puts rows m and m+8 on the same banks: a 2-way conflict on every read.)
__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

// Load a [ROWS x 64] bf16 tile (rows row0.., K columns k0..k0+64 of a row-major matrix with
// leading dimension ld) into registers: thread tid handles chunk (tid & 7) of rows (tid>>3) + 32*i.
template <int ROWS>
__device__ __forceinline__ void load_tile_regs(u32x4 (&regs)[ROWS / 32], const bf16_t* __restrict__ base, int ld,
                                               int row0, int nrows, int k0, int kmax, int tid) {
    const int chunk = tid & 7;
    const int kk = k0 + chunk * 8;
#pragma unroll
    for (int i = 0; i < ROWS / 32; ++i) {
        int row = row0 + (tid >> 3) + 32 * i;
        row = row < nrows ? row : nrows - 1;   // clamp: rows past the edge are computed but never stored
        if (kk < kmax)
            regs[i] = *reinterpret_cast<const u32x4*>(base + (size_t)row * ld + kk);
        else
            regs[i] = u32x4{0u, 0u, 0u, 0u};
    }
}

template <int ROWS>
__device__ __forceinline__ void store_tile_lds(const u32x4 (&regs)[ROWS / 32], bf16_t* lds_tile, int tid) {
    const int chunk = tid & 7;
#pragma unroll
    for (int i = 0; i < ROWS / 32; ++i) {
        const int row = (tid >> 3) + 32 * i;
        *reinterpret_cast<u32x4*>(lds_tile + row * kGemmBK + swz(row, chunk) * 8) = regs[i];
    }
}

template <int MI, int NI>
__device__ __forceinline__ void mma_tile(f32x16 (&acc)[MI][NI], const bf16_t* xs, const bf16_t* wsm, int wm, int wn,
                                         int lane) {
    const int lrow = lane & 31, khalf = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < kGemmBK / 16; ++ks) {
        bf16x8 xf[MI], wf[NI];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int row = wm + mi * 32 + lrow;
            xf[mi] = *reinterpret_cast<const bf16x8*>(xs + row * kGemmBK + swz(row, ks * 2 + khalf) * 8);
        }
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int row = wn + ni * 32 + lrow;
            wf[ni] = *reinterpret_cast<const bf16x8*>(wsm + row * kGemmBK + swz(row, ks * 2 + khalf) * 8);
        }
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ni], xf[mi], acc[mi][ni], 0, 0, 0);
    }
}

template <int MI, int NI>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(const GemmArgs a) {
    constexpr int BM = MI * 64, BN = NI * 64;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
    // [2 buffers][x tile BM x 64 | w tile BN x 64]
    constexpr int kBufElems = (BM + BN) * kGemmBK;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * (BN / 2);

    // XCD-aware tile order: consecutive workgroup ids go to different XCDs (8 of them), so give
    // each XCD a contiguous run of tiles, walked along n inside a band of tile rows.
    const int ntiles = a.tiles_m * a.tiles_n;
    int wg = blockIdx.x;
    {
        const int per_xcd = (ntiles + 7) / 8;
        const int xcd = wg % 8, local = wg / 8;
        const int remapped = xcd * per_xcd + local;
        wg = (local < per_xcd && remapped < ntiles && (ntiles % 8 == 0)) ? remapped : wg;
    }
    const int tile_m = wg / a.tiles_n, tile_n = wg % a.tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;

    const int nk_main = ceil_div(a.d_in, kGemmBK);
    const int nk_ext = a.ext_k > 0 ? a.ext_stride / kGemmBK : 0;
    const int nk = nk_main + nk_ext;

    u32x4 xr[BM / 32], wr[BN / 32];

    auto fetch = [&](int it) {   // global -> registers
        if (it < nk_main) {
            load_tile_regs<BM>(xr, a.x, a.d_in, m0, a.T, it * kGemmBK, a.d_in, tid);
            load_tile_regs<BN>(wr, a.W, a.d_in, n0, a.d_out, it * kGemmBK, a.d_in, tid);
        } else {
            load_tile_regs<BM>(xr, a.hd, a.ext_stride, m0, a.T, (it - nk_main) * kGemmBK, a.ext_stride, tid);
            load_tile_regs<BN>(wr, a.Bt, a.ext_stride, n0, a.d_out, (it - nk_main) * kGemmBK, a.ext_stride, tid);
        }
    };
    auto commit = [&](int, int buf) {   // registers -> LDS
        bf16_t* xs = smem + buf * kBufElems;
        store_tile_lds<BM>(xr, xs, tid);
        store_tile_lds<BN>(wr, xs + BM * kGemmBK, tid);
    };

    if (nk > 0) {
        fetch(0);
        commit(0, 0);
    }
    __syncthreads();
    for (int it = 0; it < nk; ++it) {
        const int buf = it & 1;
        if (it + 1 < nk) fetch(it + 1);
        const bf16_t* xs = smem + buf * kBufElems;
        mma_tile<MI, NI>(acc, xs, xs + BM * kGemmBK, wm, wn, lane);
        if (it + 1 < nk) commit(it + 1, buf ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds, per block, 4 groups of 4 consecutive columns of token row (lane & 31)
    const int lrow = lane & 31, khalf = lane >> 5;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int row = m0 + wm + mi * 32 + lrow;
        if (row >= a.T) continue;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col = n0 + wn + ni * 32 + g * 8 + khalf * 4;
                if (col >= a.d_out) continue;   // d_out % 8 == 0, so a group of 4 is all in or all out
                uint2* dst = reinterpret_cast<uint2*>(a.out + (size_t)row * a.d_out + col);
                float v0 = acc[mi][ni][g * 4 + 0], v1 = acc[mi][ni][g * 4 + 1];
                float v2 = acc[mi][ni][g * 4 + 2], v3 = acc[mi][ni][g * 4 + 3];
                if (a.accumulate) {
                    const uint2 old = *dst;
                    v0 += bf16_bits_to_float(old.x & 0xffffu);
                    v1 += bf16_bits_to_float(old.x >> 16);
                    v2 += bf16_bits_to_float(old.y & 0xffffu);
                    v3 += bf16_bits_to_float(old.y >> 16);
                }
                uint2 pk;
                pk.x = pack_bf16x2(v0, v1);
                pk.y = pack_bf16x2(v2, v3);
                *dst = pk;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Pipelined version for d_in % 64 == 0 (all model shapes): the tiles of both operands go from
// global memory straight into LDS with 16-byte buffer_load ... lds (no staging registers), the
// MFMA operand fragments are double-buffered in registers so the ds_reads of k-step s+1 are in
// flight while the MFMAs of k-step s run, and there is one barrier per 64-wide K tile, placed
// before the last k-step: behind it the next tile is visible, the tile after it is requested
// into the slot that has just been drained, and the first fragments of the next tile are read
// under the MFMAs of the last k-step.  The K tiles of the extension (hd x Bt) follow the main
// ones through the same pipeline; only the buffer resources and row strides change.
// ------------------------------------------------------------------------------------------
template <int MI, int NI>
struct Frags {
    bf16x8 x[MI];
    bf16x8 w[NI];
};

template <int MI, int NI>
__device__ __forceinline__ void load_frags(Frags<MI, NI>& f, const bf16_t* xs, const bf16_t* wsm, int wm, int wn,
                                           int lrow, int khalf, int ks) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int row = wm + mi * 32 + lrow;
        f.x[mi] = *reinterpret_cast<const bf16x8*>(xs + row * kGemmBK + swz(row, ks * 2 + khalf) * 8);
    }
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int row = wn + ni * 32 + lrow;
        f.w[ni] = *reinterpret_cast<const bf16x8*>(wsm + row * kGemmBK + swz(row, ks * 2 + khalf) * 8);
    }
}

// One MFMA operand fragment of k-step ks of an LDS tile pair: i < MI -> x block i, else W block i - MI.
template <int MI, int NI>
__device__ __forceinline__ void load_frag1(Frags<MI, NI>& f, const bf16_t* xs, const bf16_t* wsm, int wm, int wn,
                                           int lrow, int khalf, int ks, int i) {
    if (i < MI) {
        const int row = wm + i * 32 + lrow;
        f.x[i] = *reinterpret_cast<const bf16x8*>(xs + row * kGemmBK + swz(row, ks * 2 + khalf) * 8);
    } else {
        const int row = wn + (i - MI) * 32 + lrow;
        f.w[i - MI] = *reinterpret_cast<const bf16x8*>(wsm + row * kGemmBK + swz(row, ks * 2 + khalf) * 8);
    }
}

template <int MI, int NI>
__device__ __forceinline__ void mma_frags(f32x16 (&acc)[MI][NI], const Frags<MI, NI>& f) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.w[ni], f.x[mi], acc[mi][ni], 0, 0, 0);
}

// The first k-step of a tile's contraction: the accumulators start from the MFMA's own zero C operand instead of
// being cleared beforehand (256 register writes per lane in the 256 x 256 kernel, which would sit between the
// arrival of the first tile and the first MFMA).
template <int MI, int NI>
__device__ __forceinline__ void mma_frags_first(f32x16 (&acc)[MI][NI], const Frags<MI, NI>& f) {
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.w[ni], f.x[mi], zero, 0, 0, 0);
}

// A [rows x 64-element-tiles] operand as the global->LDS loads see it.  An instruction moves 8 rows
// (8 lanes x 16 B per 128-byte tile row); lane (rsub, p) fetches the chunk whose swizzled position
// (see swz) is p, so the LDS image is the swizzled layout.  Wavefront `wave` moves rows (j*4 + wave)*8 .. +8 of the tile
// as piece j.  The address is rsrc base + voff (per lane: first row of piece 0, swizzled chunk)
// + a uniform offset (piece and K tile).  The resource covers exactly the matrix, so rows past
// its last one (ragged edge tiles) are out of range for the hardware and load zeros; they only
// feed output rows or columns that are never stored.
struct DmaOperand {
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t voff;        // per lane
    uint32_t piece_step;  // bytes between pieces: 32 rows
};

__device__ __forceinline__ DmaOperand dma_operand(const bf16_t* base, int nrows, int ld, int row0, int wave, int lane) {
    DmaOperand o;
    o.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(base), 0, (uint32_t)nrows * (uint32_t)ld * 2u,
                                               0x00020000);
    // tile row of this lane in piece j: (j*4 + wave)*8 + rsub, so (row >> 1) & 7 = (wave & 1)*4 + (rsub >> 1)
    const int rsub = lane >> 3, p = lane & 7;
    o.voff = (uint32_t)(row0 + wave * 8 + rsub) * (uint32_t)ld * 2u +
             (uint32_t)((p ^ (((wave & 1) << 2) | (rsub >> 1))) << 4);
    o.piece_step = 32u * (uint32_t)ld * 2u;
    return o;
}

__device__ __forceinline__ void dma_piece(bf16_t* lds_tile, const DmaOperand& o, int ktile, int j, int wave) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(
        o.rsrc, (__attribute__((address_space(3))) void*)(lds_tile + (j * 4 + wave) * 8 * kGemmBK), 16, o.voff,
        (int)(o.piece_step * (uint32_t)j + (uint32_t)ktile * (kGemmBK * 2)), 0, 0);
}

// Instruction-order hints for one phase (the code between two sched_barrier(0)): the compiler's own
// order bunches the LDS reads and the global->LDS loads and exposes their issue time and latency;
// these groups alternate them with the MFMAs instead.  Masks: 0x008 MFMA, 0x100 LDS read, 0x020 VMEM read.
#define METEORA_SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)

// Tail of the last phase of a K tile: RM MFMAs with RV global->LDS loads spread evenly between them.
template <int RM, int RV, int J>
__device__ __forceinline__ void paced_tail() {
    if constexpr (J < RM) {
        METEORA_SGB(0x008, 1);
        constexpr int nv = RV / RM + (J < RV % RM ? 1 : 0);
        if constexpr (nv > 0) METEORA_SGB(0x020, nv);
        paced_tail<RM, RV, J + 1>();
    }
}

// Map a workgroup id to an output tile: ids are dealt round-robin to the 8 XCDs, so each XCD
// gets a contiguous run of the tile order, and the order walks groups of 4 tile rows column by
// column: the 32 tiles an XCD works on at a time share few rows of x and W in its L2.
__device__ __forceinline__ void tile_of_workgroup(int wg, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
    const int ntiles = tiles_m * tiles_n;
    int id = wg;
    if (ntiles % 8 == 0) id = (wg % 8) * (ntiles / 8) + wg / 8;
    constexpr int GM = 4;
    const int group = id / (GM * tiles_n);
    const int first_m = group * GM;
    const int gm = min(GM, tiles_m - first_m);
    const int in_group = id - group * GM * tiles_n;
    tile_m = first_m + in_group % gm;
    tile_n = in_group / gm;
}

// Epilogue shared by the pipelined kernels: store a workgroup's accumulators.
// EPI fixes at compile time which of the three forms a kernel carries (kEpiAny: decided at run time).  With one form
// the accumulators leave their registers block row by block row as they are converted; with all three behind
// run-time branches the compiler first copies every accumulator out (and spills) before it branches.
constexpr int kEpiAny = -1, kEpiStore = 0, kEpiAccumulate = 1, kEpiPartial = 2;
template <int MI, int NI, int EPI = kEpiAny>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& a, f32x16 (&acc)[MI][NI], unsigned char* smem_raw, int m0,
                                              int n0, int wm, int wn, int wave, int lane) {
    const int lrow = lane & 31, khalf = lane >> 5;
    const bool is_partial = EPI == kEpiAny ? a.partial != nullptr : EPI == kEpiPartial;
    const bool is_store = EPI == kEpiAny ? (a.partial == nullptr && !a.accumulate) : EPI == kEpiStore;
    // Epilogue.  A lane holds 4 consecutive columns per block row, so direct stores are 8-byte pieces
    // of 32 different rows per instruction; when the output is simply written (no split-K partials,
    // no accumulate) the bf16 tile is staged in this wavefront's own LDS region and stored as
    // 16-byte pieces that cover whole 128-byte lines.
    if (is_store) {
        constexpr int EST = gemm_epilogue_stride<NI>();   // bytes per staged row
        __syncthreads();                                   // every wavefront is done with the operand tiles
        unsigned char* ep = smem_raw + wave * (MI * 32) * EST;
        constexpr int LPR = NI * 4, RPI = 64 / LPR;        // lanes per staged row, rows per store instruction
        const int r_in = lane / LPR, c = (lane % LPR) * 8;
        const int col = n0 + wn + c;
        // one block row (32 tile rows) at a time, so the stores of a block row are under way while the next
        // one is converted; the region is this wavefront's own, and a wavefront's LDS accesses stay in order
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    uint2 pk;
                    pk.x = pack_bf16x2(acc[mi][ni][g * 4 + 0], acc[mi][ni][g * 4 + 1]);
                    pk.y = pack_bf16x2(acc[mi][ni][g * 4 + 2], acc[mi][ni][g * 4 + 3]);
                    *reinterpret_cast<uint2*>(ep + (mi * 32 + lrow) * EST + (ni * 32 + g * 8 + khalf * 4) * 2) = pk;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int i = 0; i < 32 / RPI; ++i) {
                const int r = mi * 32 + i * RPI + r_in;
                const int row = m0 + wm + r;
                const u32x4 v = *reinterpret_cast<const u32x4*>(ep + r * EST + c * 2);
                if (row < a.T && col < a.d_out) *reinterpret_cast<u32x4*>(a.out + (size_t)row * a.d_out + col) = v;
            }
        }
        return;
    }

    if (is_partial) {
        // fp32 split-K tile: same staging, one block row at a time, so the stores are 16-byte pieces of whole rows
        constexpr int PST = gemm_partial_stride<NI>();
        __syncthreads();
        unsigned char* ep = smem_raw + wave * 32 * PST;
        constexpr int PPR = NI * 8;                        // 16-byte pieces per staged row
        float* dst = a.partial + (size_t)blockIdx.y * a.T * a.d_out;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 v = {acc[mi][ni][g * 4 + 0], acc[mi][ni][g * 4 + 1], acc[mi][ni][g * 4 + 2],
                                     acc[mi][ni][g * 4 + 3]};
                    *reinterpret_cast<f32x4*>(ep + lrow * PST + (ni * 32 + g * 8 + khalf * 4) * 4) = v;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int i = 0; i < 32 * PPR / 64; ++i) {
                const int p = i * 64 + lane;
                const int r = p / PPR, c = (p % PPR) * 4;
                const int row = m0 + wm + mi * 32 + r, col = n0 + wn + c;
                const f32x4 v = *reinterpret_cast<const f32x4*>(ep + r * PST + c * 4);
                if (row < a.T && col < a.d_out) *reinterpret_cast<f32x4*>(dst + (size_t)row * a.d_out + col) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        return;
    }

#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int row = m0 + wm + mi * 32 + lrow;
        if (row >= a.T) continue;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col = n0 + wn + ni * 32 + g * 8 + khalf * 4;
                if (col >= a.d_out) continue;
                float v0 = acc[mi][ni][g * 4 + 0], v1 = acc[mi][ni][g * 4 + 1];
                float v2 = acc[mi][ni][g * 4 + 2], v3 = acc[mi][ni][g * 4 + 3];
                uint2* dst = reinterpret_cast<uint2*>(a.out + (size_t)row * a.d_out + col);
                if (a.accumulate) {
                    const uint2 old = *dst;
                    v0 += bf16_bits_to_float(old.x & 0xffffu);
                    v1 += bf16_bits_to_float(old.x >> 16);
                    v2 += bf16_bits_to_float(old.y & 0xffffu);
                    v3 += bf16_bits_to_float(old.y >> 16);
                }
                uint2 pk;
                pk.x = pack_bf16x2(v0, v1);
                pk.y = pack_bf16x2(v2, v3);
                *dst = pk;
            }
        }
    }
}

template <int MI, int NI>
__global__ __launch_bounds__(256) void gemm_mfma_dma_kernel(const GemmArgs a_in) {
    GemmArgs a = a_in;
    constexpr int BM = MI * 64, BN = NI * 64;
    constexpr int PX = BM / 32, PW = BN / 32;   // pieces per wavefront per tile
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
    constexpr int kBufElems = (BM + BN) * kGemmBK;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps LDS bases in SGPRs
    const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * (BN / 2);
    const int lrow = lane & 31, khalf = lane >> 5;
    int tile_m, tile_n;
    tile_of_workgroup(blockIdx.x, a.tiles_m, a.tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM;
    int n0 = tile_n * BN;
    if (a.nseg > 0) {   // uniform: the tile is an ordinary tile of its segment's matrix
        int e = 0;
        for (int i = 1; i < a.nseg; ++i)
            if (tile_n >= a_in.seg[i].tile0) e = i;
        n0 = (tile_n - a_in.seg[e].tile0) * BN;
        a.W = a_in.seg[e].W;
        a.d_out = a_in.seg[e].rows;
        a.partial = a_in.seg[e].partial;
    }

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;

    // this workgroup's share of the contraction: main K tiles [kt0, kt0 + nk_main) and/or the extension
    int kt0 = 0, nk_main = a.d_in / kGemmBK;
    int nk_ext = a.ext_k > 0 ? a.ext_stride / kGemmBK : 0;
    if (a.partial != nullptr) {
        const int split = blockIdx.y;
        if (split < a.splits) {
            kt0 = split * a.tiles_per_split;
            nk_main = max(0, min(a.tiles_per_split, nk_main - kt0));
            nk_ext = 0;
        } else {
            nk_main = 0;
        }
    }
    const int nk = nk_main + nk_ext;

    // (x, W) feed local tiles [0, nk_main), (hd, Bt) the tiles after them
    const DmaOperand ox = dma_operand(a.x, a.T, a.d_in, m0, wave, lane);
    const DmaOperand ow = dma_operand(a.W, a.d_out, a.d_in, n0, wave, lane);
    const DmaOperand oh = dma_operand(a.hd, nk_ext > 0 ? a.T : 0, a.ext_stride, m0, wave, lane);
    const DmaOperand ob = dma_operand(a.Bt, nk_ext > 0 ? a.d_out : 0, a.ext_stride, n0, wave, lane);

    // piece i of local tile `it` (x-like pieces first) into LDS slot `slot`
    auto request_piece = [&](int it, int slot, int i, auto is_ext) {
        bf16_t* xs = smem + slot * kBufElems;
        if constexpr (decltype(is_ext)::value) {
            if (i < PX) dma_piece(xs, oh, it - nk_main, i, wave);
            else dma_piece(xs + BM * kGemmBK, ob, it - nk_main, i - PX, wave);
        } else {
            if (i < PX) dma_piece(xs, ox, kt0 + it, i, wave);
            else dma_piece(xs + BM * kGemmBK, ow, kt0 + it, i - PX, wave);
        }
    };
    auto request_tile = [&](int it, int slot) {
#pragma unroll
        for (int i = 0; i < PX + PW; ++i) {
            if (it < nk_main) request_piece(it, slot, i, std::false_type{});
            else request_piece(it, slot, i, std::true_type{});
        }
    };

    Frags<MI, NI> f0, f1;
    if (nk > 1) {
        // both slots are free: request the first two tiles together, wait for the older one only
        request_tile(0, 0);
        request_tile(1, 1);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PX + PW) : "memory");
        __syncthreads();
        load_frags<MI, NI>(f0, smem, smem + BM * kGemmBK, wm, wn, lrow, khalf, 0);
    } else if (nk > 0) {
        request_tile(0, 0);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        load_frags<MI, NI>(f0, smem, smem + BM * kGemmBK, wm, wn, lrow, khalf, 0);
    }
    // One K tile = 4 phases of (MI*NI MFMA + the fragment reads of the next k-step); sched_barrier keeps
    // each phase's reads from sinking into the next phase, where they would be waited on at once.
    // In the 256x256 kernel the reads are issued one per MFMA in the first half of the phase, so each
    // has at least half a phase of MFMAs to land under.
    constexpr bool kPaced = (MI == 4 && NI == 4);   // measured: no gain from the hints on the smaller tiles
    static_assert(!kPaced || MI * NI >= MI + NI, "a phase needs one MFMA per fragment read");
    auto phase = [&](Frags<MI, NI>& fnext, const Frags<MI, NI>& fcur, const bf16_t* xs, int ks) {
        load_frags<MI, NI>(fnext, xs, xs + BM * kGemmBK, wm, wn, lrow, khalf, ks);
        mma_frags<MI, NI>(acc, fcur);
        if constexpr (kPaced) {
#pragma unroll
            for (int i = 0; i < MI + NI; ++i) { METEORA_SGB(0x008, 1); METEORA_SGB(0x100, 1); }
            METEORA_SGB(0x008, MI * NI - (MI + NI));
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // REQ: 0 = tile it+2 is a main tile, 1 = it is an extension tile, 2 = there is none (last two tiles)
    auto tile_step = [&](int it, auto req) {
        constexpr int REQ = decltype(req)::value;
        const bf16_t* xs = smem + (it & 1) * kBufElems;
        phase(f1, f0, xs, 1);
        phase(f0, f1, xs, 2);
        phase(f1, f0, xs, 3);
        // tile it+1 (requested one tile ago) must have landed; every wavefront has read tile it
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        const bf16_t* xn = smem + ((it + 1) & 1) * kBufElems;
        if constexpr (REQ < 2) {
            // Program order = the order the LDS accesses must keep (the compiler does not move an LDS
            // read across a global->LDS load): the first fragments of tile it+1 with pieces of tile
            // it+2 between them, then the remaining pieces; tile it+2 goes into the slot just drained.
            constexpr int NR = MI + NI, NPC = PX + PW;
#pragma unroll
            for (int i = 0; i < NR; ++i) {
                load_frag1<MI, NI>(f0, xn, xn + BM * kGemmBK, wm, wn, lrow, khalf, 0, i);
                request_piece(it + 2, it & 1, i, std::integral_constant<bool, REQ == 1>{});
            }
#pragma unroll
            for (int i = NR; i < NPC; ++i) request_piece(it + 2, it & 1, i, std::integral_constant<bool, REQ == 1>{});
            mma_frags<MI, NI>(acc, f1);
            if constexpr (kPaced) {
#pragma unroll
                for (int i = 0; i < NR; ++i) { METEORA_SGB(0x008, 1); METEORA_SGB(0x100, 1); METEORA_SGB(0x020, 1); }
                // the remaining pieces spread evenly over the remaining MFMAs
                constexpr int RM = MI * NI - NR, RV = NPC - NR;
                if constexpr (RM > 0) {
                    paced_tail<RM, RV, 0>();
                } else if constexpr (RV > 0) {
                    METEORA_SGB(0x020, RV);
                }
            }
        } else {
            if (it + 1 < nk) load_frags<MI, NI>(f0, xn, xn + BM * kGemmBK, wm, wn, lrow, khalf, 0);
            mma_frags<MI, NI>(acc, f1);
            if constexpr (kPaced) {
#pragma unroll
                for (int i = 0; i < MI + NI; ++i) { METEORA_SGB(0x008, 1); METEORA_SGB(0x100, 1); }
                METEORA_SGB(0x008, MI * NI - (MI + NI));
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    int it = 0;
    for (; it + 2 < nk_main; ++it) tile_step(it, std::integral_constant<int, 0>{});
    for (; it + 2 < nk; ++it) tile_step(it, std::integral_constant<int, 1>{});
    for (; it < nk; ++it) tile_step(it, std::integral_constant<int, 2>{});

    gemm_epilogue<MI, NI>(a, acc, smem_raw, m0, n0, wm, wn, wave, lane);
}

// ------------------------------------------------------------------------------------------
// The same pipeline with a three-deep ring for the W operand (2 x-slots + 3 W-slots: the whole 160 KB of
// LDS for the 256 x 256 tile).  A global->LDS load occupies the CU's address unit for ~16 cycles, so the
// four wavefronts can sustain one load per two MFMAs each; issued as one per MFMA (all pieces of a tile in
// the last phase, the only time a two-slot ring has a free slot) they stall the MFMAs queued behind them.
// Here tile it+2's W pieces go out during the first three phases of tile it, into the W-slot that no
// wavefront has read since the previous barrier, and only its x pieces wait for the barrier, spread over
// the MFMAs of the last phase.  Loads complete in order, so the barrier of tile it waits for everything
// but the newest W pieces (vmcnt = W pieces per wavefront).
// ------------------------------------------------------------------------------------------
template <int MI, int NI>
__host__ __device__ constexpr int gemm_w3_lds_bytes() {
    constexpr int ring = (2 * MI * 64 + 3 * NI * 64) * kGemmBK * 2;
    constexpr int stage = 4 * (MI * 32) * gemm_epilogue_stride<NI>();
    constexpr int pstage = 4 * 32 * gemm_partial_stride<NI>();
    constexpr int m = ring > stage ? ring : stage;
    return m > pstage ? m : pstage;
}

// how many of NPC pieces go out right after the i-th of NR fragment reads (evenly spread, the last read included)
__host__ __device__ constexpr int pieces_after_read(int i, int NPC, int NR) {
    return (i + 1) * NPC / NR - i * NPC / NR;
}

template <int N>
__device__ __forceinline__ void sgb_vmem() {
    if constexpr (N > 0) METEORA_SGB(0x020, N);
}
template <int N>
__device__ __forceinline__ void sgb_mfma() {
    if constexpr (N > 0) METEORA_SGB(0x008, N);
}

// Order of one phase: per fragment read, one MFMA, the read, MPR-1 more MFMAs, then the read's share of NPC loads.
template <int MPR, int NPC, int NR, int... I>
__device__ __forceinline__ void sgb_reads(std::integer_sequence<int, I...>) {
    ((METEORA_SGB(0x008, 1), METEORA_SGB(0x100, 1), sgb_mfma<MPR - 1>(), sgb_vmem<pieces_after_read(I, NPC, NR)>()), ...);
}

template <int MI, int NI, int EPI = kEpiAny>
__global__ __launch_bounds__(256) void gemm_mfma_w3_kernel(const GemmArgs a_in) {
    GemmArgs a = a_in;
    constexpr int BM = MI * 64, BN = NI * 64;
    constexpr int PX = BM / 32, PW = BN / 32;   // pieces per wavefront per tile
    constexpr int NR = MI + NI;                 // fragment reads per k-step
    static_assert(MI * NI >= NR, "a phase needs one MFMA per fragment read");
    constexpr int PW1 = (PW + 2) / 3, PW2 = (PW - PW1 + 1) / 2, PW3 = PW - PW1 - PW2;   // W pieces per phase
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
    constexpr int kXElems = BM * kGemmBK, kWElems = BN * kGemmBK;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * (BN / 2);
    const int lrow = lane & 31, khalf = lane >> 5;
    int tile_m, tile_n;
    tile_of_workgroup(blockIdx.x, a.tiles_m, a.tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM;
    int n0 = tile_n * BN;
    if (a.nseg > 0) {   // uniform: the tile is an ordinary tile of its segment's matrix (split-K launches only)
        int e = 0;
        for (int i = 1; i < a.nseg; ++i)
            if (tile_n >= a_in.seg[i].tile0) e = i;
        n0 = (tile_n - a_in.seg[e].tile0) * BN;
        a.W = a_in.seg[e].W;
        a.d_out = a_in.seg[e].rows;
        a.partial = a_in.seg[e].partial;
    }

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;

    // this workgroup's share of the contraction: main K tiles [kt0, kt0 + nk_main) and/or the extension
    int kt0 = 0, nk_main = a.d_in / kGemmBK;
    int nk_ext = a.ext_k > 0 ? a.ext_stride / kGemmBK : 0;
    if (a.partial != nullptr) {
        const int split = blockIdx.y;
        if (split < a.splits) {
            kt0 = split * a.tiles_per_split;
            nk_main = max(0, min(a.tiles_per_split, nk_main - kt0));
            nk_ext = 0;
        } else {
            nk_main = 0;
        }
    }
    const int nk = nk_main + nk_ext;

    const DmaOperand ox = dma_operand(a.x, a.T, a.d_in, m0, wave, lane);
    const DmaOperand ow = dma_operand(a.W, a.d_out, a.d_in, n0, wave, lane);
    const DmaOperand oh = dma_operand(a.hd, nk_ext > 0 ? a.T : 0, a.ext_stride, m0, wave, lane);
    const DmaOperand ob = dma_operand(a.Bt, nk_ext > 0 ? a.d_out : 0, a.ext_stride, n0, wave, lane);

    auto xslot = [&](int it) { return smem + (it & 1) * kXElems; };
    auto wslot = [&](int it) { return smem + 2 * kXElems + (it % 3) * kWElems; };
    // piece i of the x-like / W-like operand of local tile `it` (main tiles first, then the extension)
    auto request_x = [&](bf16_t* slot, int it, int i, auto is_ext) {
        if constexpr (decltype(is_ext)::value) dma_piece(slot, oh, it - nk_main, i, wave);
        else dma_piece(slot, ox, kt0 + it, i, wave);
    };
    auto request_w = [&](bf16_t* slot, int it, int i, auto is_ext) {
        if constexpr (decltype(is_ext)::value) dma_piece(slot, ob, it - nk_main, i, wave);
        else dma_piece(slot, ow, kt0 + it, i, wave);
    };
    auto request_tile = [&](int it) {
        if (it < nk_main) {
#pragma unroll
            for (int i = 0; i < PX; ++i) request_x(xslot(it), it, i, std::false_type{});
#pragma unroll
            for (int i = 0; i < PW; ++i) request_w(wslot(it), it, i, std::false_type{});
        } else {
#pragma unroll
            for (int i = 0; i < PX; ++i) request_x(xslot(it), it, i, std::true_type{});
#pragma unroll
            for (int i = 0; i < PW; ++i) request_w(wslot(it), it, i, std::true_type{});
        }
    };

    Frags<MI, NI> f0, f1;
    if (nk > 1) {
        request_tile(0);
        request_tile(1);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PX + PW) : "memory");
        __syncthreads();
        load_frags<MI, NI>(f0, xslot(0), wslot(0), wm, wn, lrow, khalf, 0);
    } else if (nk > 0) {
        request_tile(0);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        load_frags<MI, NI>(f0, xslot(0), wslot(0), wm, wn, lrow, khalf, 0);
    }

    // REQ: 0 = tile it+2 is a main tile, 1 = it is an extension tile, 2 = there is none (last two tiles)
    // PH: it % 6 when it is known at compile time (the unrolled main loop: every slot address is then a
    // constant and no address arithmetic sits between two tiles), -1 otherwise
    // first: the tile's first k-step starts the accumulators (tile 0 of the unrolled form)
    auto tile_step = [&](int it, auto req, auto ph, auto first) {
        constexpr int REQ = decltype(req)::value, PH = decltype(ph)::value;
        constexpr bool FIRST = decltype(first)::value;
        using IsExt = std::integral_constant<bool, REQ == 1>;
        auto xsl = [&](int d) {   // x-slot / W-slot of tile it + d
            if constexpr (PH >= 0) return smem + ((PH + d) & 1) * kXElems;
            else return xslot(it + d);
        };
        auto wsl = [&](int d) {
            if constexpr (PH >= 0) return smem + 2 * kXElems + ((PH + d) % 3) * kWElems;
            else return wslot(it + d);
        };
        const bf16_t* xs = xsl(0);
        const bf16_t* ws = wsl(0);
        bf16_t* const xreq = xsl(2);
        bf16_t* const wreq = wsl(2);
        // phases 1-3: MI*NI MFMAs of k-step ks-1, the fragment reads of k-step ks one per MFMA from the start of
        // the phase, and W pieces [P0, P0 + NPC) of tile it+2 spread between the reads (program order = the
        // order the LDS accesses keep)
        auto phase = [&](Frags<MI, NI>& fnext, const Frags<MI, NI>& fcur, int ks, auto p0, auto npc, auto start) {
            constexpr int P0 = decltype(p0)::value, NPC = REQ < 2 ? decltype(npc)::value : 0;
            int issued = 0;
#pragma unroll
            for (int i = 0; i < NR; ++i) {
                load_frag1<MI, NI>(fnext, xs, ws, wm, wn, lrow, khalf, ks, i);
                if constexpr (NPC > 0) {
#pragma unroll
                    for (int c = 0; c < pieces_after_read(i, NPC, NR); ++c) request_w(wreq, it + 2, P0 + issued++, IsExt{});
                }
            }
            if constexpr (decltype(start)::value) mma_frags_first<MI, NI>(acc, fcur);
            else mma_frags<MI, NI>(acc, fcur);
            sgb_reads<1, NPC, NR>(std::make_integer_sequence<int, NR>{});
            sgb_mfma<MI * NI - NR>();
            __builtin_amdgcn_sched_barrier(0);
        };
        phase(f1, f0, 1, std::integral_constant<int, 0>{}, std::integral_constant<int, PW1>{}, std::bool_constant<FIRST>{});
        phase(f0, f1, 2, std::integral_constant<int, PW1>{}, std::integral_constant<int, PW2>{}, std::false_type{});
        phase(f1, f0, 3, std::integral_constant<int, PW1 + PW2>{}, std::integral_constant<int, PW3>{}, std::false_type{});
        // tile it+1 (x requested one tile ago, W before that) must have landed, and every wavefront's reads of
        // tile it must be complete; the W pieces of tile it+2 just issued may still be in flight
        // (a plain s_barrier: __syncthreads() carries a fence, for which the compiler waits for every load)
        if constexpr (REQ < 2) {
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(PW) : "memory");
        } else {
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
        }
        const bf16_t* xn = xsl(1);
        const bf16_t* wnx = wsl(1);
        if constexpr (REQ < 2) {
            // first fragments of tile it+1, and the x pieces of tile it+2 into the x-slot just drained, spread
            // over the phase: MPR MFMAs per read, a read's pieces after them
            constexpr int MPR = MI * NI / NR;
            int issued = 0;
            // read order: the next phase's first MFMAs use x block 0 with every W block, then x blocks 1..
#pragma unroll
            for (int i = 0; i < NR; ++i) {
                const int fi = i == 0 ? 0 : (i <= NI ? MI + i - 1 : i - NI);
                load_frag1<MI, NI>(f0, xn, wnx, wm, wn, lrow, khalf, 0, fi);
#pragma unroll
                for (int c = 0; c < pieces_after_read(i, PX, NR); ++c) request_x(xreq, it + 2, issued++, IsExt{});
            }
            mma_frags<MI, NI>(acc, f1);
            sgb_reads<MPR, PX, NR>(std::make_integer_sequence<int, NR>{});
            sgb_mfma<MI * NI - NR * MPR>();
        } else {
            if (it + 1 < nk) load_frags<MI, NI>(f0, xn, wnx, wm, wn, lrow, khalf, 0);
            mma_frags<MI, NI>(acc, f1);
            sgb_reads<1, 0, NR>(std::make_integer_sequence<int, NR>{});
            sgb_mfma<MI * NI - NR>();
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    using Req0 = std::integral_constant<int, 0>;
    using Rt = std::integral_constant<int, -1>;
    using No = std::false_type;
    // the last extension tile may hold data in its first two k-steps only (28 adapters of rank 8: 224 of 256 columns;
    // the rest is zero padding): those two k-steps are all it gets
    const bool half_last = nk_ext > 0 && ((a.ext_k - 1) % kGemmBK) < kGemmBK / 2;
    // A wavefront whose whole piece of the tile lies past the matrix (ragged last tile row or column: the third
    // 128-column tile of the 320 routing products is half empty) moves its share of the operand tiles and keeps the
    // barriers, one per K tile like the others, and skips the fragment reads and the MFMAs.
    const bool idle = n0 + wn >= a.d_out || m0 + wm >= a.T;   // uniform per wavefront
    int it = 0;
    if (idle) {
        for (; it < nk - (half_last ? 1 : 0); ++it) {
            if (it + 2 < nk) {
                const bool ext = it + 2 >= nk_main;
#pragma unroll
                for (int i = 0; i < PW; ++i) {
                    if (ext) request_w(wslot(it + 2), it + 2, i, std::true_type{});
                    else request_w(wslot(it + 2), it + 2, i, std::false_type{});
                }
                asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(PW) : "memory");
#pragma unroll
                for (int i = 0; i < PX; ++i) {
                    if (ext) request_x(xslot(it + 2), it + 2, i, std::true_type{});
                    else request_x(xslot(it + 2), it + 2, i, std::false_type{});
                }
            } else {
                __builtin_amdgcn_s_waitcnt(0);
                __syncthreads();
            }
        }
        it = nk;
    }
    if constexpr (MI == 4 && NI == 4) {   // six tiles per trip: the period of the 2-slot and 3-slot rings
        if (nk_main > 8 && !idle) {
            // tile 0 on its own: its first k-step starts the accumulators; the trips then begin at tile 1
            tile_step(0, Req0{}, std::integral_constant<int, 0>{}, std::true_type{});
            for (it = 1; it + 7 < nk_main; it += 6) {
                tile_step(it, Req0{}, std::integral_constant<int, 1>{}, No{});
                tile_step(it + 1, Req0{}, std::integral_constant<int, 2>{}, No{});
                tile_step(it + 2, Req0{}, std::integral_constant<int, 3>{}, No{});
                tile_step(it + 3, Req0{}, std::integral_constant<int, 4>{}, No{});
                tile_step(it + 4, Req0{}, std::integral_constant<int, 5>{}, No{});
                tile_step(it + 5, Req0{}, std::integral_constant<int, 0>{}, No{});
            }
        }
    }
    for (; it + 2 < nk_main; ++it) tile_step(it, Req0{}, Rt{}, No{});
    for (; it + 2 < nk; ++it) tile_step(it, std::integral_constant<int, 1>{}, Rt{}, No{});
    for (; it < nk - (half_last ? 1 : 0); ++it) tile_step(it, std::integral_constant<int, 2>{}, Rt{}, No{});
    if (half_last && !idle) {   // uniform; its first fragments were read, behind the barrier, in the previous step's last phase
        load_frags<MI, NI>(f1, xslot(it), wslot(it), wm, wn, lrow, khalf, 1);
        mma_frags<MI, NI>(acc, f0);
        mma_frags<MI, NI>(acc, f1);
    }

    gemm_epilogue<MI, NI, EPI>(a, acc, smem_raw, m0, n0, wm, wn, wave, lane);
}

}  // namespace meteora
