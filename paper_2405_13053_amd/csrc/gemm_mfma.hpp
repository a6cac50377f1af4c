// bf16 MFMA kernel for the base projection out = x * W^T (first term of Eq. 1 / Eq. 2), with the
// LoRA expand optionally fused as an extension of the contraction:
//
//     out[t, c] = sum_{i < d_in} x[t,i] * W[c,i]  +  sum_{j < ext_k} hd[t,j] * Bst[j,c]
//
// where hd[t, a*r+q] = scale * w * h[t,slot,q] for the adapters a the token selected (zero
// elsewhere) and Bst is the stacked B[N, r, d_out] viewed as [N*r, d_out].  The second sum is
// exactly scale * sum_{i in I(x)} w_i (x A_i) B_i of Eq. 2, accumulated in the same fp32
// registers as the base term, so the output is rounded once.
//
// Tiling (gfx950): a workgroup of 4 wavefronts (2x2) owns a BM x BN output tile; each wavefront
// owns (BM/2) x (BN/2) as MI x NI blocks of v_mfma_f32_32x32x16_bf16.  K advances in steps of
// 64 through a double-buffered LDS tile; rows are 128 B and their 16-B chunks are XOR-swizzled
// with the row index so that ds_read_b128 of 8 consecutive rows touches all banks once.
// The MFMA is issued with W as the first operand, so a lane ends up with 4 consecutive output
// columns of one token row and stores them as one 8-byte word.
#pragma once
#include <type_traits>

#include "common.hpp"

namespace meteora {

constexpr int kGemmBK = 64;          // K elements per LDS tile
constexpr int kGemmChunks = 8;       // 16-byte chunks per LDS row

struct GemmArgs {
    const bf16_t* x;      // [T, d_in]
    const bf16_t* W;      // [d_out, d_in]
    const bf16_t* hd;     // [T, ext_stride] or nullptr
    const bf16_t* Bst;    // [ext_k, d_out]  or nullptr
    bf16_t* out;          // [T, d_out]
    int T, d_in, d_out;
    int ext_k;            // N*r (rows of Bst); 0 = no extension
    int ext_stride;       // row stride of hd (multiple of 8, >= ext_k)
    int accumulate;       // 1: add previous contents of out
    int tiles_m, tiles_n;
    // split-K (skinny batches): blockIdx.y = split; split s < splits takes K tiles [s*tiles_per_split, ...),
    // split == splits (only if ext_k > 0) takes the expand extension; fp32 tiles go to partial[split][T][d_out]
    float* partial;       // nullptr: no split, the kernel writes `out` itself
    int splits, tiles_per_split;
};

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ (row & 7); }

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

// Transposing load of the stacked-B tile: LDS wants [n][k] (k contiguous); memory is [k][n].
// Thread handles column n = n0 + (tid) (+256*i) ... here BN <= 256 so one column per thread and
// all 8 chunks of it; each chunk gathers 8 k-rows with 2-byte loads that are coalesced across lanes.
template <int BN>
__device__ __forceinline__ void load_bst_tile_lds(bf16_t* lds_tile, const bf16_t* __restrict__ Bst, int d_out,
                                                  int n0, int k0, int ext_k, int tid) {
    for (int n = tid; n < BN; n += 256) {
        int col = n0 + n;
        col = col < d_out ? col : d_out - 1;
#pragma unroll
        for (int c = 0; c < kGemmChunks; ++c) {
            union { uint16_t h[8]; u32x4 v; } p;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int kk = k0 + c * 8 + j;
                p.h[j] = kk < ext_k ? reinterpret_cast<const uint16_t*>(Bst)[(size_t)kk * d_out + col] : (uint16_t)0;
            }
            *reinterpret_cast<u32x4*>(lds_tile + n * kGemmBK + swz(n, c) * 8) = p.v;
        }
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
    const int nk_ext = a.ext_k > 0 ? ceil_div(a.ext_k, kGemmBK) : 0;
    const int nk = nk_main + nk_ext;

    u32x4 xr[BM / 32], wr[BN / 32];

    auto fetch = [&](int it) {   // global -> registers (x-like operand and, for the main part, W)
        if (it < nk_main) {
            load_tile_regs<BM>(xr, a.x, a.d_in, m0, a.T, it * kGemmBK, a.d_in, tid);
            load_tile_regs<BN>(wr, a.W, a.d_in, n0, a.d_out, it * kGemmBK, a.d_in, tid);
        } else {
            load_tile_regs<BM>(xr, a.hd, a.ext_stride, m0, a.T, (it - nk_main) * kGemmBK, a.ext_k, tid);
        }
    };
    auto commit = [&](int it, int buf) {   // registers -> LDS (and the transposed stacked-B tile)
        bf16_t* xs = smem + buf * kBufElems;
        bf16_t* wsm = xs + BM * kGemmBK;
        store_tile_lds<BM>(xr, xs, tid);
        if (it < nk_main)
            store_tile_lds<BN>(wr, wsm, tid);
        else
            load_bst_tile_lds<BN>(wsm, a.Bst, a.d_out, n0, (it - nk_main) * kGemmBK, a.ext_k, tid);
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
// Pipelined version for d_in % 64 == 0 (all model shapes): the tiles of x and W go from global
// memory straight into LDS with 16-byte global->LDS loads (no staging registers), the MFMA
// operand fragments are double-buffered in registers so the ds_reads of k-step s+1 are in
// flight while the MFMAs of k-step s run, and there is one barrier per 64-wide K tile, placed
// before the last k-step: behind it the next tile is visible, the tile after it is requested
// into the slot that has just been drained, and the first fragments of the next tile are read
// under the MFMAs of the last k-step.
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

template <int MI, int NI>
__device__ __forceinline__ void mma_frags(f32x16 (&acc)[MI][NI], const Frags<MI, NI>& f) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.w[ni], f.x[mi], acc[mi][ni], 0, 0, 0);
}

// One [ROWS x 64] tile, global -> LDS: an instruction moves 8 rows (8 lanes x 16 B per 128-B row);
// lane (row, p) fetches global chunk p ^ (row & 7) so the LDS image is the swizzled layout.
template <int ROWS>
__device__ __forceinline__ void dma_tile(bf16_t* lds_tile, const bf16_t* __restrict__ base, int ld, int row0,
                                         int nrows, int k0, int wave, int lane) {
    const int rsub = lane >> 3, p = lane & 7;
#pragma unroll
    for (int j = 0; j < ROWS / 32; ++j) {   // 4 waves x 8 rows per instruction
        const int row = (j * 4 + wave) * 8 + rsub;
        int grow = row0 + row;
        grow = grow < nrows ? grow : nrows - 1;
        const bf16_t* src = base + (size_t)grow * ld + k0 + ((p ^ (row & 7)) << 3);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)(lds_tile + (j * 4 + wave) * 8 * kGemmBK),
                                         16, 0, 0);
    }
}

// Steady-state form of dma_tile: the per-lane byte offsets are computed once (dma_offsets) and each
// K tile only adds a uniform base, so the loop carries no per-load address arithmetic.
template <int ROWS>
__device__ __forceinline__ void dma_offsets(uint32_t (&voff)[ROWS / 32], int ld, int row0, int nrows, int wave,
                                            int lane) {
    const int rsub = lane >> 3, p = lane & 7;
#pragma unroll
    for (int j = 0; j < ROWS / 32; ++j) {
        const int row = (j * 4 + wave) * 8 + rsub;
        int grow = row0 + row;
        grow = grow < nrows ? grow : nrows - 1;
        voff[j] = (uint32_t)grow * (uint32_t)ld * 2u + (uint32_t)((p ^ (row & 7)) << 4);
    }
}

template <int ROWS>
__device__ __forceinline__ void dma_issue(bf16_t* lds_tile, const char* base_k, const uint32_t (&voff)[ROWS / 32],
                                          int wave) {
#pragma unroll
    for (int j = 0; j < ROWS / 32; ++j) {
        const char* src = base_k + voff[j];
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)(lds_tile + (j * 4 + wave) * 8 * kGemmBK),
                                         16, 0, 0);
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

template <int MI, int NI>
__global__ __launch_bounds__(256) void gemm_mfma_dma_kernel(const GemmArgs a) {
    constexpr int BM = MI * 64, BN = NI * 64;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
    constexpr int kBufElems = (BM + BN) * kGemmBK;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps LDS bases in SGPRs
    const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * (BN / 2);
    const int lrow = lane & 31, khalf = lane >> 5;
    int tile_m, tile_n;
    tile_of_workgroup(blockIdx.x, a.tiles_m, a.tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;

    // this workgroup's share of the contraction: main K tiles [kt0, kt0 + nk_main) and/or the extension
    int kt0 = 0, nk_main = a.d_in / kGemmBK;
    int nk_ext = a.ext_k > 0 ? ceil_div(a.ext_k, kGemmBK) : 0;
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

    auto request = [&](int it, int slot) {   // start moving local K tile `it` into LDS slot `slot`
        bf16_t* xs = smem + slot * kBufElems;
        bf16_t* wsm = xs + BM * kGemmBK;
        if (it < nk_main) {
            dma_tile<BM>(xs, a.x, a.d_in, m0, a.T, (kt0 + it) * kGemmBK, wave, lane);
            dma_tile<BN>(wsm, a.W, a.d_in, n0, a.d_out, (kt0 + it) * kGemmBK, wave, lane);
        } else {
            dma_tile<BM>(xs, a.hd, a.ext_stride, m0, a.T, (it - nk_main) * kGemmBK, wave, lane);
            load_bst_tile_lds<BN>(wsm, a.Bst, a.d_out, n0, (it - nk_main) * kGemmBK, a.ext_k, tid);
        }
    };

    // steady state: byte offsets of this lane's 16-byte pieces inside a K tile, fixed for the whole loop
    uint32_t xoff[BM / 32], woff[BN / 32];
    dma_offsets<BM>(xoff, a.d_in, m0, a.T, wave, lane);
    dma_offsets<BN>(woff, a.d_in, n0, a.d_out, wave, lane);
    const char* xb = reinterpret_cast<const char*>(a.x) + (size_t)kt0 * (kGemmBK * 2);
    const char* wb = reinterpret_cast<const char*>(a.W) + (size_t)kt0 * (kGemmBK * 2);
    auto request_main = [&](int it, int slot) {
        bf16_t* xs = smem + slot * kBufElems;
        dma_issue<BM>(xs, xb + (size_t)it * (kGemmBK * 2), xoff, wave);
        dma_issue<BN>(xs + BM * kGemmBK, wb + (size_t)it * (kGemmBK * 2), woff, wave);
    };

    Frags<MI, NI> f0, f1;
    if (nk > 0) {
        request(0, 0);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (nk > 1) request(1, 1);
        load_frags<MI, NI>(f0, smem, smem + BM * kGemmBK, wm, wn, lrow, khalf, 0);
    }
    // One K tile = 4 phases of (16 MFMA + the fragment reads of the next k-step); sched_barrier keeps
    // each phase's reads from sinking into the next phase, where they would be waited on at once.
    auto tile_step = [&](int it, auto steady) {
        const bf16_t* xs = smem + (it & 1) * kBufElems;
        const bf16_t* wsm = xs + BM * kGemmBK;
        load_frags<MI, NI>(f1, xs, wsm, wm, wn, lrow, khalf, 1);
        mma_frags<MI, NI>(acc, f0);
        __builtin_amdgcn_sched_barrier(0);
        load_frags<MI, NI>(f0, xs, wsm, wm, wn, lrow, khalf, 2);
        mma_frags<MI, NI>(acc, f1);
        __builtin_amdgcn_sched_barrier(0);
        load_frags<MI, NI>(f1, xs, wsm, wm, wn, lrow, khalf, 3);
        mma_frags<MI, NI>(acc, f0);
        __builtin_amdgcn_sched_barrier(0);
        // tile it+1 (requested one tile ago) must have landed; every wavefront has read tile it
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        const bf16_t* xn = smem + ((it + 1) & 1) * kBufElems;
        if constexpr (decltype(steady)::value) {
            request_main(it + 2, it & 1);
            load_frags<MI, NI>(f0, xn, xn + BM * kGemmBK, wm, wn, lrow, khalf, 0);
        } else {
            if (it + 2 < nk) request(it + 2, it & 1);
            if (it + 1 < nk) load_frags<MI, NI>(f0, xn, xn + BM * kGemmBK, wm, wn, lrow, khalf, 0);
        }
        mma_frags<MI, NI>(acc, f1);
        __builtin_amdgcn_sched_barrier(0);
    };
    int it = 0;
    for (; it + 2 < nk_main; ++it) tile_step(it, std::true_type{});   // branch-free body
    for (; it < nk; ++it) tile_step(it, std::false_type{});            // last tiles and the expand extension

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
                if (a.partial != nullptr) {
                    const f32x4 v = {v0, v1, v2, v3};
                    *reinterpret_cast<f32x4*>(a.partial + ((size_t)blockIdx.y * a.T + row) * a.d_out + col) = v;
                    continue;
                }
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

}  // namespace meteora
