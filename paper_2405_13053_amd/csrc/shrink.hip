// Grouped LoRA shrink (first product of Eq. 2):  h[t,slot,:] = x[t,:] * A_a,  a = I(t)_slot.
//
// Work is grouped by adapter through the bucket lists: a tile is a run of pairs that share one
// adapter, so A_a is fetched once per tile and the gathered token rows stream past it.
#include "common.hpp"
#include "kernels.hpp"
#include "prep.hpp"

namespace meteora {

// ------------------------------------------------------------------------------------------
// Plain-FMA version (fp32 inputs, ranks other than 8/16, odd shapes).  One workgroup per
// (token, slot) pair in bucket order; thread (part, q) sums a stripe of d_in for rank column q.
// ------------------------------------------------------------------------------------------
template <typename TX>
__global__ __launch_bounds__(256) void shrink_fma_kernel(const TX* __restrict__ x, const TX* __restrict__ A,
                                                         const int32_t* __restrict__ topk_idx,
                                                         const float* __restrict__ topk_w,
                                                         const int32_t* __restrict__ bucket_tok,
                                                         const int32_t* __restrict__ bucket_slot,
                                                         int T, int d_in, int N, int r, int RP, int k, float scale,
                                                         float* __restrict__ h32, bf16_t* __restrict__ hdense,
                                                         int ext_stride) {
    __shared__ float red[256];
    const int pos = blockIdx.x;
    const int t = bucket_tok[pos], slot = bucket_slot[pos];
    if (t < 0 || t >= T || slot < 0 || slot >= k) return;   // uniform per workgroup; malformed lists are skipped
    const int a = topk_idx[(size_t)t * k + slot];
    if (a < 0 || a >= N) return;
    const int q = threadIdx.x % RP, part = threadIdx.x / RP, parts = 256 / RP;
    const TX* xt = x + (size_t)t * d_in;
    const TX* Aa = A + (size_t)a * d_in * r;
    float acc = 0.f;
    if (q < r)
        for (int i = part; i < d_in; i += parts) acc = fmaf(to_float(xt[i]), to_float(Aa[(size_t)i * r + q]), acc);
    red[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x < r) {
        float s = 0.f;
        for (int p = 0; p < parts; ++p) s += red[p * RP + threadIdx.x];
        if (h32) h32[((size_t)t * k + slot) * r + threadIdx.x] = s;
        if (hdense) {
            const float w = topk_w[(size_t)t * k + slot];
            hdense[(size_t)t * ext_stride + a * r + threadIdx.x] = from_float<bf16_t>(scale * w * s);
        }
    }
}

// ------------------------------------------------------------------------------------------
// MFMA version for bf16.
//
// A tile is up to 128 consecutive pairs of one adapter's bucket x one 512-wide K-slice.  As in
// the gate kernel, each of the 4 wavefronts takes a quarter of the slice: it gathers its
// 128 x 128 piece of the token rows straight from HBM into its own LDS region (16-byte
// global->LDS loads, 16 lanes per 256-byte row segment, XOR-swizzled chunks) and multiplies it
// by A_a fragments that a pack kernel has laid out in MFMA operand order (one contiguous 1 KB
// block per fragment), reusing every fragment for the 4 row blocks.  The K quarters are summed
// through LDS in a fixed order; the K-slices are written as partial sums hpart[ks][pair][r] and
// added, again in a fixed order, by the finalize kernel, which also applies scale * w and
// writes the dense bf16 operand of the fused expand (zero for adapters a token did not pick).
// ------------------------------------------------------------------------------------------
constexpr int kShrKSL = kSkinnyKSL;
constexpr int kShrKW = kSkinnyKW;
__host__ __device__ constexpr int shrink_region_bytes(int RCB, int RB) {
    const int xbytes = RB * 32 * 256, red = RB * 32 * (RCB * 128 + 16);
    return (int)align_up((size_t)(xbytes > red ? xbytes : red), 1024);
}

template <int RCB, int RB>
__global__ __launch_bounds__(256) void shrink_mfma_kernel(const bf16_t* __restrict__ x, const u32x4* __restrict__ apk,
                                                          const int32_t* __restrict__ offsets,
                                                          const int32_t* __restrict__ bucket_tok,
                                                          const int32_t* __restrict__ bucket_slot, int T, int d_in,
                                                          int N, int r, int k, int KS, float* __restrict__ hpart) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int TM = RB * 32;                              // pairs per tile
    constexpr int kRegion = shrink_region_bytes(RCB, RB);    // LDS bytes per wavefront
    __shared__ int pair_of_row[TM];
    const int lane = threadIdx.x & 63, wq = threadIdx.x >> 6;
    const int ks = blockIdx.x % KS, tile_id = blockIdx.x / KS;

    // which (adapter, tile of its bucket) is tile_id?  lane j owns adapter j.
    int a, row_start, nrows;
    {
        const int lo = (lane < N) ? offsets[lane] : 0, hi = (lane < N) ? offsets[lane + 1] : 0;
        const int tiles = ceil_div(hi - lo, TM);
        int incl = tiles;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int n = __shfl_up(incl, off);
            if (lane >= off) incl += n;
        }
        const unsigned long long m = __ballot(lane < N && tile_id < incl);
        if (m == 0ull) return;   // past the last tile: the whole workgroup leaves together
        a = __ffsll((long long)m) - 1;
        const int excl = __shfl(incl - tiles, a);
        const int blo = __shfl(lo, a), bhi = __shfl(hi, a);
        row_start = blo + (tile_id - excl) * TM;
        nrows = min(TM, bhi - row_start);
    }
    // tokens of the tile: lane l holds rows l and 64+l (clamped to the first row past the end)
    int tok0, tok1;
    {
        const int r0 = lane < nrows ? lane : 0, r1 = (TM > 64 && 64 + lane < nrows) ? 64 + lane : 0;
        tok0 = bucket_tok[row_start + r0];
        tok1 = bucket_tok[row_start + r1];
        tok0 = min(max(tok0, 0), T - 1);
        tok1 = min(max(tok1, 0), T - 1);
        if (wq == 0) {
            const int s0 = bucket_slot[row_start + r0], s1 = bucket_slot[row_start + r1];
            pair_of_row[lane] = tok0 * k + min(max(s0, 0), k - 1);
            if (TM > 64) pair_of_row[64 + lane] = tok1 * k + min(max(s1, 0), k - 1);
        }
    }
    unsigned char* region = smem + wq * kRegion;
    const int kbase = ks * kShrKSL + wq * kShrKW;
    const int nrb = ceil_div(nrows, 32);   // row blocks that hold at least one pair

    {
        const int rsub = lane >> 4, p = lane & 15;
#pragma unroll
        for (int j = 0; j < RB * 8; ++j) {
            if ((j >> 3) < nrb) {   // uniform
                const int row = 4 * j + rsub;
                const int t = __shfl(row < 64 ? tok0 : tok1, row & 63);
                int kk = kbase + ((p ^ (row & 15)) << 3);
                kk = kk <= d_in - 8 ? kk : d_in - 8;   // columns past d_in meet zero weights
                const bf16_t* src = x + (size_t)t * d_in + kk;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                                 (__attribute__((address_space(3))) void*)(region + j * 1024), 16, 0,
                                                 0);
            }
        }
    }
    bf16x8 af[8][RCB];
    {
        const int S16 = KS * (kShrKSL / 16);
        const u32x4* abase = apk + ((size_t)a * S16 + (size_t)(ks * 4 + wq) * 8) * RCB * 64 + lane;
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int cb = 0; cb < RCB; ++cb) {
                const u32x4 v = abase[(size_t)(s * RCB + cb) * 64];
                af[s][cb] = __builtin_bit_cast(bf16x8, v);
            }
    }
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_wave_barrier();

    f32x16 acc[RB][RCB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < RCB; ++cb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[rb][cb][i] = 0.f;

    const int lrow = lane & 31, khalf = lane >> 5;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        if (rb < nrb) {
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const int row = rb * 32 + lrow;
                const int pos = (s * 2 + khalf) ^ (row & 15);
                const bf16x8 xf = *reinterpret_cast<const bf16x8*>(region + row * 256 + pos * 16);
#pragma unroll
                for (int cb = 0; cb < RCB; ++cb)
                    acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[s][cb], xf, acc[rb][cb], 0, 0, 0);
            }
        }
    }

    constexpr int kRowBytes = RCB * 128 + 16;
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < RCB; ++cb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int m = rb * 32 + lrow, n = cb * 32 + g * 8 + khalf * 4;
                f32x4 v = {acc[rb][cb][g * 4 + 0], acc[rb][cb][g * 4 + 1], acc[rb][cb][g * 4 + 2],
                           acc[rb][cb][g * 4 + 3]};
                *reinterpret_cast<f32x4*>(region + m * kRowBytes + n * 4) = v;
            }
    __syncthreads();
    const size_t pairs = (size_t)T * k;
    for (int e = threadIdx.x; e < nrows * r; e += 256) {
        const int m = e / r, q = e - m * r;
        const int off = m * kRowBytes + q * 4;
        const float v0 = *reinterpret_cast<const float*>(smem + off);
        const float v1 = *reinterpret_cast<const float*>(smem + kRegion + off);
        const float v2 = *reinterpret_cast<const float*>(smem + 2 * kRegion + off);
        const float v3 = *reinterpret_cast<const float*>(smem + 3 * kRegion + off);
        hpart[((size_t)ks * pairs + pair_of_row[m]) * r + q] = (v0 + v1) + (v2 + v3);
    }
}

// ------------------------------------------------------------------------------------------
// MFMA version for bf16, whole contraction in one workgroup.
//
// A tile is up to RB*32 consecutive pairs of one adapter's bucket; the workgroup walks all of
// d_in in 512-wide slices.  Each of the 4 wavefronts takes a quarter of every slice: it gathers
// its piece of the token rows straight from HBM into its own LDS region (16-byte global->LDS
// loads, 16 lanes per 256-byte row segment, XOR-swizzled chunks) and multiplies it by A_a
// fragments already laid out in MFMA operand order (one contiguous 1 KB block per fragment).
// The loads of slice s+1 (x piece into the other half of the region, A fragments into the other
// register set) are in flight while slice s is multiplied; the wavefronts do not synchronise in
// the loop.  At the end the 4 K quarters are summed through LDS in a fixed order and the tile's
// pairs are written as h32[pair][r] and/or as their r columns of the dense expand operand
// hdense[t][a*r+q] = bf16(scale * w[t,slot] * h); the other columns of hdense must already be
// zero (the bucket scatter clears the rows).
// ------------------------------------------------------------------------------------------
__host__ __device__ constexpr int shrink_fullk_region_bytes(int RCB, int RB) {
    const int xbytes = 2 * RB * 32 * 256, red = RB * 32 * (RCB * 128 + 16);
    return (int)align_up((size_t)(xbytes > red ? xbytes : red), 1024);
}

template <int RCB, int RB>
__global__ __launch_bounds__(256) void shrink_fullk_kernel(const bf16_t* __restrict__ x, const u32x4* __restrict__ apk,
                                                           const int32_t* __restrict__ offsets,
                                                           const int32_t* __restrict__ bucket_tok,
                                                           const int32_t* __restrict__ bucket_slot,
                                                           const float* __restrict__ topk_w, int T, int d_in, int N,
                                                           int r, int k, int KS, float scale,
                                                           float* __restrict__ h32, bf16_t* __restrict__ hdense,
                                                           int ext_stride) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int TM = RB * 32;                                   // pairs per tile (<= 64)
    constexpr int kXBytes = RB * 32 * 256;                        // one x piece
    constexpr int kRegion = shrink_fullk_region_bytes(RCB, RB);   // LDS bytes per wavefront
    constexpr int kLoads = RB * 8 + 8 * RCB;                      // vector-memory instructions per slice
    static_assert(TM <= 64 && kLoads < 64, "one lane per tile row; vmcnt holds 6 bits");
    __shared__ int pair_of_row[TM];
    const int lane = threadIdx.x & 63, wq = threadIdx.x >> 6;
    const int tile_id = blockIdx.x;

    // which (adapter, tile of its bucket) is tile_id?  lane j owns adapter j.
    int a, row_start, nrows;
    {
        const int lo = (lane < N) ? offsets[lane] : 0, hi = (lane < N) ? offsets[lane + 1] : 0;
        const int tiles = ceil_div(hi - lo, TM);
        int incl = tiles;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int n = __shfl_up(incl, off);
            if (lane >= off) incl += n;
        }
        const unsigned long long m = __ballot(lane < N && tile_id < incl);
        if (m == 0ull) return;   // past the last tile: the whole workgroup leaves together
        a = __ffsll((long long)m) - 1;
        const int excl = __shfl(incl - tiles, a);
        const int blo = __shfl(lo, a), bhi = __shfl(hi, a);
        row_start = blo + (tile_id - excl) * TM;
        nrows = min(TM, bhi - row_start);
    }
    // token of tile row `lane` (rows past the end repeat row 0: loaded, multiplied, never stored)
    int tok;
    {
        const int r0 = lane < nrows ? lane : 0;
        tok = min(max(bucket_tok[row_start + r0], 0), T - 1);
        if (wq == 0 && lane < TM) pair_of_row[lane] = tok * k + min(max(bucket_slot[row_start + r0], 0), k - 1);
    }
    unsigned char* region = smem + wq * kRegion;
    const int S16 = KS * (kShrKSL / 16);
    const int rsub = lane >> 4, p = lane & 15;

    auto issue = [&](int s, int buf, bf16x8 (&af)[8][RCB]) {
        const int kbase = s * kShrKSL + wq * kShrKW;
#pragma unroll
        for (int j = 0; j < RB * 8; ++j) {
            const int row = 4 * j + rsub;
            const int t = __shfl(tok, row);
            int kk = kbase + ((p ^ (row & 15)) << 3);
            kk = kk <= d_in - 8 ? kk : d_in - 8;   // columns past d_in meet zero weights
            const bf16_t* src = x + (size_t)t * d_in + kk;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)(region + buf * kXBytes + j * 1024),
                                             16, 0, 0);
        }
        const u32x4* abase = apk + ((size_t)a * S16 + (size_t)(s * 4 + wq) * 8) * RCB * 64 + lane;
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8)
#pragma unroll
            for (int cb = 0; cb < RCB; ++cb) {
                const u32x4 v = abase[(size_t)(s8 * RCB + cb) * 64];
                af[s8][cb] = __builtin_bit_cast(bf16x8, v);
            }
    };

    f32x16 acc[RB][RCB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < RCB; ++cb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[rb][cb][i] = 0.f;
    const int lrow = lane & 31, khalf = lane >> 5;
    const int nrb = ceil_div(nrows, 32);   // row blocks that hold at least one pair

    auto compute = [&](int buf, const bf16x8 (&af)[8][RCB]) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            if (rb < nrb) {   // uniform
#pragma unroll
                for (int s8 = 0; s8 < 8; ++s8) {
                    const int row = rb * 32 + lrow;
                    const int pos = (s8 * 2 + khalf) ^ (row & 15);
                    const bf16x8 xf = *reinterpret_cast<const bf16x8*>(region + buf * kXBytes + row * 256 + pos * 16);
#pragma unroll
                    for (int cb = 0; cb < RCB; ++cb)
                        acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[s8][cb], xf, acc[rb][cb], 0, 0, 0);
                }
            }
        }
    };
    // all loads of the older slice have landed when at most the newer slice's kLoads are outstanding
    auto wait_older = [&](bool newer_in_flight) {
        if (newer_in_flight) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoads) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_wave_barrier();
    };

    // Two slices per round, branch-free while both successors exist (a branch around a load would make
    // the compiler wait for every outstanding load before the next use of a fragment register).
    bf16x8 af0[8][RCB], af1[8][RCB];
    issue(0, 0, af0);
    int s = 0;
    for (; s + 2 < KS; s += 2) {
        issue(s + 1, 1, af1);
        wait_older(true);
        compute(0, af0);
        __builtin_amdgcn_wave_barrier();   // this wavefront's reads of half 0 are done before it is refilled
        issue(s + 2, 0, af0);
        wait_older(true);
        compute(1, af1);
        __builtin_amdgcn_wave_barrier();
    }
    if (s + 1 < KS) {   // two slices left (uniform)
        issue(s + 1, 1, af1);
        wait_older(true);
        compute(0, af0);
        wait_older(false);
        compute(1, af1);
    } else {            // one slice left
        wait_older(false);
        compute(0, af0);
    }

    // ---- sum the 4 K quarters through LDS (fixed order), then emit the tile's pairs ----------------
    constexpr int kRowBytes = RCB * 128 + 16;
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < RCB; ++cb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int m = rb * 32 + lrow, n = cb * 32 + g * 8 + khalf * 4;
                f32x4 v = {acc[rb][cb][g * 4 + 0], acc[rb][cb][g * 4 + 1], acc[rb][cb][g * 4 + 2],
                           acc[rb][cb][g * 4 + 3]};
                *reinterpret_cast<f32x4*>(region + m * kRowBytes + n * 4) = v;
            }
    __syncthreads();
    for (int e = threadIdx.x; e < nrows * r; e += 256) {
        const int m = e / r, q = e - m * r;
        const int off = m * kRowBytes + q * 4;
        const float v0 = *reinterpret_cast<const float*>(smem + off);
        const float v1 = *reinterpret_cast<const float*>(smem + kRegion + off);
        const float v2 = *reinterpret_cast<const float*>(smem + 2 * kRegion + off);
        const float v3 = *reinterpret_cast<const float*>(smem + 3 * kRegion + off);
        const float h = (v0 + v1) + (v2 + v3);
        const int pair = pair_of_row[m];
        if (h32) h32[(size_t)pair * r + q] = h;
        if (hdense)
            hdense[(size_t)(pair / k) * ext_stride + a * r + q] = from_float<bf16_t>(scale * topk_w[pair] * h);
    }
}

// Sum the K-slices (fixed order) and emit h32[pair][r] and/or the dense expand operand
// hdense[t][a*r+q] = bf16(scale * w[t,slot] * h), zero where the token did not select adapter a.
// One thread per 16-byte chunk (8 columns) of hdense.  R8 = (r % 8 == 0): the chunk lies inside one
// adapter, so the thread decides once whether it is a zero chunk (most are) before touching hpart.
template <bool R8>
__global__ __launch_bounds__(256) void shrink_finalize_kernel(const float* __restrict__ hpart, int KS,
                                                              const int32_t* __restrict__ topk_idx,
                                                              const float* __restrict__ topk_w, int T, int N, int r,
                                                              int k, float scale, float* __restrict__ h32,
                                                              bf16_t* __restrict__ hdense, int ext_stride) {
    const size_t pairs = (size_t)T * k;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (hdense) {
        const int cpr = ext_stride / 8;   // 16-byte chunks per row
        if (gid < (int64_t)T * cpr) {
            const int t = (int)(gid / cpr), c = (int)(gid % cpr);
            union { bf16_t h[8]; u32x4 v; } o;
            if (R8) {
                const int a = (c * 8) / r, q0 = c * 8 - a * r;
                int slot = -1;
                if (a < N)
                    for (int s = 0; s < k; ++s)
                        if (topk_idx[(size_t)t * k + s] == a) slot = s;
                if (slot < 0) {
                    o.v = u32x4{0u, 0u, 0u, 0u};
                } else {
                    const size_t pair = (size_t)t * k + slot;
                    f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
                    // K-slices are added in order; 8 slices' loads go out together (latency-bound loop)
                    for (int ks0 = 0; ks0 < KS; ks0 += 8) {
                        f32x4 vl[8], vh[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const float* src = hpart + ((size_t)min(ks0 + u, KS - 1) * pairs + pair) * r + q0;
                            vl[u] = *reinterpret_cast<const f32x4*>(src);
                            vh[u] = *reinterpret_cast<const f32x4*>(src + 4);
                        }
#pragma unroll
                        for (int u = 0; u < 8; ++u)
                            if (ks0 + u < KS) { lo += vl[u]; hi += vh[u]; }
                    }
                    const float sw = scale * topk_w[pair];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        o.h[e] = from_float<bf16_t>(sw * lo[e]);
                        o.h[4 + e] = from_float<bf16_t>(sw * hi[e]);
                    }
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int col = c * 8 + e;
                    const int a = col / r, q = col - a * r;
                    float val = 0.f;
                    if (a < N) {
                        for (int slot = 0; slot < k; ++slot) {
                            if (topk_idx[(size_t)t * k + slot] == a) {
                                float s = 0.f;
                                for (int ks = 0; ks < KS; ++ks)
                                    s += hpart[((size_t)ks * pairs + (size_t)t * k + slot) * r + q];
                                val = scale * topk_w[(size_t)t * k + slot] * s;
                            }
                        }
                    }
                    o.h[e] = from_float<bf16_t>(val);
                }
            }
            *reinterpret_cast<u32x4*>(hdense + (size_t)t * ext_stride + c * 8) = o.v;
        }
    }
    if (h32 && gid < (int64_t)pairs * r) {
        float s = 0.f;
        for (int ks = 0; ks < KS; ++ks) s += hpart[(size_t)ks * pairs * r + gid];
        h32[gid] = s;
    }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(u32x4* __restrict__ p, size_t n16) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) p[i] = u32x4{0u, 0u, 0u, 0u};
}

static int shrink_kslices(int d_in) { return ceil_div(d_in, kShrKSL); }
static bool shrink_uses_mfma(bool bf16, int r) { return bf16 && r <= 64; }
// Whole-K tiles (one kernel, no partial sums) need enough tiles in flight to cover the memory latency:
// with fewer than 512 tiles of 32 pairs the K-split kernel + finalize is faster (measured: 4096 tokens
// x top-2 = 256 tiles: 25 us against 20; 16384 x 2: 54 against 64, and 214 against 255 at d_in = 14336).
static bool shrink_whole_k(bool bf16, int r, int64_t pairs) {
    return shrink_uses_mfma(bf16, r) && pairs >= 16384;
}
bool shrink_clears_hdense(bool bf16, int r, int T, int k) { return !shrink_whole_k(bf16, r, (int64_t)T * k); }

size_t shrink_apack_bytes(int d_in, int N, int r, bool bf16) {
    if (!shrink_uses_mfma(bf16, r)) return 0;
    return (size_t)N * shrink_kslices(d_in) * kShrKSL * ceil_div(r, 32) * 32 * sizeof(bf16_t);
}

size_t shrink_hpart_bytes(int T, int d_in, int r, int k, bool bf16) {
    if (!shrink_uses_mfma(bf16, r)) return 0;
    return (size_t)shrink_kslices(d_in) * T * k * r * sizeof(float);
}

hipError_t shrink_init_kernels() {
    hipError_t e = ensure_lds_limit(reinterpret_cast<const void*>(&shrink_fullk_kernel<1, 1>), 4 * shrink_fullk_region_bytes(1, 1));
    if (e == hipSuccess)
        e = ensure_lds_limit(reinterpret_cast<const void*>(&shrink_fullk_kernel<2, 1>), 4 * shrink_fullk_region_bytes(2, 1));
    if (e == hipSuccess)
        e = ensure_lds_limit(reinterpret_cast<const void*>(&shrink_mfma_kernel<1, 2>), 4 * shrink_region_bytes(1, 2));
    if (e == hipSuccess)
        e = ensure_lds_limit(reinterpret_cast<const void*>(&shrink_mfma_kernel<2, 2>), 4 * shrink_region_bytes(2, 2));
    return e;
}

hipError_t launch_shrink(const void* x, const void* A, const int32_t* topk_idx, const float* topk_w,
                         const int32_t* offsets, const int32_t* bucket_tok, const int32_t* bucket_slot,
                         int T, int d_in, int N, int r, int k, float scale, bool bf16,
                         void* apack, float* hpart, float* h32, void* hdense, int ext_stride,
                         hipStream_t stream) {
    const int64_t pairs = (int64_t)T * k;
    if (shrink_uses_mfma(bf16, r)) {
        const int KS = shrink_kslices(d_in), RCB = ceil_div(r, 32), S16 = KS * (kShrKSL / 16);
        // apack has been filled by launch_prep
        if (shrink_whole_k(bf16, r, pairs)) {
            auto launch_wk = [&](auto kern) -> hipError_t {
                const int smem = 4 * shrink_fullk_region_bytes(RCB, 1);
                hipError_t err = ensure_lds_limit(reinterpret_cast<const void*>(kern), smem);
                if (err != hipSuccess) return err;
                const int64_t max_tiles = ceil_div64(pairs, 32) + N;   // every bucket rounds up by at most one tile
                kern<<<(unsigned)max_tiles, 256, smem, stream>>>((const bf16_t*)x, (const u32x4*)apack, offsets,
                                                                 bucket_tok, bucket_slot, topk_w, T, d_in, N, r, k, KS,
                                                                 scale, h32, (bf16_t*)hdense, ext_stride);
                return hipGetLastError();
            };
            return RCB == 1 ? launch_wk(shrink_fullk_kernel<1, 1>) : launch_wk(shrink_fullk_kernel<2, 1>);
        }
        // 64-pair tiles: little padding in small buckets and two workgroups per CU (one loads while the
        // other computes); measured faster than 32- or 128-pair tiles on every configuration
        auto launch = [&](auto kern, int rb) -> hipError_t {
            const int smem = 4 * shrink_region_bytes(RCB, rb);
            hipError_t err = ensure_lds_limit(reinterpret_cast<const void*>(kern), smem);
            if (err != hipSuccess) return err;
            // upper bound of the tile count: every bucket rounds up by at most one tile
            const int64_t max_tiles = ceil_div64(pairs, rb * 32) + N;
            kern<<<(unsigned)(max_tiles * KS), 256, smem, stream>>>((const bf16_t*)x, (const u32x4*)apack, offsets,
                                                                  bucket_tok, bucket_slot, T, d_in, N, r, k, KS, hpart);
            return hipGetLastError();
        };
        hipError_t e;
        if (RCB == 1) e = launch(shrink_mfma_kernel<1, 2>, 2);
        else e = launch(shrink_mfma_kernel<2, 2>, 2);
        if (e != hipSuccess) return e;
        int64_t work = 0;
        if (hdense) work = (int64_t)T * (ext_stride / 8);
        if (h32 && pairs * r > work) work = pairs * r;
        if (r % 8 == 0)
            shrink_finalize_kernel<true><<<(unsigned)ceil_div64(work, 256), 256, 0, stream>>>(
                hpart, KS, topk_idx, topk_w, T, N, r, k, scale, h32, (bf16_t*)hdense, ext_stride);
        else
            shrink_finalize_kernel<false><<<(unsigned)ceil_div64(work, 256), 256, 0, stream>>>(
                hpart, KS, topk_idx, topk_w, T, N, r, k, scale, h32, (bf16_t*)hdense, ext_stride);
        return hipGetLastError();
    }
    int RP = 1;
    while (RP < r) RP <<= 1;
    if (hdense) {   // columns of adapters a token did not select must read as zero
        const size_t n16 = (size_t)T * ext_stride * sizeof(bf16_t) / 16;
        fill_zero_kernel<<<(unsigned)ceil_div64((int64_t)n16, 256), 256, 0, stream>>>((u32x4*)hdense, n16);
    }
    if (bf16)
        shrink_fma_kernel<bf16_t><<<(unsigned)pairs, 256, 0, stream>>>(
            (const bf16_t*)x, (const bf16_t*)A, topk_idx, topk_w, bucket_tok, bucket_slot, T, d_in, N, r, RP, k,
            scale, h32, (bf16_t*)hdense, ext_stride);
    else
        shrink_fma_kernel<float><<<(unsigned)pairs, 256, 0, stream>>>(
            (const float*)x, (const float*)A, topk_idx, topk_w, bucket_tok, bucket_slot, T, d_in, N, r, RP, k,
            scale, h32, (bf16_t*)hdense, ext_stride);
    return hipGetLastError();
}

}  // namespace meteora
