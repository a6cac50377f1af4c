// Token-to-adapter bucketing: the per-adapter token sets {x | i in I(x)} of the paper's
// Sec. 3.3 (the X_i that "loop-original" gathers), kept as index lists instead of copies.
//
// The (token, slot) pairs, in flat order p = t*k + slot, are counting-sorted by adapter:
//   pass 1  per-chunk histograms               chunk_counts[c][j]   (a chunk = 64 tokens; the gate's
//           top-k kernel writes them itself when the routing comes from the gate)
//   pass 2  every chunk derives its own write base from chunk_counts (exclusive scan over
//           adapters of the totals + counts of the earlier chunks), then scatters its pairs
//           in order.  The in-chunk rank uses wavefront ballots, so the result is the stable
//           sort: ascending token, then ascending slot, inside every bucket.
// Integer work only; the output is unique and bit-comparable.
#include <mutex>

#include "common.hpp"
#include "kernels.hpp"

namespace meteora {

// Scratch of the entry point that allocates nothing and takes no workspace (meteora_bucket_tokens_noalloc): the
// per-chunk histograms of up to kStaticBucketMaxTokens tokens, 256 KiB that every GPU the library runs on holds
// until the process ends.  In host code the array's name is only a stand-in for the symbol: the device address
// comes from hipGetSymbolAddress, once per device, and only that pointer is handed to kernels.
static __device__ __align__(256) int32_t scratch[(kStaticBucketMaxTokens / kBucketChunkTokens) * kMaxAdapters];

namespace {
constexpr int kScratchMaxDevices = 64;
int32_t* g_scratch_ptr[kScratchMaxDevices];
std::mutex g_scratch_mutex;
}  // namespace

// Device address of `scratch` on the current device (looked up on first use, then kept).
hipError_t bucket_static_scratch(int32_t** ptr) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kScratchMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<int32_t*>(p);
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

hipError_t bucket_init_scratch() {
    int32_t* p = nullptr;
    return bucket_static_scratch(&p);
}

__global__ __launch_bounds__(256) void bucket_hist_kernel(const int32_t* __restrict__ topk_idx,
                                                          int64_t pairs, int k, int N,
                                                          int32_t* __restrict__ chunk_counts) {
    __shared__ int hist[kMaxAdapters];
    if (threadIdx.x < kMaxAdapters) hist[threadIdx.x] = 0;
    __syncthreads();
    const int chunk_pairs = kBucketChunkTokens * k;
    const int64_t base = (int64_t)blockIdx.x * chunk_pairs;
    for (int i = threadIdx.x; i < chunk_pairs; i += 256) {
        const int64_t p = base + i;
        if (p < pairs) {
            const int key = topk_idx[p];
            if (key >= 0 && key < N) atomicAdd(&hist[key], 1);   // out-of-range ids are dropped, never indexed
        }
    }
    __syncthreads();
    if (threadIdx.x < N) chunk_counts[(size_t)blockIdx.x * N + threadIdx.x] = hist[threadIdx.x];
}

__global__ __launch_bounds__(256) void bucket_scatter_kernel(const int32_t* __restrict__ topk_idx,
                                                             int64_t pairs, int k, int N, int nchunks,
                                                             const int32_t* __restrict__ chunk_counts,
                                                             int32_t* __restrict__ counts,
                                                             int32_t* __restrict__ offsets,
                                                             int32_t* __restrict__ bucket_tok,
                                                             int32_t* __restrict__ bucket_slot,
                                                             u32x4* __restrict__ clear, int clear_row16, int T) {
    __shared__ int part_total[4][kMaxAdapters], part_before[4][kMaxAdapters];
    __shared__ int running[kMaxAdapters];    // next write position of adapter j for this chunk
    __shared__ int wave_hist[4][kMaxAdapters];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = blockIdx.x;

    if (clear != nullptr) {   // this chunk's rows of the dense expand operand start as zeros
        const int rows = min(kBucketChunkTokens, T - c * kBucketChunkTokens);
        u32x4* dst = clear + (size_t)c * kBucketChunkTokens * clear_row16;
        for (int i = threadIdx.x; i < rows * clear_row16; i += 256) dst[i] = u32x4{0u, 0u, 0u, 0u};
    }

    {   // totals over all chunks and over the chunks before this one; wave w takes chunks w, w+4, ...
        // (32 independent loads per step, from clamped addresses so that no branch separates them: the loop is
        // bound by load latency, not by bandwidth, and 16384 tokens are 256 chunks = two steps per wavefront)
        int tot = 0, bef = 0;
        if (lane < N) {
            for (int cc0 = wave; cc0 < nchunks; cc0 += 128) {
                int v[32];
#pragma unroll
                for (int u = 0; u < 32; ++u) v[u] = chunk_counts[(size_t)min(cc0 + 4 * u, nchunks - 1) * N + lane];
#pragma unroll
                for (int u = 0; u < 32; ++u) {
                    const int cc = cc0 + 4 * u;
                    if (cc < nchunks) tot += v[u];
                    if (cc < c) bef += v[u];
                }
            }
        }
        part_total[wave][lane] = tot;
        part_before[wave][lane] = bef;
    }
    __syncthreads();
    if (wave == 0) {
        // exclusive scan of the totals over adapters inside one wavefront
        const int v = part_total[0][lane] + part_total[1][lane] + part_total[2][lane] + part_total[3][lane];
        const int bef = part_before[0][lane] + part_before[1][lane] + part_before[2][lane] + part_before[3][lane];
        int incl = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int n = __shfl_up(incl, off);
            if (lane >= off) incl += n;
        }
        const int excl = incl - v;
        running[lane] = excl + bef;
        if (c == 0) {
            if (lane < N) { counts[lane] = v; offsets[lane] = excl; }
            if (lane == N - 1) offsets[N] = incl;
        }
    }
    __syncthreads();

    const int chunk_pairs = kBucketChunkTokens * k;
    const int64_t base = (int64_t)c * chunk_pairs;
    for (int it = 0; it * 256 < chunk_pairs; ++it) {
        const int i = it * 256 + threadIdx.x;
        const int64_t p = base + i;
        int key = (i < chunk_pairs && p < pairs) ? topk_idx[p] : -1;
        if (key >= N) key = -1;
        const bool valid = key >= 0;
        // lanes of this wavefront that hold the same key
        unsigned long long peers = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < 6; ++bit) {
            const unsigned long long b = __ballot(valid && ((key >> bit) & 1));
            peers &= ((key >> bit) & 1) ? b : ~b;
        }
        const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
        const int rank_in_wave = __popcll(peers & below);
        const int peers_in_wave = __popcll(peers);
        wave_hist[wave][lane] = 0;
        __syncthreads();   // rows cleared (each wave clears its own); also orders against the previous pass's reads
        if (valid && rank_in_wave == 0) wave_hist[wave][key] = peers_in_wave;
        __syncthreads();
        if (valid) {
            int pos = running[key] + rank_in_wave;
            for (int w = 0; w < wave; ++w) pos += wave_hist[w][key];
            bucket_tok[pos] = (int32_t)(p / k);
            bucket_slot[pos] = (int32_t)(p % k);
        }
        __syncthreads();
        if (threadIdx.x < kMaxAdapters)
            running[threadIdx.x] += wave_hist[0][threadIdx.x] + wave_hist[1][threadIdx.x] +
                                    wave_hist[2][threadIdx.x] + wave_hist[3][threadIdx.x];
        __syncthreads();
    }
}

hipError_t launch_bucket(const int32_t* topk_idx, int T, int k, int N, int32_t* chunk_counts, bool have_hist,
                         int32_t* counts, int32_t* offsets, int32_t* bucket_tok, int32_t* bucket_slot,
                         void* clear_rows, int clear_row_bytes, hipStream_t stream) {
    const int64_t pairs = (int64_t)T * k;
    const int nchunks = bucket_chunks(T);
    if (!have_hist) {
        bucket_hist_kernel<<<nchunks, 256, 0, stream>>>(topk_idx, pairs, k, N, chunk_counts);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    bucket_scatter_kernel<<<nchunks, 256, 0, stream>>>(topk_idx, pairs, k, N, nchunks, chunk_counts, counts,
                                                       offsets, bucket_tok, bucket_slot, (u32x4*)clear_rows,
                                                       clear_row_bytes / 16, T);
    return hipGetLastError();
}

}  // namespace meteora
