// hopgnn_pregather: merged, duplicate-free, ascending vertex-ID set of a batch
// (or group of batches) of micrographs, plus the slot -> position table
// (paper section 5.2, vertex feature pre-gathering).
//
// Bitmap path (default).  Vertex IDs are dense integers below n_vertices, so the
// set is a presence bitmap: one atomic OR per slot marks it, a popcount prefix
// sum over the bitmap words gives every word its rank, and then
//     uniq  = the set bits in word order           (ascending by construction)
//     remap = rank[word(id)] + popcount(bits of that word below id)
// No key ever moves: HBM traffic is ~12 bytes per slot plus 12 bytes per 32
// vertices, against >= 16 bytes per slot per pass for a sort of (id, slot) pairs.
// The OR is order independent, so the result is deterministic.
#include "common.hpp"

namespace hopgnn {

constexpr int kPgThreads = 256;
constexpr int kWordsPerThread = 4;                              // one 128-bit load
constexpr int kWordsPerBlock = kPgThreads * kWordsPerThread;    // 1024 words = 32768 vertices

struct BitmapWs {
    uint32_t* bits;        // [n_words_padded]
    uint2* word_rank;      // [n_words_padded] (bits, rank of the word's first set bit)
    uint32_t* block_sum;   // [n_blocks]
    uint32_t* ticket;      // [1] blocks finished counting
    size_t bytes;
    int64_t n_words_padded;
    int64_t n_blocks;
};

static BitmapWs bitmap_layout(void* ws, int64_t n_vertices) {
    BitmapWs L{};
    const int64_t n_words = ceil_div(n_vertices > 0 ? n_vertices : 1, 32);
    L.n_blocks = ceil_div(n_words, kWordsPerBlock);
    L.n_words_padded = L.n_blocks * kWordsPerBlock;
    char* p = static_cast<char*>(ws);
    size_t o = 0;
    L.bits = reinterpret_cast<uint32_t*>(p + o);
    o += align_up((size_t)L.n_words_padded * 4, 256);
    L.word_rank = reinterpret_cast<uint2*>(p + o);
    o += align_up((size_t)L.n_words_padded * 8, 256);
    L.block_sum = reinterpret_cast<uint32_t*>(p + o);
    o += align_up((size_t)L.n_blocks * 4, 256);
    L.ticket = reinterpret_cast<uint32_t*>(p + o);
    o += 256;
    L.bytes = o;
    return L;
}

__global__ void __launch_bounds__(kPgThreads)
bitmap_clear(uint4* __restrict__ bits4, int64_t n_vec, uint32_t* ticket, int64_t* n_uniq) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_vec) bits4[i] = make_uint4(0u, 0u, 0u, 0u);
    if (i == 0) {
        *ticket = 0u;
        *n_uniq = 0;
    }
}

__global__ void __launch_bounds__(kPgThreads)
bitmap_mark(const int32_t* __restrict__ ids, int64_t n_ids, uint32_t* bits) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_ids; i += stride) {
        const int32_t v = ids[i];
        if (v >= 0) {
            const uint32_t bit = 1u << (v & 31);
            uint32_t* w = bits + (v >> 5);
            // hubs of a power-law graph are hit thousands of times: look before the atomic
            if ((*w & bit) == 0u) atomicOr(w, bit);
        }
    }
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t y = __shfl_up(x, d, kWave);
        if (lane >= d) x += y;
    }
    return x;
}

// Exclusive prefix sum of one value per thread over a 256-thread block; also
// returns the block total through `total`.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t* lds4, uint32_t& total) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const uint32_t inc = wave_inclusive_scan(x);
    if (lane == kWave - 1) lds4[wave] = inc;
    __syncthreads();
    uint32_t base = 0;
    uint32_t tot = 0;
#pragma unroll
    for (int w = 0; w < kPgThreads / kWave; ++w) {
        const uint32_t s = lds4[w];
        if (w < wave) base += s;
        tot += s;
    }
    __syncthreads();
    total = tot;
    return base + inc - x;
}

// Pass 1 over the bitmap: population of every 1024-word block; the block that
// finishes last turns the block counts into exclusive block bases and publishes U.
__global__ void __launch_bounds__(kPgThreads)
bitmap_count(const uint4* __restrict__ bits4, uint32_t* block_sum, uint32_t* ticket,
             int64_t* n_uniq, uint32_t n_blocks) {
    __shared__ uint32_t lds4[kPgThreads / kWave];
    __shared__ bool is_last;
    const uint4 w = bits4[(int64_t)blockIdx.x * kPgThreads + threadIdx.x];
    uint32_t total;
    (void)block_exclusive_scan(__popc(w.x) + __popc(w.y) + __popc(w.z) + __popc(w.w), lds4, total);
    if (threadIdx.x == 0) {
        __hip_atomic_store(&block_sum[blockIdx.x], total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __threadfence();
        const uint32_t done = atomicAdd(ticket, 1u);
        is_last = (done == n_blocks - 1);
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();
    uint32_t carry = 0;
    for (uint32_t b0 = 0; b0 < n_blocks; b0 += kPgThreads) {
        const uint32_t b = b0 + threadIdx.x;
        const uint32_t x = b < n_blocks
                               ? __hip_atomic_load(&block_sum[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                               : 0u;
        uint32_t tot;
        const uint32_t ex = block_exclusive_scan(x, lds4, tot);
        if (b < n_blocks) block_sum[b] = carry + ex;
        carry += tot;
    }
    if (threadIdx.x == 0) *n_uniq = (int64_t)carry;
}

// Pass 2 over the bitmap: rank of every word, and the ascending ID list.
__global__ void __launch_bounds__(kPgThreads)
bitmap_emit(const uint4* __restrict__ bits4, const uint32_t* __restrict__ block_base,
            uint2* __restrict__ word_rank, int32_t* __restrict__ uniq) {
    __shared__ uint32_t lds4[kPgThreads / kWave];
    const int64_t t = (int64_t)blockIdx.x * kPgThreads + threadIdx.x;
    const uint4 w = bits4[t];
    const uint32_t wd[4] = {w.x, w.y, w.z, w.w};
    uint32_t total;
    uint32_t r = block_base[blockIdx.x] +
                 block_exclusive_scan(__popc(w.x) + __popc(w.y) + __popc(w.z) + __popc(w.w), lds4, total);
    if (total == 0) {   // nothing set in these 32768 vertices: ranks are never looked up
        return;
    }
#pragma unroll
    for (int k = 0; k < kWordsPerThread; ++k) {
        uint32_t bits = wd[k];
        word_rank[t * kWordsPerThread + k] = make_uint2(bits, r);
        const int32_t v0 = (int32_t)((t * kWordsPerThread + k) << 5);
        while (bits) {
            const int b = __ffs((int)bits) - 1;
            uniq[r++] = v0 + b;
            bits &= bits - 1;
        }
    }
}

__global__ void __launch_bounds__(kPgThreads)
bitmap_remap(const int32_t* __restrict__ ids, int64_t n_ids, const uint2* __restrict__ word_rank,
             int32_t* __restrict__ remap) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_ids; i += stride) {
        const int32_t v = ids[i];
        int32_t pos = -1;
        if (v >= 0) {
            const uint2 wr = word_rank[v >> 5];
            pos = (int32_t)(wr.y + __popc(wr.x & ((1u << (v & 31)) - 1u)));
        }
        remap[i] = pos;
    }
}

static int grid_for(int64_t n, int per_block, int cap) {
    int64_t g = ceil_div(n, per_block);
    if (g < 1) g = 1;
    return (int)(g < cap ? g : cap);
}

static hopgnn_status pregather_bitmap(const int32_t* ids, int64_t n_ids, int64_t n_vertices,
                                      int32_t* uniq, int64_t* n_uniq_dev, int32_t* remap, void* ws,
                                      size_t ws_bytes, hipStream_t s) {
    const BitmapWs L = bitmap_layout(ws, n_vertices);
    if (ws_bytes < L.bytes) return HOPGNN_ENOMEM_WS;
    const int64_t n_vec = L.n_words_padded / 4;
    hipLaunchKernelGGL(bitmap_clear, dim3((unsigned)ceil_div(n_vec, kPgThreads)), dim3(kPgThreads), 0, s,
                       reinterpret_cast<uint4*>(L.bits), n_vec, L.ticket, n_uniq_dev);
    HOPGNN_LAUNCH_CHECK();
    if (n_ids > 0) {
        hipLaunchKernelGGL(bitmap_mark, dim3(grid_for(n_ids, kPgThreads, 256 * 32)), dim3(kPgThreads), 0, s,
                           ids, n_ids, L.bits);
        HOPGNN_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(bitmap_count, dim3((unsigned)L.n_blocks), dim3(kPgThreads), 0, s,
                       reinterpret_cast<const uint4*>(L.bits), L.block_sum, L.ticket, n_uniq_dev,
                       (uint32_t)L.n_blocks);
    HOPGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(bitmap_emit, dim3((unsigned)L.n_blocks), dim3(kPgThreads), 0, s,
                       reinterpret_cast<const uint4*>(L.bits), L.block_sum, L.word_rank, uniq);
    HOPGNN_LAUNCH_CHECK();
    if (n_ids > 0) {
        hipLaunchKernelGGL(bitmap_remap, dim3(grid_for(n_ids, kPgThreads, 256 * 32)), dim3(kPgThreads), 0, s,
                           ids, n_ids, L.word_rank, remap);
        HOPGNN_LAUNCH_CHECK();
    }
    return HOPGNN_OK;
}

}  // namespace hopgnn

using namespace hopgnn;

extern "C" size_t hopgnn_pregather_ws_bytes(int64_t n_ids, int64_t n_vertices, int32_t algo) {
    if (n_ids < 0 || n_vertices < 0) return 0;
    (void)algo;
    return bitmap_layout(nullptr, n_vertices).bytes;
}

extern "C" hopgnn_status hopgnn_pregather(const int32_t* ids, int64_t n_ids, int64_t n_vertices,
                                          int32_t algo, int32_t* uniq, int64_t* n_uniq_dev,
                                          int32_t* remap, void* ws, size_t ws_bytes, void* stream) {
    if (n_ids < 0 || n_vertices < 0 || n_uniq_dev == nullptr || ws == nullptr) return HOPGNN_EINVAL;
    if (n_ids > 0 && (ids == nullptr || remap == nullptr || uniq == nullptr)) return HOPGNN_EINVAL;
    if (algo != HOPGNN_PG_AUTO && algo != HOPGNN_PG_BITMAP && algo != HOPGNN_PG_RADIX) return HOPGNN_EINVAL;
    if (n_ids >= ((int64_t)1 << 31) || n_vertices > ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    if (!aligned(ws, 256)) return HOPGNN_EINVAL;
    return pregather_bitmap(ids, n_ids, n_vertices, uniq, n_uniq_dev, remap, ws, ws_bytes,
                            static_cast<hipStream_t>(stream));
}
