// hopgnn_pregather: merged, duplicate-free, ascending vertex-ID set of a batch
// (or group of batches) of micrographs, plus the slot -> position table
// (paper section 5.2, vertex feature pre-gathering).
//
// Bitmap path (default).  Vertex IDs are dense integers below n_vertices, so the
// set is a presence map: every slot stores a 1 into its vertex's byte, the bytes
// are packed 32:1 into bitmap words, a popcount prefix sum over the words gives
// every word its rank, and then
//     uniq  = the set bits in word order           (ascending by construction)
//     remap = rank[word(id)] + popcount(bits of that word below id)
// No key ever moves: HBM traffic is ~9 bytes per slot plus ~2.4 bytes per vertex,
// against >= 16 bytes per slot per pass for a sort of (id, slot) pairs.
// Marking uses plain byte stores, not atomic ORs on bitmap words: on power-law
// graphs the hubs are hit thousands of times per batch and same-address atomics
// serialise in L2 (measured: 0.3 ms for 0.9 M slots), while racing stores of the
// same value just overwrite each other.  The result does not depend on any order.
#include "common.hpp"

namespace hopgnn {

constexpr int kPgThreads = 256;
constexpr int kWordsPerThread = 4;                              // one 128-bit load
constexpr int kWordsPerBlock = kPgThreads * kWordsPerThread;    // 1024 words = 32768 vertices

struct BitmapWs {
    uint8_t* present;      // [32 * n_words_padded] one byte per vertex
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
    L.present = reinterpret_cast<uint8_t*>(p + o);
    o += align_up((size_t)L.n_words_padded * 32, 256);
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
present_clear(uint4* __restrict__ present16, int64_t n_vec, uint32_t* ticket, int64_t* n_uniq) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride)
        present16[i] = make_uint4(0u, 0u, 0u, 0u);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *ticket = 0u;
        *n_uniq = 0;
    }
}

__global__ void __launch_bounds__(kPgThreads)
present_mark(const int32_t* __restrict__ ids, int64_t n_ids, uint8_t* __restrict__ present) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_ids; i += stride) {
        const int32_t v = ids[i];
        if (v >= 0) present[v] = 1;
    }
}

// 4 presence bytes (each 0 or 1) -> 4 bits: byte k lands on bit 24+k of x * 0x01020408.
__device__ __forceinline__ uint32_t pack4(uint32_t x) { return ((x * 0x01020408u) >> 24) & 0xFu; }
__device__ __forceinline__ uint32_t pack16(const uint4& q) {
    return pack4(q.x) | (pack4(q.y) << 4) | (pack4(q.z) << 8) | (pack4(q.w) << 12);
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

// Pass 1: pack the presence bytes of 4 words per thread into the bitmap, count every
// 1024-word block; the block that finishes last turns the block counts into exclusive
// block bases and publishes U.
__global__ void __launch_bounds__(kPgThreads)
bitmap_pack_count(const uint4* __restrict__ present16, uint4* __restrict__ bits4, uint32_t* block_sum,
                  uint32_t* ticket, int64_t* n_uniq, uint32_t n_blocks) {
    __shared__ uint32_t lds4[kPgThreads / kWave];
    __shared__ bool is_last;
    // A wave covers 8 KiB of presence bytes = 256 bitmap words.  Load k of lane l is the
    // 16-byte piece k*64+l of that range (fully coalesced) = one half of word k*32 + l/2;
    // lanes 2j and 2j+1 exchange halves and the even lane stores the word.
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave_id = ((int64_t)blockIdx.x * kPgThreads + threadIdx.x) / kWave;
    const uint4* src = present16 + wave_id * (kWave * 8);
    uint32_t* dst = reinterpret_cast<uint32_t*>(bits4) + wave_id * (kWave * kWordsPerThread);
    uint4 q[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) q[k] = src[k * kWave + lane];
    uint32_t mine = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const uint32_t half = pack16(q[k]);
        mine += __popc(half);
        const uint32_t other = __shfl_xor(half, 1, kWave);
        if ((lane & 1) == 0) dst[k * 32 + (lane >> 1)] = half | (other << 16);
    }
    uint32_t total;
    (void)block_exclusive_scan(mine, lds4, total);
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
    const int64_t n_vec = L.n_words_padded * 2;   // 16-byte words of the presence map
    hipLaunchKernelGGL(present_clear, dim3(grid_for(n_vec, kPgThreads, 256 * 16)), dim3(kPgThreads), 0, s,
                       reinterpret_cast<uint4*>(L.present), n_vec, L.ticket, n_uniq_dev);
    HOPGNN_LAUNCH_CHECK();
    if (n_ids > 0) {
        hipLaunchKernelGGL(present_mark, dim3(grid_for(n_ids, kPgThreads, 256 * 32)), dim3(kPgThreads), 0, s,
                           ids, n_ids, L.present);
        HOPGNN_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(bitmap_pack_count, dim3((unsigned)L.n_blocks), dim3(kPgThreads), 0, s,
                       reinterpret_cast<const uint4*>(L.present), reinterpret_cast<uint4*>(L.bits),
                       L.block_sum, L.ticket, n_uniq_dev, (uint32_t)L.n_blocks);
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
