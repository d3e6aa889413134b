// hopgnn_pregather: merged, duplicate-free, ascending vertex-ID set of a batch
// (or group of batches) of micrographs, plus the slot -> position table
// (paper section 5.2, vertex feature pre-gathering).
//
// Bitmap path (default).  Vertex IDs are dense integers below n_vertices, so the
// set is a presence map: every slot stores a 1 into its vertex's byte, the bytes
// are packed 32:1 into bitmap words, a popcount prefix sum over the words gives
// every word its rank (kept as rank inside its 1024-word chunk + the chunk's base), and then
//     uniq  = the set bits in word order           (ascending by construction)
//     remap = base[chunk(id)] + rank[word(id)] + popcount(bits of that word below id)
// Both depend only on the packing pass, so they share one launch.
// No key ever moves: HBM traffic is ~9 bytes per slot plus ~2.4 bytes per vertex,
// against >= 16 bytes per slot per pass for a sort of (id, slot) pairs.
// Marking uses plain byte stores, not atomic ORs on bitmap words: on power-law
// graphs the hubs are hit thousands of times per batch and same-address atomics
// serialise in L2 (measured: 0.3 ms for 0.9 M slots), while racing stores of the
// same value just overwrite each other.  The result does not depend on any order.
#include <mutex>

#include "pregather_internal.hpp"

namespace hopgnn {

// level-major slot layout of a batch (see hopgnn_sample)
struct SlotShape {
    int32_t n_layers;
    int32_t P[kMaxLayers + 1];      // slots per micrograph at level h
    int32_t base[kMaxLayers + 2];   // first slot of level h
};

constexpr int kPgThreads = 256;
constexpr int kWordsPerThread = 4;                              // one 128-bit load
constexpr int kWordsPerBlock = kPgThreads * kWordsPerThread;    // 1024 words = 32768 vertices

constexpr int kMaxPackGrid = 1024;
// Up to this many chunks (2 M vertices) the packing pass scans its own chunk counts ("last
// workgroup to finish"); beyond it the scan is a launch of its own, see bitmap_scan_sums.
constexpr int kTicketChunks = 64;

struct BitmapWs {
    uint8_t* present;      // [32 * n_words_padded] one byte per vertex
    uint2* word_rank;      // [n_words_padded] (bits, rank of the word's first set bit inside its chunk)
    uint32_t* block_sum;   // [n_blocks] set bits per 1024-word chunk, then their exclusive prefix sum
    uint32_t* ticket;      // [1] workgroups that finished counting (small inputs only, see kTicketChunks)
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
        if (n_uniq != nullptr) *n_uniq = 0;
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

// Pass 1: pack the presence bytes into bitmap words, rank every word inside its 1024-word chunk
// and count the chunk; the workgroup that finishes last turns the chunk counts into exclusive
// chunk bases and publishes U.  With UNMARK the marks are wiped as they are read (only the
// 16-byte pieces that hold one) and the ticket is reset, which leaves the presence map and the
// ticket as hopgnn_pregather_ws_init left them.
template <bool UNMARK, bool TICKET>
__global__ void __launch_bounds__(kPgThreads)
bitmap_pack_count(uint4* __restrict__ present16, uint2* __restrict__ word_rank, uint32_t* block_sum,
                  uint32_t* ticket, int64_t* n_uniq, uint32_t n_blocks) {
    __shared__ uint32_t lds4[kPgThreads / kWave];
    __shared__ bool is_last;
    // A wave covers 8 KiB of presence bytes = 256 bitmap words.  Load k of lane l is the
    // 16-byte piece k*64+l of that range (fully coalesced) = one half of word k*32 + l/2;
    // lanes 2j and 2j+1 exchange halves and the even lane owns the word.
    // A workgroup takes chunks blockIdx.x, blockIdx.x + gridDim.x, ... and draws ONE ticket at the
    // end (one ticket per chunk serialised thousands of same-address atomics on large graphs).
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    for (uint32_t chunk = blockIdx.x; chunk < n_blocks; chunk += gridDim.x) {
        const int64_t wave_id = (int64_t)chunk * (kPgThreads / kWave) + wave;
        uint4* src = present16 + wave_id * (kWave * 8);
        uint2* dst = word_rank + wave_id * (kWave * kWordsPerThread);
        uint4 q[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) q[k] = src[k * kWave + lane];
        if (UNMARK) {
            // Wipe only the pieces that hold a mark while they are few (sparse partial-line writes);
            // once more than a quarter of a 1 KiB run is marked, rewrite the whole run (full lines).
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const bool marked = (q[k].x | q[k].y | q[k].z | q[k].w) != 0u;
                const bool dense = __popcll(__ballot(marked)) > kWave / 4;
                if (marked || dense) src[k * kWave + lane] = make_uint4(0u, 0u, 0u, 0u);
            }
        }
        // word k*32 + lane/2 of the wave, its popcount on the even lane, and its rank among the
        // wave's 256 words in word order (row k before row k+1, lanes in order inside a row)
        uint32_t word[8], rank[8];
        uint32_t wave_total = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const uint32_t half = pack16(q[k]);
            const uint32_t other = __shfl_xor(half, 1, kWave);
            word[k] = half | (other << 16);
            const uint32_t cnt = (lane & 1) == 0 ? __popc(word[k]) : 0u;
            const uint32_t inc = wave_inclusive_scan(cnt);
            rank[k] = wave_total + inc - cnt;
            wave_total += __shfl(inc, kWave - 1, kWave);
        }
        if (lane == 0) lds4[wave] = wave_total;
        __syncthreads();
        uint32_t wave_base = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kPgThreads / kWave; ++w) {
            const uint32_t t = lds4[w];
            if (w < wave) wave_base += t;
            total += t;
        }
        __syncthreads();
        if ((lane & 1) == 0) {
#pragma unroll
            for (int k = 0; k < 8; ++k) dst[k * 32 + (lane >> 1)] = make_uint2(word[k], wave_base + rank[k]);
        }
        if (threadIdx.x == 0)
            __hip_atomic_store(&block_sum[chunk], total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (!TICKET) return;      // the chunk counts are scanned by a launch of their own
    if (threadIdx.x == 0) {
        __threadfence();
        is_last = atomicAdd(ticket, 1u) == gridDim.x - 1;
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
    if (threadIdx.x == 0) {
        *n_uniq = (int64_t)carry;
        if (UNMARK) *ticket = 0u;
    }
}

// The scan of the chunk counts as a launch of its own (one workgroup): exclusive prefix in place,
// U published.  Used when there are many chunks: the in-kernel variant needs a device-scope
// release fence in every workgroup before it draws its ticket, and with thousands of workgroups
// those fences cost far more than one small launch.
__global__ void __launch_bounds__(kPgThreads)
bitmap_scan_sums(uint32_t* __restrict__ block_sum, uint32_t n_blocks, int64_t* __restrict__ n_uniq) {
    __shared__ uint32_t lds4[kPgThreads / kWave];
    // thread t owns the contiguous run [t*per, (t+1)*per): sum it, scan the 256 run sums, write back
    const uint32_t per = (n_blocks + kPgThreads - 1) / kPgThreads;
    const uint32_t b0 = threadIdx.x * per, b1 = b0 + per < n_blocks ? b0 + per : n_blocks;
    uint32_t mine = 0;
    for (uint32_t b = b0; b < b1; ++b) mine += block_sum[b];
    uint32_t total;
    uint32_t run = block_exclusive_scan(mine, lds4, total);
    for (uint32_t b = b0; b < b1; ++b) {
        const uint32_t x = block_sum[b];
        block_sum[b] = run;
        run += x;
    }
    if (threadIdx.x == 0 && n_uniq != nullptr) *n_uniq = (int64_t)total;
}

// Pass 2, one launch for both outputs.  Workgroups [0, n_emit_blocks) walk one chunk of the
// bitmap each and write its set bits to uniq in word order; the others fill remap for a strided
// share of the slots.
__global__ void __launch_bounds__(kPgThreads)
bitmap_emit_remap(const uint2* __restrict__ word_rank, const uint32_t* __restrict__ block_base,
                  uint32_t n_emit_blocks, int32_t* __restrict__ uniq, const int32_t* __restrict__ ids, int64_t n_ids,
                  int32_t* __restrict__ remap) {
    if (blockIdx.x < n_emit_blocks) {
        const int64_t t = (int64_t)blockIdx.x * kPgThreads + threadIdx.x;
        const uint4* wr = reinterpret_cast<const uint4*>(word_rank + t * kWordsPerThread);
        const uint4 a = wr[0], b = wr[1];              // (bits, rank) of words 4t .. 4t+3
        const uint32_t wd[4] = {a.x, a.z, b.x, b.z};
        const uint32_t rk[4] = {a.y, a.w, b.y, b.w};
        if ((wd[0] | wd[1] | wd[2] | wd[3]) == 0u) return;
        const uint32_t base = block_base[blockIdx.x];
#pragma unroll
        for (int k = 0; k < kWordsPerThread; ++k) {
            uint32_t bits = wd[k];
            uint32_t r = base + rk[k];
            const int32_t v0 = (int32_t)((t * kWordsPerThread + k) << 5);
            while (bits) {
                const int bit = __ffs((int)bits) - 1;
                uniq[r++] = v0 + bit;
                bits &= bits - 1;
            }
        }
        return;
    }
    const int64_t stride = (int64_t)(gridDim.x - n_emit_blocks) * blockDim.x;
    for (int64_t i = (int64_t)(blockIdx.x - n_emit_blocks) * blockDim.x + threadIdx.x; i < n_ids; i += stride) {
        const int32_t v = ids[i];
        int32_t pos = -1;
        if (v >= 0) {
            const uint2 wr = word_rank[v >> 5];
            pos = (int32_t)(block_base[v >> 15] + wr.y + __popc(wr.x & ((1u << (v & 31)) - 1u)));
        }
        remap[i] = pos;
    }
}

static int grid_for(int64_t n, int per_block, int cap) {
    int64_t g = ceil_div(n, per_block);
    if (g < 1) g = 1;
    return (int)(g < cap ? g : cap);
}

// Packing pass + the fused second pass, from a presence map that holds the marks of `ids`.
static hopgnn_status bitmap_from_marks(const BitmapWs& L, bool unmark, const int32_t* ids, int64_t n_ids,
                                       int32_t* uniq, int64_t* n_uniq_dev, int32_t* remap, hipStream_t s) {
    const dim3 pack_grid((unsigned)(L.n_blocks < kMaxPackGrid ? L.n_blocks : kMaxPackGrid));
    const bool ticket = L.n_blocks <= kTicketChunks;
    auto pack = unmark ? (ticket ? bitmap_pack_count<true, true> : bitmap_pack_count<true, false>)
                       : (ticket ? bitmap_pack_count<false, true> : bitmap_pack_count<false, false>);
    hipLaunchKernelGGL(pack, pack_grid, dim3(kPgThreads), 0, s, reinterpret_cast<uint4*>(L.present), L.word_rank,
                       L.block_sum, L.ticket, n_uniq_dev, (uint32_t)L.n_blocks);
    HOPGNN_LAUNCH_CHECK();
    if (!ticket) {
        hipLaunchKernelGGL(bitmap_scan_sums, dim3(1), dim3(kPgThreads), 0, s, L.block_sum, (uint32_t)L.n_blocks,
                           n_uniq_dev);
        HOPGNN_LAUNCH_CHECK();
    }
    const unsigned remap_blocks = n_ids > 0 ? (unsigned)grid_for(n_ids, kPgThreads, 256 * 32) : 0u;
    hipLaunchKernelGGL(bitmap_emit_remap, dim3((unsigned)L.n_blocks + remap_blocks), dim3(kPgThreads), 0, s, L.word_rank,
                       L.block_sum, (uint32_t)L.n_blocks, uniq, ids, n_ids, remap);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
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
    // unmark while packing: whatever state the workspace came in, it leaves clean
    return bitmap_from_marks(L, true, ids, n_ids, uniq, n_uniq_dev, remap, s);
}

// ------------------------------------------------------------------ radix path --
//
// LSD radix sort of (key, slot) pairs, 8 bits per pass, then head flags + prefix sum:
//     key = id for valid slots, 2^bits for invalid ones (bits = width of n_vertices-1), so
//           invalid slots sort behind every vertex and ceil((bits+1)/8) passes suffice;
//     a pass = per-tile digit histogram -> exclusive scan over (digit, tile) -> stable
//           scatter.  Ranking inside a tile is by wavefront ballots (the lanes holding the
//           same digit are found with 8 ballots, one per digit bit), and the tile is first
//           put in digit order in LDS so that runs of equal digits leave as coalesced writes;
//     uniq = first key of every run of equal valid keys, remap[slot] = number of runs before it.
// Identical output to the bitmap path (ascending uniq, same remap).  It moves 16 bytes per
// slot per pass, so it only pays when n_vertices is huge next to the number of slots.

constexpr int kRxThreads = 256;
constexpr int kRxIpt = 8;                                  // items per thread
constexpr int kRxTile = kRxThreads * kRxIpt;               // 2048 items per workgroup
constexpr int kRxWaves = kRxThreads / kWave;

struct RadixWs {
    uint32_t *keys[2], *vals[2];   // ping-pong pair buffers [n]
    uint32_t* flags;               // [n] head flags, then their exclusive prefix
    uint32_t* hist;                // [256][n_tiles], scanned in place
    uint32_t* sums;                // chunk sums of the scans
    uint32_t* ticket;
    size_t bytes;
    int64_t n_tiles, scan_len_max;
};

static RadixWs radix_layout(void* ws, int64_t n_ids) {
    RadixWs L{};
    const int64_t n = n_ids > 0 ? n_ids : 1;
    L.n_tiles = ceil_div(n, kRxTile);
    const int64_t hist_len = 256 * L.n_tiles;
    L.scan_len_max = hist_len > n ? hist_len : n;
    char* p = static_cast<char*>(ws);
    size_t o = 0;
    auto take = [&](size_t bytes) {
        char* q = p + o;
        o += align_up(bytes, 256);
        return q;
    };
    for (int i = 0; i < 2; ++i) L.keys[i] = reinterpret_cast<uint32_t*>(take((size_t)n * 4));
    for (int i = 0; i < 2; ++i) L.vals[i] = reinterpret_cast<uint32_t*>(take((size_t)n * 4));
    L.flags = reinterpret_cast<uint32_t*>(take((size_t)n * 4));
    L.hist = reinterpret_cast<uint32_t*>(take((size_t)hist_len * 4));
    L.sums = reinterpret_cast<uint32_t*>(take((size_t)ceil_div(L.scan_len_max, kWordsPerBlock) * 4));
    L.ticket = reinterpret_cast<uint32_t*>(take(256));
    L.bytes = o;
    return L;
}

__device__ __forceinline__ uint32_t radix_key(int32_t id, uint32_t invalid_key) {
    return id >= 0 ? (uint32_t)id : invalid_key;
}

// Item order inside a tile: wave w, round j, lane l  <->  index base + w*512 + j*64 + l,
// i.e. ascending index, which is what makes the ballot ranking stable.
template <bool FIRST>
__global__ void __launch_bounds__(kRxThreads)
radix_histogram(const uint32_t* __restrict__ keys_in, int64_t n, int shift, uint32_t invalid_key,
                uint32_t* __restrict__ hist, uint32_t n_tiles) {
    __shared__ uint32_t counts[256];
    counts[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kRxTile;
#pragma unroll
    for (int j = 0; j < kRxIpt; ++j) {
        const int64_t i = base + j * kRxThreads + threadIdx.x;
        if (i < n) {
            const uint32_t key = FIRST ? radix_key((int32_t)keys_in[i], invalid_key) : keys_in[i];
            atomicAdd(&counts[(key >> shift) & 255u], 1u);
        }
    }
    __syncthreads();
    hist[(int64_t)threadIdx.x * n_tiles + blockIdx.x] = counts[threadIdx.x];
}

template <bool FIRST>
__global__ void __launch_bounds__(kRxThreads)
radix_scatter(const uint32_t* __restrict__ keys_in, const uint32_t* __restrict__ vals_in, int64_t n,
              int shift, uint32_t invalid_key, const uint32_t* __restrict__ hist, uint32_t n_tiles,
              uint32_t* __restrict__ keys_out, uint32_t* __restrict__ vals_out) {
    __shared__ uint32_t wave_count[kRxWaves][256];   // per wave, per digit: count, then start inside the digit
    __shared__ uint32_t digit_start[256];            // start of the digit's run in the tile
    __shared__ uint32_t lds4[kRxWaves];
    __shared__ uint32_t skey[kRxTile], sval[kRxTile];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t base = (int64_t)blockIdx.x * kRxTile;
    const int64_t left = n - base;
    const uint32_t count = (uint32_t)(left < kRxTile ? left : kRxTile);
#pragma unroll
    for (int w = 0; w < kRxWaves; ++w) wave_count[w][tid] = 0;
    __syncthreads();

    uint32_t key[kRxIpt], val[kRxIpt], rank[kRxIpt];
    const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
    for (int j = 0; j < kRxIpt; ++j) {
        const uint32_t local = wave * (kWave * kRxIpt) + j * kWave + lane;
        const bool on = local < count;
        key[j] = 0;
        val[j] = 0;
        if (on) {
            const int64_t i = base + local;
            key[j] = FIRST ? radix_key((int32_t)keys_in[i], invalid_key) : keys_in[i];
            val[j] = FIRST ? (uint32_t)i : vals_in[i];
        }
        const uint32_t d = (key[j] >> shift) & 255u;
        // lanes of this wave that are active and hold the same digit
        uint64_t peers = __ballot(on);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const uint64_t vote = __ballot(on && ((d >> b) & 1u));
            peers &= ((d >> b) & 1u) ? vote : ~vote;
        }
        rank[j] = 0;
        if (on) {
            const int leader = __ffsll((long long)peers) - 1;
            uint32_t prev = 0;
            if (lane == leader) {
                prev = wave_count[wave][d];
                wave_count[wave][d] = prev + (uint32_t)__popcll(peers);
            }
            prev = __shfl(prev, leader, kWave);
            rank[j] = prev + (uint32_t)__popcll(peers & below);
        }
        // the next round reads the counters this round's leaders wrote (same wave: LDS ops of a
        // wave complete in order, no barrier needed)
    }
    __syncthreads();
    {   // thread d: waves in order -> start of every wave inside digit d, and the digit's total
        uint32_t off = 0;
#pragma unroll
        for (int w = 0; w < kRxWaves; ++w) {
            const uint32_t t = wave_count[w][tid];
            wave_count[w][tid] = off;
            off += t;
        }
        uint32_t total;
        digit_start[tid] = block_exclusive_scan(off, lds4, total);
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kRxIpt; ++j) {
        const uint32_t local = wave * (kWave * kRxIpt) + j * kWave + lane;
        if (local < count) {
            const uint32_t d = (key[j] >> shift) & 255u;
            const uint32_t p = digit_start[d] + wave_count[wave][d] + rank[j];
            skey[p] = key[j];
            sval[p] = val[j];
        }
    }
    __syncthreads();
    for (uint32_t p = tid; p < count; p += kRxThreads) {
        const uint32_t k = skey[p];
        const uint32_t d = (k >> shift) & 255u;
        const int64_t g = (int64_t)hist[(int64_t)d * n_tiles + blockIdx.x] + (p - digit_start[d]);
        keys_out[g] = k;
        vals_out[g] = sval[p];
    }
}

// In-place exclusive prefix sum of a[0..len): chunk sums, the last workgroup scans them
// (and may publish the grand total), then every chunk is rescanned with its base.
template <bool TICKET>
__global__ void __launch_bounds__(kPgThreads)
scan_chunk_sums(const uint32_t* __restrict__ a, int64_t len, uint32_t* __restrict__ sums, uint32_t n_chunks,
                uint32_t* ticket, int64_t* total_out) {
    __shared__ uint32_t lds4[kPgThreads / kWave];
    __shared__ bool is_last;
    for (uint32_t chunk = blockIdx.x; chunk < n_chunks; chunk += gridDim.x) {
        const int64_t i0 = ((int64_t)chunk * kPgThreads + threadIdx.x) * kWordsPerThread;
        uint32_t s = 0;
#pragma unroll
        for (int k = 0; k < kWordsPerThread; ++k)
            if (i0 + k < len) s += a[i0 + k];
        uint32_t total;
        (void)block_exclusive_scan(s, lds4, total);
        if (threadIdx.x == 0)
            __hip_atomic_store(&sums[chunk], total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (!TICKET) return;      // many chunks: bitmap_scan_sums scans the sums in a launch of its own
    if (threadIdx.x == 0) {
        __threadfence();
        is_last = (atomicAdd(ticket, 1u) == gridDim.x - 1);
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();
    uint32_t carry = 0;
    for (uint32_t b0 = 0; b0 < n_chunks; b0 += kPgThreads) {
        const uint32_t b = b0 + threadIdx.x;
        const uint32_t x = b < n_chunks ? __hip_atomic_load(&sums[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
        uint32_t tot;
        const uint32_t ex = block_exclusive_scan(x, lds4, tot);
        if (b < n_chunks) sums[b] = carry + ex;
        carry += tot;
    }
    if (threadIdx.x == 0) {
        *ticket = 0u;   // ready for the next scan on this stream
        if (total_out != nullptr) *total_out = (int64_t)carry;
    }
}

__global__ void __launch_bounds__(kPgThreads)
scan_apply(uint32_t* __restrict__ a, int64_t len, const uint32_t* __restrict__ sums) {
    __shared__ uint32_t lds4[kPgThreads / kWave];
    const int64_t i0 = ((int64_t)blockIdx.x * kPgThreads + threadIdx.x) * kWordsPerThread;
    uint32_t v[kWordsPerThread];
    uint32_t s = 0;
#pragma unroll
    for (int k = 0; k < kWordsPerThread; ++k) {
        v[k] = i0 + k < len ? a[i0 + k] : 0u;
        s += v[k];
    }
    uint32_t total;
    uint32_t run = sums[blockIdx.x] + block_exclusive_scan(s, lds4, total);
#pragma unroll
    for (int k = 0; k < kWordsPerThread; ++k) {
        if (i0 + k < len) a[i0 + k] = run;
        run += v[k];
    }
}

__global__ void __launch_bounds__(kPgThreads)
radix_head_flags(const uint32_t* __restrict__ keys, int64_t n, uint32_t invalid_key, uint32_t* __restrict__ flags,
                 uint32_t* ticket) {
    const int64_t i = (int64_t)blockIdx.x * kPgThreads + threadIdx.x;
    if (i == 0) *ticket = 0u;
    if (i < n) {
        const uint32_t k = keys[i];
        flags[i] = (k < invalid_key && (i == 0 || keys[i - 1] != k)) ? 1u : 0u;
    }
}

__global__ void __launch_bounds__(kPgThreads)
radix_emit(const uint32_t* __restrict__ keys, const uint32_t* __restrict__ vals, const uint32_t* __restrict__ excl,
           int64_t n, uint32_t invalid_key, int32_t* __restrict__ uniq, int32_t* __restrict__ remap) {
    const int64_t i = (int64_t)blockIdx.x * kPgThreads + threadIdx.x;
    if (i >= n) return;
    const uint32_t k = keys[i];
    if (k >= invalid_key) {
        remap[vals[i]] = -1;
        return;
    }
    const bool head = i == 0 || keys[i - 1] != k;
    const uint32_t e = excl[i];                 // heads strictly before i
    if (head) uniq[e] = (int32_t)k;
    remap[vals[i]] = (int32_t)(head ? e : e - 1);
}

__global__ void set_count_zero(int64_t* n_uniq) { *n_uniq = 0; }

static hopgnn_status scan_in_place(uint32_t* a, int64_t len, const RadixWs& L, int64_t* total_out, hipStream_t s) {
    const int64_t n_chunks = ceil_div(len, kWordsPerBlock);
    const dim3 grid((unsigned)(n_chunks < 1024 ? n_chunks : 1024));
    if (n_chunks <= kTicketChunks) {
        hipLaunchKernelGGL(scan_chunk_sums<true>, grid, dim3(kPgThreads), 0, s, a, len, L.sums, (uint32_t)n_chunks,
                           L.ticket, total_out);
        HOPGNN_LAUNCH_CHECK();
    } else {
        hipLaunchKernelGGL(scan_chunk_sums<false>, grid, dim3(kPgThreads), 0, s, a, len, L.sums, (uint32_t)n_chunks,
                           L.ticket, total_out);
        HOPGNN_LAUNCH_CHECK();
        hipLaunchKernelGGL(bitmap_scan_sums, dim3(1), dim3(kPgThreads), 0, s, L.sums, (uint32_t)n_chunks, total_out);
        HOPGNN_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(scan_apply, dim3((unsigned)n_chunks), dim3(kPgThreads), 0, s, a, len, L.sums);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

static hopgnn_status pregather_radix(const int32_t* ids, int64_t n_ids, int64_t n_vertices, int32_t* uniq,
                                     int64_t* n_uniq_dev, int32_t* remap, void* ws, size_t ws_bytes,
                                     hipStream_t s) {
    const RadixWs L = radix_layout(ws, n_ids);
    if (ws_bytes < L.bytes) return HOPGNN_ENOMEM_WS;
    if (n_ids == 0) {
        hipLaunchKernelGGL(set_count_zero, dim3(1), dim3(1), 0, s, n_uniq_dev);
        HOPGNN_LAUNCH_CHECK();
        return HOPGNN_OK;
    }
    int bits = 0;
    while (bits < 31 && ((int64_t)1 << bits) < n_vertices) ++bits;   // ids < 2^bits
    const uint32_t invalid_key = 1u << bits;
    const int passes = (bits + 1 + 7) / 8;
    const uint32_t n_tiles = (uint32_t)L.n_tiles;
    const int64_t n_blocks_1d = ceil_div(n_ids, kPgThreads);

    // the ticket is zeroed by radix_head_flags' counterpart below on every call; the first scan of
    // this call needs it zero too
    hipLaunchKernelGGL(set_count_zero, dim3(1), dim3(1), 0, s, reinterpret_cast<int64_t*>(L.ticket));
    HOPGNN_LAUNCH_CHECK();
    int cur = 0;
    for (int p = 0; p < passes; ++p) {
        const int shift = 8 * p;
        const uint32_t* kin = p == 0 ? reinterpret_cast<const uint32_t*>(ids) : L.keys[cur];
        const uint32_t* vin = p == 0 ? nullptr : L.vals[cur];
        if (p == 0)
            hipLaunchKernelGGL(radix_histogram<true>, dim3(n_tiles), dim3(kRxThreads), 0, s, kin, n_ids, shift,
                               invalid_key, L.hist, n_tiles);
        else
            hipLaunchKernelGGL(radix_histogram<false>, dim3(n_tiles), dim3(kRxThreads), 0, s, kin, n_ids, shift,
                               invalid_key, L.hist, n_tiles);
        HOPGNN_LAUNCH_CHECK();
        hopgnn_status st = scan_in_place(L.hist, 256 * (int64_t)n_tiles, L, nullptr, s);
        if (st != HOPGNN_OK) return st;
        const int nxt = p == 0 ? 0 : cur ^ 1;
        if (p == 0)
            hipLaunchKernelGGL(radix_scatter<true>, dim3(n_tiles), dim3(kRxThreads), 0, s, kin, vin, n_ids, shift,
                               invalid_key, L.hist, n_tiles, L.keys[nxt], L.vals[nxt]);
        else
            hipLaunchKernelGGL(radix_scatter<false>, dim3(n_tiles), dim3(kRxThreads), 0, s, kin, vin, n_ids, shift,
                               invalid_key, L.hist, n_tiles, L.keys[nxt], L.vals[nxt]);
        HOPGNN_LAUNCH_CHECK();
        cur = nxt;
    }
    hipLaunchKernelGGL(radix_head_flags, dim3((unsigned)n_blocks_1d), dim3(kPgThreads), 0, s, L.keys[cur], n_ids,
                       invalid_key, L.flags, L.ticket);
    HOPGNN_LAUNCH_CHECK();
    hopgnn_status st = scan_in_place(L.flags, n_ids, L, n_uniq_dev, s);
    if (st != HOPGNN_OK) return st;
    hipLaunchKernelGGL(radix_emit, dim3((unsigned)n_blocks_1d), dim3(kPgThreads), 0, s, L.keys[cur], L.vals[cur],
                       L.flags, n_ids, invalid_key, uniq, remap);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

// --------------------------------------------------------- locality statistics --

constexpr int kLocThreads = 256;
constexpr int32_t kLocEmpty = -1;

// One workgroup per micrograph: its slots are inserted into an open-addressing hash set in
// LDS (atomicCAS); the thread that claims a free cell has found a new distinct vertex.
__global__ void __launch_bounds__(kLocThreads)
micrograph_locality(const int32_t* __restrict__ ids, int32_t n_seeds, SlotShape sh,
                    const int32_t* __restrict__ owner, uint32_t table_mask, int32_t* __restrict__ n_total,
                    int32_t* __restrict__ n_coloc) {
    extern __shared__ int32_t table[];
    __shared__ uint32_t lds4[kLocThreads / kWave];
    const int32_t m = blockIdx.x;
    for (uint32_t i = threadIdx.x; i <= table_mask; i += kLocThreads) table[i] = kLocEmpty;
    __syncthreads();
    const int32_t root = ids[m];
    if (root < 0) {            // no root, no micrograph (uniform over the workgroup)
        if (threadIdx.x == 0) n_total[m] = n_coloc[m] = 0;
        return;
    }
    const int32_t root_home = owner[root];
    uint32_t tot = 0, col = 0;
    for (int32_t h = 0; h <= sh.n_layers; ++h) {
        const int32_t* lvl = ids + sh.base[h] + (int64_t)m * sh.P[h];
        for (int32_t p = threadIdx.x; p < sh.P[h]; p += kLocThreads) {
            const int32_t v = lvl[p];
            if (v < 0) continue;
            uint32_t cell = ((uint32_t)v * 2654435761u) & table_mask;
            while (true) {     // ends: the table has more cells than a micrograph has slots
                const int32_t old = atomicCAS(&table[cell], kLocEmpty, v);
                if (old == kLocEmpty) {   // first time this vertex is seen in the micrograph
                    ++tot;
                    if (v != root && owner[v] == root_home) ++col;
                    break;
                }
                if (old == v) break;
                cell = (cell + 1) & table_mask;
            }
        }
    }
    uint32_t t_all, c_all;
    (void)block_exclusive_scan(tot, lds4, t_all);
    (void)block_exclusive_scan(col, lds4, c_all);
    if (threadIdx.x == 0) {
        n_total[m] = (int32_t)t_all;
        n_coloc[m] = (int32_t)c_all;
    }
}

__global__ void __launch_bounds__(kPgThreads)
owner_flags(const int32_t* __restrict__ uniq, int64_t n_host, const int64_t* __restrict__ n_dev,
            const int32_t* __restrict__ owner, int32_t server, uint32_t* __restrict__ flags, uint32_t* ticket) {
    const int64_t i = (int64_t)blockIdx.x * kPgThreads + threadIdx.x;
    if (i == 0) *ticket = 0u;
    if (i >= n_host) return;
    int64_t n = n_host;
    if (n_dev != nullptr) n = *n_dev < n ? *n_dev : n;
    flags[i] = (i < n && owner[uniq[i]] != server) ? 1u : 0u;
}

__global__ void __launch_bounds__(kPgThreads)
owner_compact(const int32_t* __restrict__ uniq, int64_t n_host, const int64_t* __restrict__ n_dev,
              const int32_t* __restrict__ owner, int32_t server, const uint32_t* __restrict__ excl,
              int32_t* __restrict__ remote) {
    const int64_t i = (int64_t)blockIdx.x * kPgThreads + threadIdx.x;
    int64_t n = n_host;
    if (n_dev != nullptr) n = *n_dev < n ? *n_dev : n;
    if (i >= n) return;
    const int32_t v = uniq[i];
    if (owner[v] != server) remote[excl[i]] = v;
}

struct SplitWs {
    uint32_t *flags, *sums, *ticket;
    size_t bytes;
};
static SplitWs split_layout(void* ws, int64_t n_uniq) {
    SplitWs L{};
    const int64_t n = n_uniq > 0 ? n_uniq : 1;
    char* p = static_cast<char*>(ws);
    size_t o = 0;
    L.flags = reinterpret_cast<uint32_t*>(p + o);
    o += align_up((size_t)n * 4, 256);
    L.sums = reinterpret_cast<uint32_t*>(p + o);
    o += align_up((size_t)ceil_div(n, kWordsPerBlock) * 4, 256);
    L.ticket = reinterpret_cast<uint32_t*>(p + o);
    o += 256;
    L.bytes = o;
    return L;
}

}  // namespace hopgnn

using namespace hopgnn;

// The bitmap path costs ~0.6 us per million vertices (it packs and ranks the whole vertex range)
// plus ~25 us per million slots, the radix path ~90 us of launches plus ~50 us per million slots.
// Measured on MI355X (us, bitmap vs radix): 0.11 M slots / 1 M vertices 21 vs 75; 0.94 M / 2.4 M 41 vs
// 105; 4.55 M / 100 M 208 vs 310; 0.57 M / 100 M 67 vs 117; 0.26 M / 100 M 59 vs 103; 0.26 M / 1500 M
// 950 vs 105.  AUTO takes the sort where that model says it is cheaper.
static int32_t pick_algo(int32_t algo, int64_t n_ids, int64_t n_vertices) {
    if (algo != HOPGNN_PG_AUTO) return algo;
    return n_vertices > 133000000 + 42 * n_ids ? HOPGNN_PG_RADIX : HOPGNN_PG_BITMAP;
}

namespace hopgnn {

uint8_t* pregather_marks_map(void* ws, size_t ws_bytes, int64_t n_ids, int64_t n_vertices, int32_t algo) {
    if (ws == nullptr || !aligned(ws, 256) || n_ids < 0 || n_vertices < 0) return nullptr;
    if (pick_algo(algo, n_ids, n_vertices) != HOPGNN_PG_BITMAP) return nullptr;
    const BitmapWs L = bitmap_layout(ws, n_vertices);
    return ws_bytes >= L.bytes ? L.present : nullptr;
}

hopgnn_status pregather_from_marks(const int32_t* ids, int64_t n_ids, int64_t n_vertices, int32_t* uniq,
                                   int64_t* n_uniq_dev, int32_t* remap, void* ws, size_t ws_bytes, hipStream_t s) {
    if (n_ids < 0 || n_vertices < 0 || n_uniq_dev == nullptr || ws == nullptr) return HOPGNN_EINVAL;
    if (n_ids > 0 && (ids == nullptr || remap == nullptr || uniq == nullptr)) return HOPGNN_EINVAL;
    if (n_ids >= ((int64_t)1 << 31) || n_vertices > ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    const BitmapWs L = bitmap_layout(ws, n_vertices);
    if (ws_bytes < L.bytes) return HOPGNN_ENOMEM_WS;
    return bitmap_from_marks(L, true, ids, n_ids, uniq, n_uniq_dev, remap, s);
}

}  // namespace hopgnn

extern "C" hopgnn_status hopgnn_pregather_ws_init(void* ws, size_t ws_bytes, int64_t n_ids, int64_t n_vertices,
                                                  int32_t algo, void* stream) {
    if (ws == nullptr || n_ids < 0 || n_vertices < 0 || !aligned(ws, 256)) return HOPGNN_EINVAL;
    if (algo != HOPGNN_PG_AUTO && algo != HOPGNN_PG_BITMAP && algo != HOPGNN_PG_RADIX) return HOPGNN_EINVAL;
    if (pick_algo(algo, n_ids, n_vertices) == HOPGNN_PG_RADIX)
        return ws_bytes >= radix_layout(nullptr, n_ids).bytes ? HOPGNN_OK : HOPGNN_ENOMEM_WS;   // nothing to prepare
    const BitmapWs L = bitmap_layout(ws, n_vertices);
    if (ws_bytes < L.bytes) return HOPGNN_ENOMEM_WS;
    const int64_t n_vec = L.n_words_padded * 2;
    hipLaunchKernelGGL(present_clear, dim3(grid_for(n_vec, kPgThreads, 256 * 16)), dim3(kPgThreads), 0,
                       static_cast<hipStream_t>(stream), reinterpret_cast<uint4*>(L.present), n_vec, L.ticket,
                       static_cast<int64_t*>(nullptr));
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

extern "C" size_t hopgnn_pregather_ws_bytes(int64_t n_ids, int64_t n_vertices, int32_t algo) {
    if (n_ids < 0 || n_vertices < 0) return 0;
    if (pick_algo(algo, n_ids, n_vertices) == HOPGNN_PG_RADIX) return radix_layout(nullptr, n_ids).bytes;
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
    if (pick_algo(algo, n_ids, n_vertices) == HOPGNN_PG_RADIX)
        return pregather_radix(ids, n_ids, n_vertices, uniq, n_uniq_dev, remap, ws, ws_bytes,
                               static_cast<hipStream_t>(stream));
    return pregather_bitmap(ids, n_ids, n_vertices, uniq, n_uniq_dev, remap, ws, ws_bytes,
                            static_cast<hipStream_t>(stream));
}

// ---------------------------------------------------- no-allocation entry point --
//
// hopgnn_pregather for callers that cannot allocate or hand over a workspace: the bitmap path's
// scratch lives in a file-scope device array.  In host code the array's name is only a stand-in;
// its address on the current device comes from hipGetSymbolAddress, once per device.

constexpr int64_t kStaticMaxVertices = (int64_t)1 << 24;
constexpr size_t kStaticScratchBytes = (size_t)24 << 20;   // presence bytes + word ranks + chunk sums for 2^24 vertices
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kStaticMaxDevices = 64;
static void* g_scratch_ptr[kStaticMaxDevices];             // per device: where that device's copy of `scratch` lives
static std::mutex g_scratch_mutex;

static hopgnn_status static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kStaticMaxDevices) return HOPGNN_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return HOPGNN_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return HOPGNN_OK;
}

extern "C" int64_t hopgnn_pregather_static_max_vertices(void) { return kStaticMaxVertices; }

extern "C" hopgnn_status hopgnn_pregather_static(const int32_t* ids, int64_t n_ids, int64_t n_vertices, int32_t* uniq,
                                                 int64_t* n_uniq_dev, int32_t* remap, void* stream) {
    if (n_ids < 0 || n_vertices < 0 || n_uniq_dev == nullptr) return HOPGNN_EINVAL;
    if (n_ids > 0 && (ids == nullptr || remap == nullptr || uniq == nullptr)) return HOPGNN_EINVAL;
    if (n_ids >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    if (n_vertices > kStaticMaxVertices) return HOPGNN_ERANGE;          // beyond the static scratch
    if (bitmap_layout(nullptr, n_vertices).bytes > kStaticScratchBytes) return HOPGNN_ERANGE;
    void* ws = nullptr;
    const hopgnn_status st = static_scratch(&ws);
    if (st != HOPGNN_OK) return st;
    // the bitmap path clears the part of the scratch it uses before marking, so whatever the last
    // call on this device left there does not matter
    return pregather_bitmap(ids, n_ids, n_vertices, uniq, n_uniq_dev, remap, ws, kStaticScratchBytes,
                            static_cast<hipStream_t>(stream));
}

extern "C" hopgnn_status hopgnn_micrograph_locality(const int32_t* ids, int32_t n_seeds, const int32_t* fanouts,
                                                    int32_t n_layers, const int32_t* owner, int32_t* n_total,
                                                    int32_t* n_coloc, void* stream) {
    if (fanouts == nullptr || n_seeds < 0 || n_layers < 1 || n_layers > kMaxLayers) return HOPGNN_EINVAL;
    SlotShape sh{};
    sh.n_layers = n_layers;
    sh.P[0] = 1;
    sh.base[0] = 0;
    int64_t t_seed = 1;
    for (int32_t h = 1; h <= n_layers; ++h) {
        if (fanouts[h - 1] < 1) return HOPGNN_EINVAL;
        const int64_t p = (int64_t)sh.P[h - 1] * fanouts[h - 1];
        t_seed += p;
        if (t_seed > 16384) return HOPGNN_ERANGE;   // hash set of 2*T_seed cells must fit 160 KB of LDS
        sh.P[h] = (int32_t)p;
    }
    if (n_seeds == 0) return HOPGNN_OK;
    if (ids == nullptr || owner == nullptr || n_total == nullptr || n_coloc == nullptr) return HOPGNN_EINVAL;
    if ((int64_t)n_seeds * t_seed >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    for (int32_t h = 1; h <= n_layers + 1; ++h) sh.base[h] = sh.base[h - 1] + n_seeds * sh.P[h - 1];
    uint32_t cells = 64;
    while (cells < 2 * (uint32_t)t_seed) cells *= 2;   // load factor <= 1/2
    const size_t lds = (size_t)cells * 4;
    if (lds > 64 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(micrograph_locality),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return HOPGNN_EHIP;
    hipLaunchKernelGGL(micrograph_locality, dim3(n_seeds), dim3(kLocThreads), lds, static_cast<hipStream_t>(stream),
                       ids, n_seeds, sh, owner, cells - 1, n_total, n_coloc);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

extern "C" size_t hopgnn_split_ws_bytes(int64_t n_uniq) {
    if (n_uniq < 0) return 0;
    return split_layout(nullptr, n_uniq).bytes;
}

extern "C" hopgnn_status hopgnn_split_by_owner(const int32_t* uniq, int64_t n_uniq, const int64_t* n_uniq_dev,
                                               const int32_t* owner, int32_t server, int32_t* remote,
                                               int64_t* n_remote_dev, void* ws, size_t ws_bytes, void* stream) {
    if (n_uniq < 0 || n_remote_dev == nullptr || ws == nullptr || !aligned(ws, 256)) return HOPGNN_EINVAL;
    if (n_uniq >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n_uniq == 0) {
        hipLaunchKernelGGL(set_count_zero, dim3(1), dim3(1), 0, s, n_remote_dev);
        HOPGNN_LAUNCH_CHECK();
        return HOPGNN_OK;
    }
    if (uniq == nullptr || owner == nullptr || remote == nullptr) return HOPGNN_EINVAL;
    const SplitWs L = split_layout(ws, n_uniq);
    if (ws_bytes < L.bytes) return HOPGNN_ENOMEM_WS;
    const unsigned blocks = (unsigned)ceil_div(n_uniq, kPgThreads);
    hipLaunchKernelGGL(owner_flags, dim3(blocks), dim3(kPgThreads), 0, s, uniq, n_uniq, n_uniq_dev, owner, server,
                       L.flags, L.ticket);
    HOPGNN_LAUNCH_CHECK();
    const int64_t n_chunks = ceil_div(n_uniq, kWordsPerBlock);
    const dim3 scan_grid((unsigned)(n_chunks < 1024 ? n_chunks : 1024));
    if (n_chunks <= kTicketChunks) {
        hipLaunchKernelGGL(scan_chunk_sums<true>, scan_grid, dim3(kPgThreads), 0, s, L.flags, n_uniq, L.sums,
                           (uint32_t)n_chunks, L.ticket, n_remote_dev);
        HOPGNN_LAUNCH_CHECK();
    } else {
        hipLaunchKernelGGL(scan_chunk_sums<false>, scan_grid, dim3(kPgThreads), 0, s, L.flags, n_uniq, L.sums,
                           (uint32_t)n_chunks, L.ticket, n_remote_dev);
        HOPGNN_LAUNCH_CHECK();
        hipLaunchKernelGGL(bitmap_scan_sums, dim3(1), dim3(kPgThreads), 0, s, L.sums, (uint32_t)n_chunks, n_remote_dev);
        HOPGNN_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(scan_apply, dim3((unsigned)n_chunks), dim3(kPgThreads), 0, s, L.flags, n_uniq, L.sums);
    HOPGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(owner_compact, dim3(blocks), dim3(kPgThreads), 0, s, uniq, n_uniq, n_uniq_dev, owner, server,
                       L.flags, remote);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}
