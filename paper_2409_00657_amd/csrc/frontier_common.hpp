// Device helpers shared by the per-micrograph frontier samplers (one workgroup per micrograph):
// the hash finaliser, workgroup prefix sums, an LDS bitonic sort and the packing of distinct values.
#pragma once
#include "common.hpp"

namespace hopgnn {

constexpr uint32_t kFrNone = 0xFFFFFFFFu;      // "no vertex": sorts after every vertex id

__host__ __device__ __forceinline__ uint64_t fr_finalise64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ uint32_t fr_shfl_up(uint32_t x, int d) { return __shfl_up(x, d, kWave); }
__device__ __forceinline__ uint64_t fr_shfl_up(uint64_t x, int d) {
    const uint32_t lo = __shfl_up((uint32_t)x, d, kWave), hi = __shfl_up((uint32_t)(x >> 32), d, kWave);
    return ((uint64_t)hi << 32) | lo;
}

// Exclusive prefix sum of one value per thread over a workgroup of THREADS; `total` = their sum.
// lds needs THREADS / 64 elements; every thread of the workgroup must call it.
template <int THREADS, typename T>
__device__ __forceinline__ T fr_block_scan(T x, T* lds, T& total) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    T inc = x;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const T y = fr_shfl_up(inc, d);
        if (lane >= d) inc += y;
    }
    if (lane == kWave - 1) lds[wave] = inc;
    __syncthreads();
    T wave_base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < THREADS / kWave; ++w) {
        const T s = lds[w];
        if (w < wave) wave_base += s;
        tot += s;
    }
    __syncthreads();
    total = tot;
    return wave_base + inc - x;
}

// Ascending bitonic sort of a[0, n2) in LDS, n2 a power of two; the caller has synchronised after
// filling a, and the sort ends synchronised.
template <int THREADS>
__device__ __forceinline__ void fr_bitonic_sort(uint32_t* a, uint32_t n2) {
    const uint32_t tid = threadIdx.x;
    for (uint32_t k = 2; k <= n2; k <<= 1)
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            for (uint32_t i = tid; i < n2; i += THREADS) {
                const uint32_t p = i ^ j;
                if (p > i) {
                    const uint32_t x = a[i], y = a[p];
                    if ((x > y) == ((i & k) == 0)) {
                        a[i] = y;
                        a[p] = x;
                    }
                }
            }
            __syncthreads();
        }
}

// The distinct values of the sorted srt[0, n2) other than kFrNone, packed in order into out (which
// must not alias srt); returns their number to every thread.  lds4: THREADS / 64 words.
template <int THREADS>
__device__ __forceinline__ uint32_t fr_pack_distinct(const uint32_t* srt, uint32_t n2, uint32_t* out, uint32_t* lds4) {
    const uint32_t tid = threadIdx.x;
    uint32_t carry = 0;
    for (uint32_t i0 = 0; i0 < n2; i0 += THREADS) {
        const uint32_t i = i0 + tid;
        const uint32_t v = i < n2 ? srt[i] : kFrNone;
        const uint32_t head = (v != kFrNone && (i == 0 || srt[i - 1] != v)) ? 1u : 0u;
        uint32_t total;
        const uint32_t pos = carry + fr_block_scan<THREADS, uint32_t>(head, lds4, total);
        if (head) out[pos] = v;
        carry += total;
    }
    __syncthreads();
    return carry;
}

// First position in the ascending a[0, n) whose value is not below x.
__device__ __forceinline__ uint32_t fr_lower_bound(const uint32_t* a, uint32_t n, uint32_t x) {
    uint32_t lo = 0, hi = n;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (a[mid] < x) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

}  // namespace hopgnn
