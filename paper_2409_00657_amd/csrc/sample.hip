// hopgnn_sample: counter-hash k-hop sampling, one micrograph per root vertex
// (paper section 2 "sampling", section 4 "micrograph definition").
//
// One workgroup owns one micrograph and walks its levels in order; a level is
// written to HBM (coalesced inside the micrograph's slice of the level-major
// array) and read back by the same workgroup after a barrier, so all hops of
// all micrographs run in a single launch.  Work per slot is two dependent
// random reads (row bounds, then one neighbour) - latency bound, hidden by
// keeping every micrograph's workgroup resident at once.
#include <type_traits>

#include "pregather_internal.hpp"

namespace hopgnn {

struct SampleShape {
    int32_t n_layers;
    int32_t f[kMaxLayers + 1];      // f[h], h = 1..L
    int32_t P[kMaxLayers + 1];      // P[h] = slots per micrograph at level h
    int32_t base[kMaxLayers + 2];   // base[h] = first slot of level h; base[L+1] = T
};

__device__ __forceinline__ uint64_t finalise64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Exact unsigned 64-bit remainder (a multiply-high range reduction would pick
// different neighbours and is not an acceptable substitute).
__device__ __forceinline__ uint64_t mod_u64(uint64_t x, uint64_t d) {
    return x % d;
}

// Batches sampled by one launch: blockIdx.y picks the batch, i.e. its seeds, its key (first
// hash round already applied on the host) and its slice of the outputs.
constexpr int kMaxBatchesPerLaunch = 64;
struct BatchKeys {
    uint64_t keyed[kMaxBatchesPerLaunch];
};

constexpr int kSampleUnroll = 4;

template <typename OffT>
__global__ void __launch_bounds__(256)
sample_micrographs(const OffT* __restrict__ offsets, const int32_t* __restrict__ indices,
                   const int32_t* __restrict__ seeds, int32_t n_seeds, SampleShape sh,
                   BatchKeys keys, int32_t* ids, int32_t* indptr, int32_t* slot_idx, int64_t slot_idx_stride,
                   uint8_t* __restrict__ present, int32_t m_offset, int32_t seeds_per_key, int32_t has_edges) {
    // Two ways to carry several keys: blockIdx.y = one batch (own seeds, key and output slices) of
    // n_seeds micrographs each, or ONE level-major batch whose micrographs m_offset + blockIdx.x
    // take the key of their block of seeds_per_key consecutive seeds (then gridDim.y = 1).
    const int32_t m = m_offset + (int32_t)blockIdx.x;
    const int32_t B = n_seeds;
    const uint32_t batch = blockIdx.y;
    const uint64_t keyed = keys.keyed[batch + blockIdx.x / (uint32_t)seeds_per_key];
    seeds += (int64_t)batch * B;
    ids += (int64_t)batch * sh.base[sh.n_layers + 1];
    if (slot_idx != nullptr) slot_idx += (int64_t)batch * slot_idx_stride;
    if (batch != 0) indptr = nullptr;      // the segment offsets are the same for every batch of one shape
    const int32_t root = seeds[m];
    if (threadIdx.x == 0) {
        ids[m] = root;
        if (present != nullptr && root >= 0) present[root] = 1;   // the pre-gather's presence map
        if (indptr != nullptr && m == 0) indptr[sh.base[sh.n_layers]] = sh.base[sh.n_layers + 1] - B;
    }
    for (int32_t h = 1; h <= sh.n_layers; ++h) {
        const uint32_t f = sh.f[h];
        const int32_t P = sh.P[h];
        const int32_t* parents = ids + sh.base[h - 1] + (int64_t)m * sh.P[h - 1];
        int32_t* children = ids + sh.base[h] + (int64_t)m * P;
        // Several slots per thread and round: every slot is a chain of dependent random reads
        // (parent, its two row bounds, one neighbour), so the chains of a round are issued side by
        // side - all bounds, then all neighbours - instead of one after the other.  Loads are
        // unconditional from clamped, in-bounds addresses; what must not count is masked afterwards.
        auto level = [&](auto unroll) {
        constexpr int U = decltype(unroll)::value;
        for (uint32_t c0 = threadIdx.x; c0 < (uint32_t)P; c0 += blockDim.x * U) {
            uint32_t q[U], j[U];
            int32_t v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t c = c0 + u * blockDim.x;
                const uint32_t cc = c < (uint32_t)P ? c : 0u;
                q[u] = cc / f;
                j[u] = cc - q[u] * f;
                v[u] = (h == 1) ? root : parents[q[u]];
                if (c >= (uint32_t)P) v[u] = -1;
            }
            int64_t o0[U], deg[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t vv = v[u] >= 0 ? v[u] : 0;
                o0[u] = has_edges ? (int64_t)offsets[vv] : 0;             // no edges: no vertex has a row to read
                deg[u] = has_edges ? (int64_t)offsets[vv + 1] - o0[u] : 0;
                if (v[u] < 0) deg[u] = 0;
            }
            int32_t child[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint64_t x = finalise64((keyed ^ (((uint64_t)(uint32_t)root << 32) | (uint32_t)v[u])) +
                                        0x9E3779B97F4A7C15ull);
                x = finalise64((x ^ (((uint64_t)(uint32_t)h << 32) | j[u])) + 0x9E3779B97F4A7C15ull);
                const int64_t e = deg[u] > 0 ? o0[u] + (int64_t)mod_u64(x, (uint64_t)deg[u]) : 0;
                child[u] = has_edges ? indices[e] : -1;
                if (deg[u] <= 0) child[u] = -1;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t c = c0 + u * blockDim.x;
                if (c >= (uint32_t)P) continue;
                children[c] = child[u];
                if (present != nullptr && child[u] >= 0) present[child[u]] = 1;
                if (slot_idx != nullptr && h < sh.n_layers) {   // non-leaf child: its own row in later layers
                    const int32_t slot = sh.base[h] + m * P + (int32_t)c;
                    slot_idx[slot - B] = child[u] >= 0 ? slot : -1;
                }
                if (indptr != nullptr && j[u] == 0)
                    indptr[sh.base[h - 1] + m * sh.P[h - 1] + (int32_t)q[u]] =
                        sh.base[h] + (m * sh.P[h - 1] + (int32_t)q[u]) * (int32_t)f - B;
            }
        }
        };
        // a level no wider than the workgroup has one slot per thread: nothing to batch
        if ((uint32_t)P > blockDim.x) level(std::integral_constant<int, kSampleUnroll>{});
        else level(std::integral_constant<int, 1>{});
        __syncthreads();   // this level is visible to the whole workgroup before the next hop
    }
}

static uint64_t host_finalise64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

}  // namespace hopgnn

using namespace hopgnn;

extern "C" int64_t hopgnn_slots_per_seed(const int32_t* fanouts, int32_t n_layers) {
    if (fanouts == nullptr || n_layers < 1 || n_layers > kMaxLayers) return -1;
    int64_t p = 1, t = 1;
    for (int32_t h = 0; h < n_layers; ++h) {
        if (fanouts[h] < 1) return -1;
        p *= fanouts[h];
        if (p > (int64_t)1 << 31) return -1;
        t += p;
    }
    return t;
}

namespace hopgnn {

hopgnn_status sample_batches(const hopgnn_csr* g, const int32_t* seeds, int32_t n_seeds, const int32_t* fanouts,
                             int32_t n_layers, const uint64_t* keys, int32_t n_batches, int32_t* ids, int32_t* indptr,
                             int32_t* slot_idx, int64_t slot_idx_stride, uint8_t* present, void* stream) {
    if (g == nullptr || fanouts == nullptr || n_seeds < 0 || n_batches < 0) return HOPGNN_EINVAL;
    const int64_t t_seed = hopgnn_slots_per_seed(fanouts, n_layers);
    if (t_seed < 0) return HOPGNN_EINVAL;
    if (g->n_vertices < 0 || g->n_edges < 0 || g->n_vertices > ((int64_t)1 << 31)) return HOPGNN_EINVAL;
    if (n_seeds == 0 || n_batches == 0) return HOPGNN_OK;
    if (g->offsets == nullptr || seeds == nullptr || ids == nullptr || keys == nullptr) return HOPGNN_EINVAL;
    if (g->n_edges > 0 && g->indices == nullptr) return HOPGNN_EINVAL;
    const int64_t T = (int64_t)n_seeds * t_seed;
    if (T * n_batches >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;

    SampleShape sh{};
    sh.n_layers = n_layers;
    sh.P[0] = 1;
    sh.base[0] = 0;
    for (int32_t h = 1; h <= n_layers; ++h) {
        sh.f[h] = fanouts[h - 1];
        sh.P[h] = sh.P[h - 1] * sh.f[h];
        sh.base[h] = sh.base[h - 1] + n_seeds * sh.P[h - 1];
    }
    sh.base[n_layers + 1] = sh.base[n_layers] + n_seeds * sh.P[n_layers];
    if (slot_idx != nullptr && n_batches > 1 && slot_idx_stride < (int64_t)sh.base[n_layers] - n_seeds)
        return HOPGNN_EINVAL;              // the batches' neighbour lists would overlap

    int threads = 64;
    while (threads < 256 && threads < sh.P[n_layers]) threads *= 2;
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int32_t b0 = 0; b0 < n_batches; b0 += kMaxBatchesPerLaunch) {
        const int32_t nb = n_batches - b0 < kMaxBatchesPerLaunch ? n_batches - b0 : kMaxBatchesPerLaunch;
        BatchKeys bk{};
        for (int32_t i = 0; i < nb; ++i) bk.keyed[i] = host_finalise64(keys[b0 + i] + 0x9E3779B97F4A7C15ull);
        const int32_t* sd = seeds + (int64_t)b0 * n_seeds;
        int32_t* id = ids + (int64_t)b0 * T;
        int32_t* ip = b0 == 0 ? indptr : nullptr;
        int32_t* si = slot_idx != nullptr ? slot_idx + (int64_t)b0 * slot_idx_stride : nullptr;
        const dim3 grid((unsigned)n_seeds, (unsigned)nb);
        if (g->offsets_i64)
            hipLaunchKernelGGL(sample_micrographs<int64_t>, grid, dim3(threads), 0, s,
                               static_cast<const int64_t*>(g->offsets), g->indices, sd, n_seeds, sh, bk, id, ip, si,
                               slot_idx_stride, present, 0, n_seeds, g->n_edges > 0 ? 1 : 0);
        else
            hipLaunchKernelGGL(sample_micrographs<int32_t>, grid, dim3(threads), 0, s,
                               static_cast<const int32_t*>(g->offsets), g->indices, sd, n_seeds, sh, bk, id, ip, si,
                               slot_idx_stride, present, 0, n_seeds, g->n_edges > 0 ? 1 : 0);
        HOPGNN_LAUNCH_CHECK();
    }
    return HOPGNN_OK;
}

hopgnn_status sample_merged(const hopgnn_csr* g, const int32_t* seeds, int32_t n_seeds, int32_t seeds_per_key,
                            const int32_t* fanouts, int32_t n_layers, const uint64_t* keys, int32_t* ids,
                            int32_t* indptr, int32_t* slot_idx, uint8_t* present, void* stream) {
    if (g == nullptr || fanouts == nullptr || n_seeds < 0 || seeds_per_key < 1) return HOPGNN_EINVAL;
    const int64_t t_seed = hopgnn_slots_per_seed(fanouts, n_layers);
    if (t_seed < 0) return HOPGNN_EINVAL;
    if (g->n_vertices < 0 || g->n_edges < 0 || g->n_vertices > ((int64_t)1 << 31)) return HOPGNN_EINVAL;
    if (n_seeds == 0) return HOPGNN_OK;
    if (g->offsets == nullptr || seeds == nullptr || ids == nullptr || keys == nullptr) return HOPGNN_EINVAL;
    if (g->n_edges > 0 && g->indices == nullptr) return HOPGNN_EINVAL;
    if ((int64_t)n_seeds * t_seed >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;

    SampleShape sh{};
    sh.n_layers = n_layers;
    sh.P[0] = 1;
    sh.base[0] = 0;
    for (int32_t h = 1; h <= n_layers; ++h) {
        sh.f[h] = fanouts[h - 1];
        sh.P[h] = sh.P[h - 1] * sh.f[h];
        sh.base[h] = sh.base[h - 1] + n_seeds * sh.P[h - 1];
    }
    sh.base[n_layers + 1] = sh.base[n_layers] + n_seeds * sh.P[n_layers];
    int threads = 64;
    while (threads < 256 && threads < sh.P[n_layers]) threads *= 2;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int32_t n_keys = (int32_t)ceil_div(n_seeds, seeds_per_key);
    for (int32_t k0 = 0; k0 < n_keys; k0 += kMaxBatchesPerLaunch) {     // 64 keys fit one launch's arguments
        const int32_t nk = n_keys - k0 < kMaxBatchesPerLaunch ? n_keys - k0 : kMaxBatchesPerLaunch;
        BatchKeys bk{};
        for (int32_t i = 0; i < nk; ++i) bk.keyed[i] = host_finalise64(keys[k0 + i] + 0x9E3779B97F4A7C15ull);
        const int64_t m0 = (int64_t)k0 * seeds_per_key;
        const int64_t count = (int64_t)nk * seeds_per_key < n_seeds - m0 ? (int64_t)nk * seeds_per_key : n_seeds - m0;
        const dim3 grid((unsigned)count, 1u);
        if (g->offsets_i64)
            hipLaunchKernelGGL(sample_micrographs<int64_t>, grid, dim3(threads), 0, s,
                               static_cast<const int64_t*>(g->offsets), g->indices, seeds, n_seeds, sh, bk, ids, indptr,
                               slot_idx, (int64_t)0, present, (int32_t)m0, seeds_per_key, g->n_edges > 0 ? 1 : 0);
        else
            hipLaunchKernelGGL(sample_micrographs<int32_t>, grid, dim3(threads), 0, s,
                               static_cast<const int32_t*>(g->offsets), g->indices, seeds, n_seeds, sh, bk, ids, indptr,
                               slot_idx, (int64_t)0, present, (int32_t)m0, seeds_per_key, g->n_edges > 0 ? 1 : 0);
        HOPGNN_LAUNCH_CHECK();
    }
    return HOPGNN_OK;
}

}  // namespace hopgnn

extern "C" hopgnn_status hopgnn_sample_merged(const hopgnn_csr* g, const int32_t* seeds, int32_t n_seeds,
                                              int32_t seeds_per_key, const int32_t* fanouts, int32_t n_layers,
                                              const uint64_t* keys, int32_t* ids, int32_t* indptr, int32_t* slot_idx,
                                              void* stream) {
    return sample_merged(g, seeds, n_seeds, seeds_per_key, fanouts, n_layers, keys, ids, indptr, slot_idx, nullptr,
                         stream);
}

extern "C" hopgnn_status hopgnn_sample(const hopgnn_csr* g, const int32_t* seeds, int32_t n_seeds,
                                       const int32_t* fanouts, int32_t n_layers, uint64_t key,
                                       int32_t* ids, int32_t* indptr, int32_t* slot_idx,
                                       void* stream) {
    return sample_batches(g, seeds, n_seeds, fanouts, n_layers, &key, 1, ids, indptr, slot_idx, 0, nullptr, stream);
}

extern "C" hopgnn_status hopgnn_sample_group(const hopgnn_csr* g, const int32_t* seeds, int32_t n_seeds,
                                             const int32_t* fanouts, int32_t n_layers, const uint64_t* keys,
                                             int32_t n_batches, int32_t* ids, int32_t* indptr, int32_t* slot_idx,
                                             int64_t slot_idx_stride, void* stream) {
    return sample_batches(g, seeds, n_seeds, fanouts, n_layers, keys, n_batches, ids, indptr, slot_idx, slot_idx_stride,
                          nullptr, stream);
}

extern "C" const char* hopgnn_status_str(hopgnn_status s) {
    switch (s) {
        case HOPGNN_OK: return "ok";
        case HOPGNN_EINVAL: return "invalid argument";
        case HOPGNN_ENOMEM_WS: return "workspace too small";
        case HOPGNN_ERANGE: return "size out of range";
        case HOPGNN_EHIP: return "HIP launch failed";
    }
    return "unknown status";
}
