// hopgnn_sample_dedup: k-hop sampling with per-micrograph deduplicated frontiers.
//
// A micrograph is the set of vertices its sampling reaches (paper section 4, "micrograph
// definition", which counts distinct vertices).  The children a vertex draws depend only on
// (key, root, vertex, hop, j), so equal vertices at one level of one micrograph carry identical
// subtrees in the slot tree of hopgnn_sample; here every (level, vertex) pair of a micrograph is
// kept once.  The rows computed for the roots are the same, over fewer rows below them (on
// power-law graphs with replacement about half the valid slots of a level are repeats).
//
//   dedup_sample   one workgroup per micrograph: per hop it draws the children of the current
//                  distinct vertices into LDS, sorts them (bitonic, in LDS), keeps the distinct ones
//                  in ascending order and finds every child's position by binary search; node lists
//                  and child positions go to per-micrograph staging slices of slot-tree capacity
//   dedup_scan     exclusive sums of the per-micrograph node counts, level by level
//   dedup_compact  level-major global numbering: node vertices, CSR of child node indices
//                  (parallel edges kept, -1 where a vertex has no neighbours), unused tails filled
#include "frontier_common.hpp"
#include "pregather_internal.hpp"

namespace hopgnn {

constexpr int kDdThreads = 256;
constexpr int kDdMaxLevel = 4096;      // most slots one micrograph may have at one level
constexpr uint32_t kDdNone = kFrNone;
constexpr int kDdScanThreads = 1024;    // the one-workgroup scan of the node counts

constexpr int kDdKeysPerLaunch = 64;
struct DedupKeys {
    uint64_t keyed[kDdKeysPerLaunch];      // first hash round already applied on the host
};

struct DedupShape {
    int32_t n_layers;
    int32_t f[kMaxLayers + 1];      // f[h], h = 1..L
    int32_t P[kMaxLayers + 1];      // slot-tree slots per micrograph at level h
    int32_t base[kMaxLayers + 2];   // first slot of level h in the slot-tree layout; base[L+1] = T
};

// LDS (dynamic): three arrays of `cap` words, cap = the last level's slot count rounded up to a
// power of two - a few KiB for the usual fanouts, so that many micrographs share a CU; THREADS
// is chosen to match (64 .. 256).
template <typename OffT, int THREADS>
__global__ void __launch_bounds__(THREADS)
dedup_sample(const OffT* __restrict__ offsets, const int32_t* __restrict__ indices, const int32_t* __restrict__ seeds,
             int32_t n_seeds, DedupShape sh, DedupKeys keys, int32_t m_offset, int32_t seeds_per_key,
             int32_t* __restrict__ stage_nodes, int32_t* __restrict__ stage_child, int32_t* __restrict__ cnt,
             uint32_t cap) {
    extern __shared__ uint32_t dd_lds[];
    uint32_t* cur = dd_lds;                   // distinct vertices of the current level, ascending
    uint32_t* ent = dd_lds + cap;             // children in draw order (kDdNone: none)
    uint32_t* srt = dd_lds + 2 * cap;         // the same, sorted
    __shared__ uint32_t lds4[THREADS / kWave];
    const int32_t m = m_offset + (int32_t)blockIdx.x, B = n_seeds;
    const uint64_t keyed = keys.keyed[blockIdx.x / (uint32_t)seeds_per_key];   // one key per block of seeds
    const int tid = threadIdx.x;
    const int32_t root = seeds[m];
    if (tid == 0) {
        cur[0] = (uint32_t)root;
        stage_nodes[m] = root;
        cnt[m] = 1;
    }
    __syncthreads();
    uint32_t n_cur = 1;
    for (int32_t h = 1; h <= sh.n_layers; ++h) {
        const uint32_t f = (uint32_t)sh.f[h];
        const uint32_t n_cand = n_cur * f;
        uint32_t n2 = 1;
        while (n2 < n_cand) n2 <<= 1;
        // draw: entry c = (node q, draw j)
        for (uint32_t c = tid; c < n2; c += THREADS) {
            uint32_t child = kDdNone;
            if (c < n_cand) {
                const uint32_t q = c / f, j = c - q * f;
                const int32_t v = (int32_t)cur[q];
                if (v >= 0) {
                    const int64_t o0 = (int64_t)offsets[v];
                    const int64_t deg = (int64_t)offsets[(int64_t)v + 1] - o0;
                    if (deg > 0) {
                        uint64_t x = fr_finalise64((keyed ^ (((uint64_t)(uint32_t)root << 32) | (uint32_t)v)) +
                                                   0x9E3779B97F4A7C15ull);
                        x = fr_finalise64((x ^ (((uint64_t)(uint32_t)h << 32) | j)) + 0x9E3779B97F4A7C15ull);
                        child = (uint32_t)indices[o0 + (int64_t)(x % (uint64_t)deg)];
                    }
                }
                ent[c] = child;
            }
            srt[c] = child;
        }
        __syncthreads();
        // ascending sort (kDdNone sorts last), then the distinct values packed into cur, the next
        // level's node list (cur is free: every draw of this hop has been made)
        fr_bitonic_sort<THREADS>(srt, n2);
        const uint32_t n_next = fr_pack_distinct<THREADS>(srt, n2, cur, lds4);
        // this micrograph's slices of the staging arrays (slot-tree capacity)
        int32_t* nodes_out = stage_nodes + sh.base[h] + (int64_t)m * sh.P[h];
        int32_t* child_out = stage_child + (sh.base[h] - B) + (int64_t)m * sh.P[h];
        for (uint32_t i = tid; i < n_next; i += THREADS) nodes_out[i] = (int32_t)cur[i];
        for (uint32_t c = tid; c < n_cand; c += THREADS) {
            const uint32_t child = ent[c];
            int32_t pos = -1;
            if (child != kDdNone) pos = (int32_t)fr_lower_bound(cur, n_next, child);      // the value is there
            child_out[c] = pos;
        }
        if (tid == 0) cnt[(int64_t)h * B + m] = (int32_t)n_next;
        __syncthreads();
        n_cur = n_next;
    }
}

// One workgroup: per level the exclusive sums of the micrographs' node counts, the first node of
// every level and the first entry of every level's nodes.
__global__ void __launch_bounds__(kDdScanThreads)
dedup_scan(const int32_t* __restrict__ cnt, int32_t n_seeds, DedupShape sh, int32_t* __restrict__ mg_off,
           int64_t* __restrict__ level_start, int64_t* __restrict__ ent_start) {
    __shared__ uint32_t lds4[kDdScanThreads / kWave];
    int64_t nodes = 0, ents = 0;
    // thread t owns the contiguous run [t*per, (t+1)*per) of micrographs: sum it, scan the run sums
    const int32_t per = (n_seeds + kDdScanThreads - 1) / kDdScanThreads;
    const int32_t m0 = threadIdx.x * per, m1 = m0 + per < n_seeds ? m0 + per : n_seeds;
    for (int32_t h = 0; h <= sh.n_layers; ++h) {
        if (threadIdx.x == 0) {
            level_start[h] = nodes;
            ent_start[h] = ents;
        }
        const int32_t* c = cnt + (int64_t)h * n_seeds;
        uint32_t mine = 0;
        for (int32_t mm = m0; mm < m1; ++mm) mine += (uint32_t)c[mm];
        uint32_t total;
        uint32_t run = fr_block_scan<kDdScanThreads, uint32_t>(mine, lds4, total);
        for (int32_t mm = m0; mm < m1; ++mm) {
            mg_off[(int64_t)h * n_seeds + mm] = (int32_t)run;
            run += (uint32_t)c[mm];
        }
        nodes += total;
        if (h < sh.n_layers) ents += (int64_t)total * sh.f[h + 1];
    }
    if (threadIdx.x == 0) {
        level_start[sh.n_layers + 1] = nodes;
        ent_start[sh.n_layers + 1] = ents;       // total entries
    }
}

// One thread per staging slot (level h, micrograph m, i-th node of that micrograph's level).
__global__ void __launch_bounds__(kDdThreads)
dedup_compact(const int32_t* __restrict__ stage_nodes, const int32_t* __restrict__ stage_child,
              const int32_t* __restrict__ cnt, const int32_t* __restrict__ mg_off,
              const int64_t* __restrict__ level_start, const int64_t* __restrict__ ent_start, int32_t n_seeds,
              DedupShape sh, int32_t* __restrict__ node_vertex, int32_t* __restrict__ indptr,
              int32_t* __restrict__ idx, uint8_t* __restrict__ present) {
    const int32_t L = sh.n_layers, B = n_seeds;
    const int64_t T = sh.base[L + 1], S = sh.base[L];
    const int64_t t = (int64_t)blockIdx.x * kDdThreads + threadIdx.x;
    if (t >= T) return;
    // unused tails: no vertex, empty segments, no child
    const int64_t n_nodes = level_start[L + 1], n_nonleaf = level_start[L], nnz = ent_start[L + 1];
    if (t >= n_nodes) node_vertex[t] = -1;
    if (t >= n_nonleaf && t <= S) indptr[t] = (int32_t)nnz;
    if (t >= nnz && t < T - B) idx[t] = -1;
    int32_t h = 0;
    while (h < L && t >= sh.base[h + 1]) ++h;
    const int64_t o = t - sh.base[h];
    const int32_t mg = (int32_t)(o / sh.P[h]), i = (int32_t)(o - (int64_t)mg * sh.P[h]);
    if (i >= cnt[(int64_t)h * B + mg]) return;
    const int64_t local = (int64_t)mg_off[(int64_t)h * B + mg] + i;       // rank inside the level
    const int64_t gi = level_start[h] + local;
    const int32_t vertex = stage_nodes[t];
    node_vertex[gi] = vertex;
    if (present != nullptr && vertex >= 0) present[vertex] = 1;     // the pre-gather's presence map
    if (h == L) return;
    const int32_t f = sh.f[h + 1];
    const int64_t e0 = ent_start[h] + local * f;
    indptr[gi] = (int32_t)e0;
    const int32_t* child = stage_child + (sh.base[h + 1] - B) + ((int64_t)mg * sh.P[h] + i) * f;
    const int64_t next0 = level_start[h + 1] + mg_off[(int64_t)(h + 1) * B + mg];
    for (int32_t j = 0; j < f; ++j) {
        const int32_t c = child[j];
        idx[e0 + j] = c >= 0 ? (int32_t)(next0 + c) : -1;
    }
}

__global__ void __launch_bounds__(kDdThreads)
compose_idx(const int32_t* __restrict__ idx, int64_t n, const int32_t* __restrict__ map, int32_t* __restrict__ out) {
    const int64_t stride = (int64_t)gridDim.x * kDdThreads;
    for (int64_t e = (int64_t)blockIdx.x * kDdThreads + threadIdx.x; e < n; e += stride) {
        const int32_t u = idx[e];
        out[e] = u >= 0 ? map[u] : -1;
    }
}

// Locality counts of the micrographs of a frontier structure (paper section 4, "data locality in
// micrographs").  One workgroup per micrograph walks its levels: the nodes of a micrograph's level
// are contiguous and every one of them is an entry of one of its previous-level nodes, so the next
// level's range is [smallest entry, largest entry] of the current range's segments.  Vertices go
// into an open-addressing hash set in LDS; the thread that claims a free cell has found a new one.
constexpr int kFlThreads = 256;

__global__ void __launch_bounds__(kFlThreads)
frontier_locality(const int32_t* __restrict__ node_vertex, const int64_t* __restrict__ level_start,
                  const int32_t* __restrict__ indptr, const int32_t* __restrict__ idx, int32_t n_layers,
                  const int32_t* __restrict__ owner, uint32_t table_mask, int32_t* __restrict__ n_total,
                  int32_t* __restrict__ n_coloc) {
    extern __shared__ int32_t fl_table[];
    __shared__ uint32_t lds4[kFlThreads / kWave];
    __shared__ int32_t next_lo, next_hi;
    __shared__ int32_t overflow;              // set when a vertex found no cell: the table was too small
    const int32_t m = blockIdx.x;
    const uint32_t tid = threadIdx.x;
    if (tid == 0) overflow = 0;
    for (uint32_t i = tid; i <= table_mask; i += kFlThreads) fl_table[i] = -1;
    const int32_t root = node_vertex[m];
    const int32_t root_home = root >= 0 ? owner[root] : -1;
    const int64_t n_nonleaf = level_start[n_layers];
    uint32_t tot = 0, col = 0;
    int32_t lo = m, hi = m + 1;               // node range of the current level
    for (int32_t h = 0; h <= n_layers && lo < hi; ++h) {
        __syncthreads();
        if (tid == 0) {
            next_lo = 0x7FFFFFFF;
            next_hi = -1;
        }
        __syncthreads();
        for (int32_t q = lo + (int32_t)tid; q < hi; q += kFlThreads) {
            const int32_t v = node_vertex[q];
            if (v < 0) continue;
            uint32_t cell = ((uint32_t)v * 2654435761u) & table_mask;
            // at most one pass over the table: with the capacity the caller promised it is never more
            // than half full; a micrograph with more distinct vertices than cells cannot be counted -
            // the probe ends after one pass and the micrograph reports -1 instead of a wrong count
            bool placed = false;
            for (uint32_t probe = 0; probe <= table_mask && !placed; ++probe) {
                const int32_t old = atomicCAS(&fl_table[cell], -1, v);
                if (old == -1) {   // first time this vertex is seen in the micrograph
                    ++tot;
                    if (v != root && owner[v] == root_home) ++col;
                    placed = true;
                } else if (old == v) {
                    placed = true;
                }
                cell = (cell + 1) & table_mask;
            }
            if (!placed) overflow = 1;
        }
        if (h == n_layers || hi > n_nonleaf) break;        // leaves have no segments (uniform)
        int32_t mn = 0x7FFFFFFF, mx = -1;
        for (int32_t e = indptr[lo] + (int32_t)tid; e < indptr[hi]; e += kFlThreads) {
            const int32_t u = idx[e];
            if (u >= 0) {
                mn = u < mn ? u : mn;
                mx = u > mx ? u : mx;
            }
        }
        if (mx >= 0) {
            atomicMin(&next_lo, mn);
            atomicMax(&next_hi, mx);
        }
        __syncthreads();
        lo = next_lo;
        hi = next_hi + 1;
    }
    uint32_t t_all, c_all;
    (void)fr_block_scan<kFlThreads, uint32_t>(tot, lds4, t_all);
    (void)fr_block_scan<kFlThreads, uint32_t>(col, lds4, c_all);     // (its barriers order `overflow` too)
    if (tid == 0) {
        n_total[m] = overflow ? -1 : (int32_t)t_all;
        n_coloc[m] = overflow ? -1 : (int32_t)c_all;
    }
}

struct DedupWs {
    size_t nodes_bytes, child_bytes, cnt_bytes, ent_start_bytes, total;
};
static DedupWs dedup_ws_layout(int64_t T, int64_t B, int32_t L) {
    DedupWs W{};
    W.nodes_bytes = align_up((size_t)T * 4, 256);
    W.child_bytes = align_up((size_t)(T - B > 0 ? T - B : 1) * 4, 256);
    W.cnt_bytes = align_up((size_t)(L + 1) * B * 4, 256);          // once for cnt, once for mg_off
    W.ent_start_bytes = align_up((size_t)(L + 2) * 8, 256);
    W.total = W.nodes_bytes + W.child_bytes + 2 * W.cnt_bytes + W.ent_start_bytes;
    return W;
}

}  // namespace hopgnn

using namespace hopgnn;

extern "C" size_t hopgnn_sample_dedup_ws_bytes(int32_t n_seeds, const int32_t* fanouts, int32_t n_layers) {
    const int64_t t_seed = hopgnn_slots_per_seed(fanouts, n_layers);
    if (t_seed < 0 || n_seeds < 0) return 0;
    return dedup_ws_layout(t_seed * n_seeds, n_seeds, n_layers).total;
}

extern "C" hopgnn_status hopgnn_sample_dedup(const hopgnn_csr* g, const int32_t* seeds, int32_t n_seeds,
                                             int32_t seeds_per_key, const int32_t* fanouts, int32_t n_layers,
                                             const uint64_t* keys, int32_t* node_vertex, int64_t* level_start,
                                             int32_t* indptr, int32_t* idx, void* ws, size_t ws_bytes, void* stream) {
    return sample_dedup(g, seeds, n_seeds, seeds_per_key, fanouts, n_layers, keys, node_vertex, level_start, indptr, idx,
                        ws, ws_bytes, nullptr, stream);
}

hopgnn_status hopgnn::sample_dedup(const hopgnn_csr* g, const int32_t* seeds, int32_t n_seeds, int32_t seeds_per_key,
                                   const int32_t* fanouts, int32_t n_layers, const uint64_t* keys, int32_t* node_vertex,
                                   int64_t* level_start, int32_t* indptr, int32_t* idx, void* ws, size_t ws_bytes,
                                   uint8_t* present, void* stream) {
    if (g == nullptr || fanouts == nullptr || n_seeds < 0 || seeds_per_key < 1) return HOPGNN_EINVAL;
    const int64_t t_seed = hopgnn_slots_per_seed(fanouts, n_layers);
    if (t_seed < 0) return HOPGNN_EINVAL;
    if (g->n_vertices < 0 || g->n_edges < 0 || g->n_vertices > ((int64_t)1 << 31)) return HOPGNN_EINVAL;
    if (n_seeds == 0) return HOPGNN_OK;
    if (g->offsets == nullptr || seeds == nullptr || keys == nullptr || node_vertex == nullptr || level_start == nullptr ||
        indptr == nullptr || idx == nullptr || ws == nullptr)
        return HOPGNN_EINVAL;
    if (g->n_edges > 0 && g->indices == nullptr) return HOPGNN_EINVAL;
    const int64_t T = (int64_t)n_seeds * t_seed;
    if (T >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    if (!aligned(ws, 256)) return HOPGNN_EINVAL;

    DedupShape sh{};
    sh.n_layers = n_layers;
    sh.P[0] = 1;
    sh.base[0] = 0;
    for (int32_t h = 1; h <= n_layers; ++h) {
        sh.f[h] = fanouts[h - 1];
        sh.P[h] = sh.P[h - 1] * sh.f[h];
        sh.base[h] = sh.base[h - 1] + n_seeds * sh.P[h - 1];
    }
    sh.base[n_layers + 1] = sh.base[n_layers] + n_seeds * sh.P[n_layers];
    if (sh.P[n_layers] > kDdMaxLevel) return HOPGNN_ERANGE;     // a level of one micrograph must fit the LDS sort

    const DedupWs W = dedup_ws_layout(T, n_seeds, n_layers);
    if (ws_bytes < W.total) return HOPGNN_ENOMEM_WS;
    char* p = static_cast<char*>(ws);
    int32_t* stage_nodes = reinterpret_cast<int32_t*>(p);
    int32_t* stage_child = reinterpret_cast<int32_t*>(p + W.nodes_bytes);
    int32_t* cnt = reinterpret_cast<int32_t*>(p + W.nodes_bytes + W.child_bytes);
    int32_t* mg_off = reinterpret_cast<int32_t*>(p + W.nodes_bytes + W.child_bytes + W.cnt_bytes);
    int64_t* ent_start = reinterpret_cast<int64_t*>(p + W.nodes_bytes + W.child_bytes + 2 * W.cnt_bytes);

    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t cap = 1;
    while (cap < (uint32_t)sh.P[n_layers]) cap <<= 1;
    const size_t lds = (size_t)3 * cap * sizeof(uint32_t);
    // wide workgroups sort a long level faster, narrow ones keep more micrographs resident (a CU
    // holds 2048 threads): 256 threads only while all micrographs still fit the chip at once
    const int threads = cap >= 1024 && (cap >= 4096 || n_seeds <= 2048) ? 256 : (cap >= 256 ? 128 : 64);
    const void* off = g->offsets;
    const int32_t n_keys = (int32_t)ceil_div(n_seeds, seeds_per_key);
    for (int32_t k0 = 0; k0 < n_keys; k0 += kDdKeysPerLaunch) {     // 64 keys fit one launch's arguments
        const int32_t nk = n_keys - k0 < kDdKeysPerLaunch ? n_keys - k0 : kDdKeysPerLaunch;
        DedupKeys dk{};
        for (int32_t i = 0; i < nk; ++i) dk.keyed[i] = fr_finalise64(keys[k0 + i] + 0x9E3779B97F4A7C15ull);
        const int64_t m0 = (int64_t)k0 * seeds_per_key;
        const int64_t count = (int64_t)nk * seeds_per_key < n_seeds - m0 ? (int64_t)nk * seeds_per_key : n_seeds - m0;
#define HOPGNN_DD_LAUNCH(OffT, THREADS)                                                                              \
    hipLaunchKernelGGL((dedup_sample<OffT, THREADS>), dim3((unsigned)count), dim3(THREADS), lds, s,                  \
                       static_cast<const OffT*>(off), g->indices, seeds, n_seeds, sh, dk, (int32_t)m0, seeds_per_key, \
                       stage_nodes, stage_child, cnt, cap)
        if (g->offsets_i64) {
            if (threads == 256) HOPGNN_DD_LAUNCH(int64_t, 256);
            else if (threads == 128) HOPGNN_DD_LAUNCH(int64_t, 128);
            else HOPGNN_DD_LAUNCH(int64_t, 64);
        } else {
            if (threads == 256) HOPGNN_DD_LAUNCH(int32_t, 256);
            else if (threads == 128) HOPGNN_DD_LAUNCH(int32_t, 128);
            else HOPGNN_DD_LAUNCH(int32_t, 64);
        }
#undef HOPGNN_DD_LAUNCH
        HOPGNN_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(dedup_scan, dim3(1), dim3(kDdScanThreads), 0, s, cnt, n_seeds, sh, mg_off, level_start, ent_start);
    HOPGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(dedup_compact, dim3((unsigned)ceil_div(T, kDdThreads)), dim3(kDdThreads), 0, s, stage_nodes,
                       stage_child, cnt, mg_off, level_start, ent_start, n_seeds, sh, node_vertex, indptr, idx, present);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

extern "C" hopgnn_status hopgnn_compose_idx(const int32_t* idx, int64_t n, const int32_t* map, int32_t* out,
                                            void* stream) {
    if (n < 0) return HOPGNN_EINVAL;
    if (n == 0) return HOPGNN_OK;
    if (idx == nullptr || map == nullptr || out == nullptr) return HOPGNN_EINVAL;
    const int64_t want = ceil_div(n, kDdThreads);
    hipLaunchKernelGGL(compose_idx, dim3((unsigned)(want < 8192 ? want : 8192)), dim3(kDdThreads), 0,
                       static_cast<hipStream_t>(stream), idx, n, map, out);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}

extern "C" hopgnn_status hopgnn_frontier_locality(const int32_t* node_vertex, const int64_t* level_start,
                                                  const int32_t* indptr, const int32_t* idx, int32_t n_seeds,
                                                  int32_t n_layers, int64_t nodes_per_seed, const int32_t* owner,
                                                  int32_t* n_total, int32_t* n_coloc, void* stream) {
    if (n_seeds < 0 || n_layers < 1 || n_layers > kMaxLayers || nodes_per_seed < 1) return HOPGNN_EINVAL;
    if (nodes_per_seed > 16384) return HOPGNN_ERANGE;   // hash set of 2 * nodes_per_seed cells must fit 160 KB of LDS
    if (n_seeds == 0) return HOPGNN_OK;
    if (node_vertex == nullptr || level_start == nullptr || indptr == nullptr || idx == nullptr || owner == nullptr ||
        n_total == nullptr || n_coloc == nullptr)
        return HOPGNN_EINVAL;
    uint32_t cells = 64;
    while (cells < 2 * (uint32_t)nodes_per_seed) cells *= 2;   // load factor <= 1/2
    const size_t lds = (size_t)cells * 4;
    if (lds > 64 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(frontier_locality), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds) != hipSuccess)
        return HOPGNN_EHIP;
    hipLaunchKernelGGL(frontier_locality, dim3((unsigned)n_seeds), dim3(kFlThreads), lds, static_cast<hipStream_t>(stream),
                       node_vertex, level_start, indptr, idx, n_layers, owner, cells - 1, n_total, n_coloc);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}
