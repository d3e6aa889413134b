// hopgnn_sample_layerwise: layer-wise sampling of micrographs (paper section 4 measures the
// locality of micrographs under node-wise and under layer-wise sampling).  Per micrograph and hop
// a budget of s_h draws is made for the WHOLE layer: uniformly, with replacement, over the
// concatenated neighbour lists of the previous level's nodes, so a vertex is drawn with probability
// proportional to the number of edges from the previous level into it.  The level's nodes are the
// distinct drawn vertices in ascending order; every edge between the previous level's nodes and
// them is kept, each (node, node) pair once.
//
//   lw_draw       one workgroup per micrograph; per hop: prefix sums of the previous level's degrees
//                 (LDS), the draws (position -> node by binary search in the prefix sums), an LDS
//                 bitonic sort + distinct.  The next hop needs only the node list, so the pass over
//                 the neighbour lists is NOT done here: hub vertices make one micrograph's lists
//                 100x longer than the median's, and a workgroup per micrograph would wait for them
//   lw_chunks     cuts every (micrograph, hop)'s concatenated lists into chunks of kLwChunk entries
//                 and numbers the chunks (one workgroup, exclusive sums)
//   lw_adjacency  edge-balanced: every workgroup takes the same number of chunks, looks every
//                 neighbour up in that hop's new node list (a hashed membership bit first: nearly
//                 all are outside) and sets a bit in the (previous node x node) matrix
//   lw_segments   per micrograph: the rows of the bit matrices become the segments
//   lw_scan       exclusive sums of the per-micrograph node and entry counts, level by level
//   lw_compact    level-major global numbering: node vertices, CSR of node indices, tails filled
#include "frontier_common.hpp"
#include "pregather_internal.hpp"

namespace hopgnn {

constexpr int kLwThreads = 256;           // scan, compaction and the adjacency pass
constexpr int kLwChunkThreads = 1024;     // the one-workgroup scans (chunk numbers, node and entry counts)
constexpr int kLwSegThreads = 128;
constexpr int kLwMaxLevel = 1024;         // largest budget of one level
constexpr int kLwMaxPairs = 65536;        // largest product of two consecutive budgets
constexpr int kLwKeysPerLaunch = 64;
constexpr int kLwUnroll = 8;              // neighbour loads in flight per thread in the adjacency pass
constexpr uint32_t kLwChunk = 8192;       // list entries per chunk
constexpr int kLwAdjGrid = 8192;          // workgroups of the adjacency pass: short contiguous shares balance best

struct LwKeys {
    uint64_t keyed[kLwKeysPerLaunch];     // first hash round already applied on the host
};

struct LwShape {
    int32_t n_layers;
    int32_t s[kMaxLayers + 1];            // node capacity of level h per micrograph; s[0] = 1
    int32_t nbase[kMaxLayers + 2];        // first staging slot of level h's nodes; [L+1] = node capacity
    int32_t ebase[kMaxLayers + 1];        // first staging slot of the entries of level h's nodes; [L] = entry capacity
    int32_t wbase[kMaxLayers + 1];        // first word of the bit matrices of level h's nodes; [L] = all words
};

__host__ __device__ __forceinline__ uint32_t lw_words(const LwShape& sh, int32_t h) {     // per row, level h -> h+1
    return ((uint32_t)sh.s[h + 1] + 31) / 32;
}

struct LwLds {
    uint32_t max_s, cap2, filt_words;
    size_t draw_bytes, adj_bytes;
};
static LwLds lw_lds_layout(const LwShape& sh) {
    LwLds l{};
    for (int32_t h = 0; h <= sh.n_layers; ++h) l.max_s = (uint32_t)sh.s[h] > l.max_s ? (uint32_t)sh.s[h] : l.max_s;
    l.cap2 = 1;
    while (l.cap2 < l.max_s) l.cap2 <<= 1;
    // membership filter of a level's nodes: 32 bits per node of the largest level keep false hits rare
    l.filt_words = l.cap2 < 64 ? 64 : l.cap2;
    // lw_draw: pref (u64, max_s + 1), obase (u64, max_s), then cur, nxt (max_s each), srt (cap2)
    l.draw_bytes = (size_t)(2 * l.max_s + 1) * 8 + ((size_t)2 * l.max_s + l.cap2) * 4;
    // lw_adjacency: pref, obase, abase (u64), then rel (max_s + 1), nxt (max_s), filt
    l.adj_bytes = (size_t)(3 * l.max_s + 1) * 8 + ((size_t)2 * l.max_s + 1 + l.filt_words) * 4;
    return l;
}

template <typename OffT, int THREADS>
__global__ void __launch_bounds__(THREADS)
lw_draw(const OffT* __restrict__ offsets, const int32_t* __restrict__ indices, const int32_t* __restrict__ seeds,
        int32_t n_seeds, LwShape sh, LwKeys keys, int32_t m_offset, int32_t seeds_per_key, uint32_t max_s, uint32_t cap2,
        int32_t* __restrict__ stage_nodes, uint64_t* __restrict__ stage_pref, uint64_t* __restrict__ stage_obase,
        uint64_t* __restrict__ pair_len, uint32_t* __restrict__ gbits, int32_t* __restrict__ cnt) {
    extern __shared__ uint64_t lw_lds[];
    uint64_t* pref = lw_lds;                                             // exclusive degree sums, [n_cur + 1]
    uint64_t* obase = lw_lds + max_s + 1;                                // first list entry of every node
    uint32_t* cur = reinterpret_cast<uint32_t*>(obase + max_s);          // previous level's nodes, ascending
    uint32_t* nxt = cur + max_s;                                         // this level's nodes
    uint32_t* srt = nxt + max_s;                                         // [cap2] drawn vertices
    __shared__ uint64_t lds8[THREADS / kWave];
    __shared__ uint32_t lds4[THREADS / kWave];
    const int32_t m = m_offset + (int32_t)blockIdx.x, B = n_seeds;
    const uint64_t keyed = keys.keyed[blockIdx.x / (uint32_t)seeds_per_key];
    const uint32_t tid = threadIdx.x;
    const int32_t root = seeds[m];
    // the micrograph's draws: hash(key, root, no vertex, hop, j)
    const uint64_t rooted =
        fr_finalise64((keyed ^ (((uint64_t)(uint32_t)root << 32) | 0xFFFFFFFFull)) + 0x9E3779B97F4A7C15ull);
    // this micrograph's bit matrices start empty
    for (int32_t h = 0; h < sh.n_layers; ++h) {
        const uint32_t n = (uint32_t)sh.s[h] * lw_words(sh, h);
        uint32_t* mat = gbits + sh.wbase[h] + (int64_t)m * n;
        for (uint32_t i = tid; i < n; i += THREADS) mat[i] = 0;
    }
    if (tid == 0) {
        cur[0] = (uint32_t)root;
        stage_nodes[m] = root;
        cnt[m] = 1;
    }
    __syncthreads();
    uint32_t n_cur = 1;
    for (int32_t h = 1; h <= sh.n_layers; ++h) {
        const uint32_t s_h = (uint32_t)sh.s[h];
        const int64_t prev_slot = sh.nbase[h - 1] + (int64_t)m * sh.s[h - 1];
        // exclusive sums of the previous level's degrees
        uint64_t carry = 0;
        for (uint32_t i0 = 0; i0 < n_cur; i0 += THREADS) {
            const uint32_t i = i0 + tid;
            uint64_t deg = 0, o0 = 0;
            if (i < n_cur && (int32_t)cur[i] >= 0) {          // only a seed can be negative: no neighbours
                const int64_t v = (int64_t)cur[i];
                o0 = (uint64_t)offsets[v];
                deg = (uint64_t)offsets[v + 1] - o0;
            }
            uint64_t total;
            const uint64_t ex = carry + fr_block_scan<THREADS, uint64_t>(deg, lds8, total);
            if (i < n_cur) {
                pref[i] = ex;
                obase[i] = o0;
                stage_pref[prev_slot + i] = ex;
                stage_obase[prev_slot + i] = o0;
            }
            carry += total;
        }
        const uint64_t D = carry;
        if (tid == 0) {
            pref[n_cur] = D;
            pair_len[(int64_t)(h - 1) * B + m] = D;
        }
        __syncthreads();
        if (D == 0) {          // no candidate (uniform over the workgroup): this and all later levels are empty
            if (tid == 0) cnt[(int64_t)h * B + m] = 0;
            n_cur = 0;
            continue;
        }
        // the draws
        uint32_t n2 = 1;
        while (n2 < s_h) n2 <<= 1;
        for (uint32_t j = tid; j < n2; j += THREADS) {
            uint32_t v = kFrNone;
            if (j < s_h) {
                const uint64_t x = fr_finalise64((rooted ^ (((uint64_t)(uint32_t)h << 32) | j)) + 0x9E3779B97F4A7C15ull);
                const uint64_t p = x % D;
                uint32_t lo = 0, hi = n_cur;          // the last q with pref[q] <= p
                while (hi - lo > 1) {
                    const uint32_t mid = (lo + hi) >> 1;
                    if (pref[mid] <= p) lo = mid;
                    else hi = mid;
                }
                v = (uint32_t)indices[obase[lo] + (p - pref[lo])];
            }
            srt[j] = v;
        }
        __syncthreads();
        fr_bitonic_sort<THREADS>(srt, n2);
        const uint32_t n_next = fr_pack_distinct<THREADS>(srt, n2, nxt, lds4);
        int32_t* nodes_out = stage_nodes + sh.nbase[h] + (int64_t)m * s_h;
        for (uint32_t i = tid; i < n_next; i += THREADS) nodes_out[i] = (int32_t)nxt[i];
        if (tid == 0) cnt[(int64_t)h * B + m] = (int32_t)n_next;
        __syncthreads();
        uint32_t* t = cur;
        cur = nxt;
        nxt = t;
        n_cur = n_next;
    }
}

// One workgroup: chunk_start[pair] = number of chunks before (hop, micrograph) pair `pair`,
// chunk_start[n_pairs] = all chunks.  Thread t owns a contiguous run of pairs.
__global__ void __launch_bounds__(kLwChunkThreads)
lw_chunks(const uint64_t* __restrict__ pair_len, int32_t n_pairs, uint32_t* __restrict__ chunk_start) {
    __shared__ uint32_t lds4[kLwChunkThreads / kWave];
    const int32_t per = (n_pairs + kLwChunkThreads - 1) / kLwChunkThreads;
    const int32_t p0 = threadIdx.x * per, p1 = p0 + per < n_pairs ? p0 + per : n_pairs;
    uint32_t mine = 0, total;
    for (int32_t i = p0; i < p1; ++i) mine += (uint32_t)((pair_len[i] + kLwChunk - 1) / kLwChunk);
    uint32_t run = fr_block_scan<kLwChunkThreads, uint32_t>(mine, lds4, total);
    for (int32_t i = p0; i < p1; ++i) {
        chunk_start[i] = run;
        run += (uint32_t)((pair_len[i] + kLwChunk - 1) / kLwChunk);
    }
    if (threadIdx.x == 0) chunk_start[n_pairs] = total;
}

// Every workgroup takes an equal, contiguous share of the chunks.  A chunk is kLwChunk consecutive
// entries of one (hop, micrograph) pair's concatenated neighbour lists; a thread's positions inside
// it ascend, so its list pointer only advances, and kLwUnroll independent loads are in flight.
__global__ void __launch_bounds__(kLwThreads)
lw_adjacency(const int32_t* __restrict__ indices, int32_t n_seeds, LwShape sh, uint32_t max_s, uint32_t filt_words,
             const int32_t* __restrict__ stage_nodes, const uint64_t* __restrict__ stage_pref,
             const uint64_t* __restrict__ stage_obase, const uint64_t* __restrict__ pair_len,
             const uint32_t* __restrict__ chunk_start, const int32_t* __restrict__ cnt, uint32_t* __restrict__ gbits) {
    extern __shared__ uint64_t lw_lds[];
    uint64_t* pref = lw_lds;
    uint64_t* obase = lw_lds + max_s + 1;
    uint64_t* abase = obase + max_s;                      // per chunk: list entry of chunk position 0, per list
    uint32_t* rel = reinterpret_cast<uint32_t*>(abase + max_s);      // per chunk: list starts relative to the chunk
    uint32_t* nxt = rel + max_s + 1;
    uint32_t* filt = nxt + max_s;
    __shared__ int32_t found;
    const uint32_t filt_shift = 32u - (uint32_t)__builtin_ctz(filt_words * 32u);
    const uint32_t tid = threadIdx.x;
    const int32_t B = n_seeds, n_pairs = sh.n_layers * B;
    const uint32_t total = chunk_start[n_pairs];
    const uint32_t share = (total + gridDim.x - 1) / gridDim.x;
    const uint32_t c0 = blockIdx.x * share, c1 = c0 + share < total ? c0 + share : total;
    if (c0 >= c1) return;
    // the pair of the first chunk: the last pair whose first chunk is not after c0, in two rounds
    if (tid == 0) found = 0;
    __syncthreads();
    const int32_t stride = (n_pairs + kLwThreads - 1) / kLwThreads;
    {
        const int64_t i = (int64_t)tid * stride;
        if (i < n_pairs && chunk_start[i] <= c0) atomicMax(&found, (int32_t)i);
    }
    __syncthreads();
    const int32_t coarse = found;
    __syncthreads();
    for (int32_t t = tid; t < stride; t += kLwThreads) {
        const int32_t i = coarse + t;
        if (i < n_pairs && chunk_start[i] <= c0) atomicMax(&found, i);
    }
    __syncthreads();
    int32_t pair = found, loaded = -1;
    uint32_t n_prev = 0, n_next = 0, words = 0;
    uint64_t D = 0;
    uint32_t* mat = nullptr;
    for (uint32_t c = c0; c < c1; ++c) {
        while (chunk_start[pair + 1] <= c) ++pair;          // c < total = chunk_start[n_pairs]
        if (pair != loaded) {
            __syncthreads();                                // the previous pair's lists are no longer read
            loaded = pair;
            const int32_t h = pair / B, m = pair - h * B;   // level of the previous nodes, micrograph
            n_prev = (uint32_t)cnt[(int64_t)h * B + m];
            n_next = (uint32_t)cnt[(int64_t)(h + 1) * B + m];
            D = pair_len[pair];
            words = lw_words(sh, h);
            mat = gbits + sh.wbase[h] + (int64_t)m * sh.s[h] * words;
            const int64_t prev_slot = sh.nbase[h] + (int64_t)m * sh.s[h];
            const int32_t* nodes = stage_nodes + sh.nbase[h + 1] + (int64_t)m * sh.s[h + 1];
            for (uint32_t i = tid; i < n_prev; i += kLwThreads) {
                pref[i] = stage_pref[prev_slot + i];
                obase[i] = stage_obase[prev_slot + i];
            }
            if (tid == 0) pref[n_prev] = D;
            for (uint32_t i = tid; i < filt_words; i += kLwThreads) filt[i] = 0;
            for (uint32_t i = tid; i < n_next; i += kLwThreads) nxt[i] = (uint32_t)nodes[i];
            __syncthreads();
            for (uint32_t i = tid; i < n_next; i += kLwThreads) {
                const uint32_t hsh = (nxt[i] * 0x9E3779B1u) >> filt_shift;
                atomicOr(&filt[hsh >> 5], 1u << (hsh & 31));
            }
            __syncthreads();
        }
        // the chunk in 32-bit positions: rel[q] = where list q starts inside the chunk (clamped to
        // [0, kLwChunk]), abase[q] = the list entry that chunk position 0 would be
        const uint64_t start = (uint64_t)(c - chunk_start[pair]) * kLwChunk;
        const uint32_t len = (uint32_t)(start + kLwChunk < D ? kLwChunk : D - start);
        __syncthreads();                                    // the previous chunk's tables are no longer read
        for (uint32_t i = tid; i <= n_prev; i += kLwThreads) {
            const uint64_t pr = pref[i];
            rel[i] = pr <= start ? 0u : (pr - start >= kLwChunk ? kLwChunk : (uint32_t)(pr - start));
            if (i < n_prev) abase[i] = obase[i] + (start - pr);        // modulo 2^64: abase + position is exact
        }
        __syncthreads();
        uint32_t q = 0;
        if (tid < len) {                                    // the last q with rel[q] <= the thread's first position
            uint32_t hi = n_prev;
            while (hi - q > 1) {
                const uint32_t mid = (q + hi) >> 1;
                if (rel[mid] <= tid) q = mid;
                else hi = mid;
            }
        }
        for (uint32_t p0 = tid; p0 < len; p0 += kLwUnroll * kLwThreads) {
            uint32_t v[kLwUnroll], qq[kLwUnroll];
#pragma unroll
            for (int u = 0; u < kLwUnroll; ++u) {
                const uint32_t pl = p0 + u * kLwThreads;
                v[u] = kFrNone;
                qq[u] = 0;
                if (pl < len) {
                    while (rel[q + 1] <= pl) ++q;          // rel[n_prev] >= len > pl: q stays below n_prev
                    qq[u] = q;
                    v[u] = (uint32_t)indices[abase[q] + pl];
                }
            }
#pragma unroll
            for (int u = 0; u < kLwUnroll; ++u) {
                if (v[u] == kFrNone) continue;
                const uint32_t hsh = (v[u] * 0x9E3779B1u) >> filt_shift;
                if (((filt[hsh >> 5] >> (hsh & 31)) & 1u) == 0) continue;
                const uint32_t pos = fr_lower_bound(nxt, n_next, v[u]);
                if (pos < n_next && nxt[pos] == v[u]) atomicOr(&mat[qq[u] * words + (pos >> 5)], 1u << (pos & 31));
            }
        }
    }
}

// One workgroup per micrograph: the rows of its bit matrices become segments (positions of the
// set bits, ascending), with their exclusive offsets inside the micrograph's hop.
__global__ void __launch_bounds__(kLwSegThreads)
lw_segments(int32_t n_seeds, LwShape sh, const uint32_t* __restrict__ gbits, const int32_t* __restrict__ cnt,
            int32_t* __restrict__ stage_eoff, int32_t* __restrict__ stage_child, int32_t* __restrict__ ecnt) {
    __shared__ uint32_t lds4[kLwSegThreads / kWave];
    const int32_t m = blockIdx.x, B = n_seeds;
    const uint32_t tid = threadIdx.x;
    for (int32_t h = 0; h < sh.n_layers; ++h) {
        const uint32_t n_cur = (uint32_t)cnt[(int64_t)h * B + m], words = lw_words(sh, h);
        const uint32_t* mat = gbits + sh.wbase[h] + (int64_t)m * sh.s[h] * words;
        int32_t* eoff_out = stage_eoff + sh.nbase[h] + (int64_t)m * sh.s[h];
        int32_t* child_out = stage_child + sh.ebase[h] + (int64_t)m * sh.s[h] * sh.s[h + 1];
        uint32_t ecarry = 0;
        for (uint32_t i0 = 0; i0 < n_cur; i0 += kLwSegThreads) {
            const uint32_t i = i0 + tid;
            uint32_t c = 0;
            if (i < n_cur)
                for (uint32_t w = 0; w < words; ++w) c += (uint32_t)__popc(mat[i * words + w]);
            uint32_t total;
            const uint32_t ex = ecarry + fr_block_scan<kLwSegThreads, uint32_t>(c, lds4, total);
            if (i < n_cur) {
                eoff_out[i] = (int32_t)ex;
                uint32_t at = ex;
                for (uint32_t w = 0; w < words; ++w) {
                    uint32_t word = mat[i * words + w];
                    while (word != 0) {
                        const uint32_t b = (uint32_t)__ffs((int)word) - 1;
                        child_out[at++] = (int32_t)(w * 32 + b);
                        word &= word - 1;
                    }
                }
            }
            ecarry += total;
        }
        if (tid == 0) ecnt[(int64_t)h * B + m] = (int32_t)ecarry;
    }
}

// One workgroup: per level the exclusive sums of the micrographs' node counts and of the entry
// counts of that level's nodes, the first node of every level and the first entry of every level.
__global__ void __launch_bounds__(kLwChunkThreads)
lw_scan(const int32_t* __restrict__ cnt, const int32_t* __restrict__ ecnt, int32_t n_seeds, int32_t n_layers,
        int32_t* __restrict__ mg_off, int32_t* __restrict__ mg_eoff, int64_t* __restrict__ level_start,
        int64_t* __restrict__ ent_start) {
    __shared__ uint32_t lds4[kLwChunkThreads / kWave];
    int64_t nodes = 0, ents = 0;
    // thread t owns the contiguous run [t*per, (t+1)*per) of micrographs: sum it, scan the run sums
    const int32_t per = (n_seeds + kLwChunkThreads - 1) / kLwChunkThreads;
    const int32_t m0 = threadIdx.x * per, m1 = m0 + per < n_seeds ? m0 + per : n_seeds;
    for (int32_t h = 0; h <= n_layers; ++h) {
        if (threadIdx.x == 0) level_start[h] = nodes;
        const int32_t* c = cnt + (int64_t)h * n_seeds;
        uint32_t mine = 0, total;
        for (int32_t mm = m0; mm < m1; ++mm) mine += (uint32_t)c[mm];
        uint32_t run = fr_block_scan<kLwChunkThreads, uint32_t>(mine, lds4, total);
        for (int32_t mm = m0; mm < m1; ++mm) {
            mg_off[(int64_t)h * n_seeds + mm] = (int32_t)run;
            run += (uint32_t)c[mm];
        }
        nodes += total;
        if (h == n_layers) break;
        if (threadIdx.x == 0) ent_start[h] = ents;
        const int32_t* e = ecnt + (int64_t)h * n_seeds;
        mine = 0;
        for (int32_t mm = m0; mm < m1; ++mm) mine += (uint32_t)e[mm];
        run = fr_block_scan<kLwChunkThreads, uint32_t>(mine, lds4, total);
        for (int32_t mm = m0; mm < m1; ++mm) {
            mg_eoff[(int64_t)h * n_seeds + mm] = (int32_t)run;
            run += (uint32_t)e[mm];
        }
        ents += total;
    }
    if (threadIdx.x == 0) {
        level_start[n_layers + 1] = nodes;
        ent_start[n_layers] = ents;       // total entries
    }
}

// One thread per staging slot: first the node slots (level h, micrograph, i-th node), then the
// entry slots (level h of the source node, micrograph, i-th entry of that micrograph's level).
__global__ void __launch_bounds__(kLwThreads)
lw_compact(const int32_t* __restrict__ stage_nodes, const int32_t* __restrict__ stage_eoff,
           const int32_t* __restrict__ stage_child, const int32_t* __restrict__ cnt, const int32_t* __restrict__ ecnt,
           const int32_t* __restrict__ mg_off, const int32_t* __restrict__ mg_eoff,
           const int64_t* __restrict__ level_start, const int64_t* __restrict__ ent_start, int32_t n_seeds, LwShape sh,
           int32_t* __restrict__ node_vertex, int32_t* __restrict__ indptr, int32_t* __restrict__ idx,
           uint8_t* __restrict__ present) {
    const int32_t L = sh.n_layers, B = n_seeds;
    const int64_t T = sh.nbase[L + 1], S = sh.nbase[L], E = sh.ebase[L];
    const int64_t t = (int64_t)blockIdx.x * kLwThreads + threadIdx.x;
    const int64_t n_nodes = level_start[L + 1], n_nonleaf = level_start[L], nnz = ent_start[L];
    if (t < T) {
        // unused tails: no vertex, empty segments
        if (t >= n_nodes) node_vertex[t] = -1;
        if (t >= n_nonleaf && t <= S) indptr[t] = (int32_t)nnz;
        int32_t h = 0;
        while (h < L && t >= sh.nbase[h + 1]) ++h;
        const int64_t o = t - sh.nbase[h];
        const int32_t mg = (int32_t)(o / sh.s[h]), i = (int32_t)(o - (int64_t)mg * sh.s[h]);
        if (i >= cnt[(int64_t)h * B + mg]) return;
        const int64_t gi = level_start[h] + mg_off[(int64_t)h * B + mg] + i;
        const int32_t vertex = stage_nodes[t];
        node_vertex[gi] = vertex;
        if (present != nullptr && vertex >= 0) present[vertex] = 1;          // the pre-gather's presence map
        if (h < L) indptr[gi] = (int32_t)(ent_start[h] + mg_eoff[(int64_t)h * B + mg] + stage_eoff[t]);
        return;
    }
    const int64_t e = t - T;
    if (e >= E) return;
    if (e >= nnz) idx[e] = -1;                                // unused tail
    int32_t h = 0;
    while (h < L - 1 && e >= sh.ebase[h + 1]) ++h;
    const int64_t o = e - sh.ebase[h];
    const int64_t per = (int64_t)sh.s[h] * sh.s[h + 1];
    const int32_t mg = (int32_t)(o / per), i = (int32_t)(o - (int64_t)mg * per);
    if (i >= ecnt[(int64_t)h * B + mg]) return;
    idx[ent_start[h] + mg_eoff[(int64_t)h * B + mg] + i] =
        (int32_t)(level_start[h + 1] + mg_off[(int64_t)(h + 1) * B + mg] + stage_child[e]);
}

struct LwWs {
    size_t nodes_bytes, eoff_bytes, child_bytes, cnt_bytes, ecnt_bytes, ent_start_bytes, pref_bytes, len_bytes,
        chunk_bytes, bits_bytes, total;
};
static LwWs lw_ws_layout(int64_t T, int64_t S, int64_t E, int64_t words, int64_t B, int32_t L) {
    LwWs W{};
    W.nodes_bytes = align_up((size_t)T * 4, 256);
    W.eoff_bytes = align_up((size_t)S * 4, 256);
    W.child_bytes = align_up((size_t)E * 4, 256);
    W.cnt_bytes = align_up((size_t)(L + 1) * B * 4, 256);          // once for cnt, once for mg_off
    W.ecnt_bytes = align_up((size_t)L * B * 4, 256);               // once for ecnt, once for mg_eoff
    W.ent_start_bytes = align_up((size_t)(L + 1) * 8, 256);
    W.pref_bytes = align_up((size_t)S * 8, 256);                   // once for the degree sums, once for the list bases
    W.len_bytes = align_up((size_t)L * B * 8, 256);
    W.chunk_bytes = align_up((size_t)(L * B + 1) * 4, 256);
    W.bits_bytes = align_up((size_t)words * 4, 256);
    W.total = W.nodes_bytes + W.eoff_bytes + W.child_bytes + 2 * W.cnt_bytes + 2 * W.ecnt_bytes + W.ent_start_bytes +
              2 * W.pref_bytes + W.len_bytes + W.chunk_bytes + W.bits_bytes;
    return W;
}

// Words of one seed's bit matrices.
static int64_t lw_bit_words(const int32_t* budgets, int32_t n_layers) {
    int64_t words = 0, prev = 1;
    for (int32_t h = 1; h <= n_layers; ++h) {
        words += prev * ((budgets[h - 1] + 31) / 32);
        prev = budgets[h - 1];
    }
    return words;
}

// Per-seed capacities; false if a budget is out of range.
static bool lw_caps(const int32_t* budgets, int32_t n_layers, int64_t caps[3]) {
    if (budgets == nullptr || n_layers < 1 || n_layers > kMaxLayers) return false;
    int64_t nodes = 1, nonleaf = 0, entries = 0, prev = 1;
    for (int32_t h = 1; h <= n_layers; ++h) {
        const int64_t s = budgets[h - 1];
        if (s < 1 || s > kLwMaxLevel || prev * s > kLwMaxPairs) return false;
        nonleaf += prev;
        entries += prev * s;
        nodes += s;
        prev = s;
    }
    caps[0] = nodes;
    caps[1] = nonleaf;
    caps[2] = entries;
    return true;
}

}  // namespace hopgnn

using namespace hopgnn;

extern "C" hopgnn_status hopgnn_layerwise_caps(const int32_t* budgets, int32_t n_layers, int64_t* caps) {
    if (caps == nullptr) return HOPGNN_EINVAL;
    if (budgets == nullptr || n_layers < 1 || n_layers > kMaxLayers) return HOPGNN_EINVAL;
    for (int32_t h = 0; h < n_layers; ++h)
        if (budgets[h] < 1) return HOPGNN_EINVAL;
    return lw_caps(budgets, n_layers, caps) ? HOPGNN_OK : HOPGNN_ERANGE;
}

extern "C" size_t hopgnn_sample_layerwise_ws_bytes(int32_t n_seeds, const int32_t* budgets, int32_t n_layers) {
    int64_t caps[3];
    if (n_seeds < 0 || !lw_caps(budgets, n_layers, caps)) return 0;
    return lw_ws_layout(caps[0] * n_seeds, caps[1] * n_seeds, caps[2] * n_seeds, lw_bit_words(budgets, n_layers) * n_seeds,
                        n_seeds, n_layers).total;
}

extern "C" hopgnn_status hopgnn_sample_layerwise(const hopgnn_csr* g, const int32_t* seeds, int32_t n_seeds,
                                                 int32_t seeds_per_key, const int32_t* budgets, int32_t n_layers,
                                                 const uint64_t* keys, int32_t* node_vertex, int64_t* level_start,
                                                 int32_t* indptr, int32_t* idx, void* ws, size_t ws_bytes, void* stream) {
    return sample_layerwise(g, seeds, n_seeds, seeds_per_key, budgets, n_layers, keys, node_vertex, level_start, indptr,
                            idx, ws, ws_bytes, nullptr, stream);
}

hopgnn_status hopgnn::sample_layerwise(const hopgnn_csr* g, const int32_t* seeds, int32_t n_seeds, int32_t seeds_per_key,
                                       const int32_t* budgets, int32_t n_layers, const uint64_t* keys,
                                       int32_t* node_vertex, int64_t* level_start, int32_t* indptr, int32_t* idx, void* ws,
                                       size_t ws_bytes, uint8_t* present, void* stream) {
    if (g == nullptr || n_seeds < 0 || seeds_per_key < 1) return HOPGNN_EINVAL;
    int64_t caps[3];
    hopgnn_status rc = hopgnn_layerwise_caps(budgets, n_layers, caps);
    if (rc != HOPGNN_OK) return rc;
    if (g->n_vertices < 0 || g->n_edges < 0 || g->n_vertices > ((int64_t)1 << 31)) return HOPGNN_EINVAL;
    if (n_seeds == 0) return HOPGNN_OK;
    if (g->offsets == nullptr || seeds == nullptr || keys == nullptr || node_vertex == nullptr || level_start == nullptr ||
        indptr == nullptr || idx == nullptr || ws == nullptr)
        return HOPGNN_EINVAL;
    if (g->n_edges > 0 && g->indices == nullptr) return HOPGNN_EINVAL;
    const int64_t T = caps[0] * n_seeds, S = caps[1] * n_seeds, E = caps[2] * n_seeds;
    if (T + E >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
    if (!aligned(ws, 256)) return HOPGNN_EINVAL;

    LwShape sh{};
    sh.n_layers = n_layers;
    sh.s[0] = 1;
    sh.nbase[0] = 0;
    sh.ebase[0] = 0;
    sh.wbase[0] = 0;
    for (int32_t h = 1; h <= n_layers; ++h) {
        sh.s[h] = budgets[h - 1];
        sh.nbase[h] = sh.nbase[h - 1] + n_seeds * sh.s[h - 1];
        sh.ebase[h] = sh.ebase[h - 1] + n_seeds * sh.s[h - 1] * sh.s[h];
        sh.wbase[h] = sh.wbase[h - 1] + n_seeds * sh.s[h - 1] * ((sh.s[h] + 31) / 32);
    }
    sh.nbase[n_layers + 1] = sh.nbase[n_layers] + n_seeds * sh.s[n_layers];

    const LwWs W = lw_ws_layout(T, S, E, sh.wbase[n_layers], n_seeds, n_layers);
    if (ws_bytes < W.total) return HOPGNN_ENOMEM_WS;
    char* p = static_cast<char*>(ws);
    auto take = [&p](size_t bytes) {
        char* at = p;
        p += bytes;
        return at;
    };
    int32_t* stage_nodes = reinterpret_cast<int32_t*>(take(W.nodes_bytes));
    int32_t* stage_eoff = reinterpret_cast<int32_t*>(take(W.eoff_bytes));
    int32_t* stage_child = reinterpret_cast<int32_t*>(take(W.child_bytes));
    int32_t* cnt = reinterpret_cast<int32_t*>(take(W.cnt_bytes));
    int32_t* mg_off = reinterpret_cast<int32_t*>(take(W.cnt_bytes));
    int32_t* ecnt = reinterpret_cast<int32_t*>(take(W.ecnt_bytes));
    int32_t* mg_eoff = reinterpret_cast<int32_t*>(take(W.ecnt_bytes));
    int64_t* ent_start = reinterpret_cast<int64_t*>(take(W.ent_start_bytes));
    uint64_t* stage_pref = reinterpret_cast<uint64_t*>(take(W.pref_bytes));
    uint64_t* stage_obase = reinterpret_cast<uint64_t*>(take(W.pref_bytes));
    uint64_t* pair_len = reinterpret_cast<uint64_t*>(take(W.len_bytes));
    uint32_t* chunk_start = reinterpret_cast<uint32_t*>(take(W.chunk_bytes));
    uint32_t* gbits = reinterpret_cast<uint32_t*>(take(W.bits_bytes));

    hipStream_t s = static_cast<hipStream_t>(stream);
    const LwLds lds = lw_lds_layout(sh);
    // drawing is a few dozen hashes and a short sort per hop: narrow workgroups unless the budgets are large
    const int threads = lds.max_s > 256 ? 256 : (lds.max_s > 64 ? 128 : 64);
    const void* off = g->offsets;
    const int32_t n_keys = (int32_t)ceil_div(n_seeds, seeds_per_key);
    for (int32_t k0 = 0; k0 < n_keys; k0 += kLwKeysPerLaunch) {     // 64 keys fit one launch's arguments
        const int32_t nk = n_keys - k0 < kLwKeysPerLaunch ? n_keys - k0 : kLwKeysPerLaunch;
        LwKeys lk{};
        for (int32_t i = 0; i < nk; ++i) lk.keyed[i] = fr_finalise64(keys[k0 + i] + 0x9E3779B97F4A7C15ull);
        const int64_t m0 = (int64_t)k0 * seeds_per_key;
        const int64_t count = (int64_t)nk * seeds_per_key < n_seeds - m0 ? (int64_t)nk * seeds_per_key : n_seeds - m0;
#define HOPGNN_LW_LAUNCH(OffT, THREADS)                                                                             \
    hipLaunchKernelGGL((lw_draw<OffT, THREADS>), dim3((unsigned)count), dim3(THREADS), lds.draw_bytes, s,            \
                       static_cast<const OffT*>(off), g->indices, seeds, n_seeds, sh, lk, (int32_t)m0, seeds_per_key, \
                       lds.max_s, lds.cap2, stage_nodes, stage_pref, stage_obase, pair_len, gbits, cnt)
        if (g->offsets_i64) {
            if (threads == 256) HOPGNN_LW_LAUNCH(int64_t, 256);
            else if (threads == 128) HOPGNN_LW_LAUNCH(int64_t, 128);
            else HOPGNN_LW_LAUNCH(int64_t, 64);
        } else {
            if (threads == 256) HOPGNN_LW_LAUNCH(int32_t, 256);
            else if (threads == 128) HOPGNN_LW_LAUNCH(int32_t, 128);
            else HOPGNN_LW_LAUNCH(int32_t, 64);
        }
#undef HOPGNN_LW_LAUNCH
        HOPGNN_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(lw_chunks, dim3(1), dim3(kLwChunkThreads), 0, s, pair_len, n_layers * n_seeds, chunk_start);
    HOPGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(lw_adjacency, dim3(kLwAdjGrid), dim3(kLwThreads), lds.adj_bytes, s, g->indices, n_seeds, sh,
                       lds.max_s, lds.filt_words, stage_nodes, stage_pref, stage_obase, pair_len, chunk_start, cnt, gbits);
    HOPGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(lw_segments, dim3((unsigned)n_seeds), dim3(kLwSegThreads), 0, s, n_seeds, sh, gbits, cnt, stage_eoff,
                       stage_child, ecnt);
    HOPGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(lw_scan, dim3(1), dim3(kLwChunkThreads), 0, s, cnt, ecnt, n_seeds, n_layers, mg_off, mg_eoff,
                       level_start, ent_start);
    HOPGNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(lw_compact, dim3((unsigned)ceil_div(T + E, kLwThreads)), dim3(kLwThreads), 0, s, stage_nodes,
                       stage_eoff, stage_child, cnt, ecnt, mg_off, mg_eoff, level_start, ent_start, n_seeds, sh,
                       node_vertex, indptr, idx, present);
    HOPGNN_LAUNCH_CHECK();
    return HOPGNN_OK;
}
