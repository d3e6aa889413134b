/*
 * hopgnn.h - C ABI of the MI355X (gfx950) micrograph hot path of HopGNN
 * (arxiv 2409.00657): one worker's share of a micrograph-based training step
 * on one GPU.
 *
 *   hopgnn_sample     k-hop neighbour sampling, one micrograph per root vertex
 *   hopgnn_pregather  merged, duplicate-free vertex-ID set of a batch (or a
 *                     group of batches) of micrographs + slot -> position table
 *   hopgnn_gather     copy of the feature rows of that set into a dense buffer
 *   hopgnn_sage_fwd   one GraphSAGE-mean layer: CSR segmented mean of neighbour
 *                     rows, then the W_self / W_neigh projection
 *
 * Conventions for every call
 *   - Pointers marked DEVICE are HIP device pointers owned by the caller; the
 *     library never allocates, frees or keeps them.  Pointers marked HOST are
 *     ordinary host memory read during the call.
 *   - `stream` is a hipStream_t passed as void*; all device work is enqueued on
 *     it and no call synchronises.  The library holds no global state.
 *   - Argument errors that the host can see are reported before any launch.
 *     Vertex IDs inside device arrays are the caller's contract: they must lie
 *     in [0, n_vertices) (or be negative = "invalid slot" where allowed).
 *   - Results are pure functions of the inputs and bit-stable from run to run
 *     (no result depends on the order in which atomics land).
 */
#ifndef HOPGNN_H
#define HOPGNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HOPGNN_OK = 0,
    HOPGNN_EINVAL = 1,    /* NULL / negative / inconsistent argument            */
    HOPGNN_ENOMEM_WS = 2, /* workspace smaller than the *_ws_bytes query         */
    HOPGNN_ERANGE = 3,    /* a size exceeds what the 32-bit slot arrays can hold */
    HOPGNN_EHIP = 4       /* a HIP launch failed                                 */
} hopgnn_status;

typedef enum { HOPGNN_F32 = 0, HOPGNN_BF16 = 1, HOPGNN_F16 = 2 } hopgnn_dtype;

/* neighbour aggregators of hopgnn_sage_fwd_agg */
typedef enum { HOPGNN_AGG_MEAN = 0, HOPGNN_AGG_SUM = 1, HOPGNN_AGG_MAX = 2 } hopgnn_agg;

/* How hopgnn_pregather builds the set. Both give identical results. */
typedef enum {
    HOPGNN_PG_AUTO = 0,   /* bitmap unless n_vertices > 133e6 + 42 * n_ids               */
    HOPGNN_PG_BITMAP = 1, /* presence bitmap over the vertex range + popcount ranks     */
    HOPGNN_PG_RADIX = 2   /* LSD radix sort of (id, slot) pairs, head flags, scan       */
} hopgnn_pg_algo;

/* Read-only graph topology in CSR form (replicated per worker in the paper,
 * section 2, because it is small next to the features). Row v lists the
 * vertices that v samples from and aggregates over. */
typedef struct {
    int64_t n_vertices;
    int64_t n_edges;
    const void *offsets;    /* DEVICE [n_vertices+1], int32 or int64 (see offsets_i64) */
    int32_t offsets_i64;    /* 0: int32 offsets, 1: int64 offsets                      */
    const int32_t *indices; /* DEVICE [n_edges]                                        */
} hopgnn_csr;

const char *hopgnn_status_str(hopgnn_status s);

/*
 * Slots per micrograph, T_seed = sum_{h=0..L} P_h, P_0 = 1, P_h = f_1*...*f_h
 * (fanouts[0] applies at the root).  Returns -1 if n_layers < 1 or n_layers > 8
 * or any fanout < 1.  HOST only.
 */
int64_t hopgnn_slots_per_seed(const int32_t *fanouts /*HOST*/, int32_t n_layers);

/*
 * Sampling (paper section 2 "sampling"; section 4 "micrograph definition": a
 * k-hop computation graph per root vertex of the mini-batch).
 *
 * For each of the n_seeds roots a fixed-shape tree of slots is filled, with
 * replacement:  child j (0-based) at hop h (1-based) of a slot holding vertex v
 * in the micrograph of root r is
 *     indices[offsets[v] + hash64(key, r, v, h, j) mod deg(v)]
 * (exact unsigned 64-bit remainder), or -1 if v < 0 or deg(v) = 0.  hash64 is a
 * three-step chain of the SplitMix64 finaliser absorbing key, (r,v), (h,j).
 *
 * ids    DEVICE out [n_seeds*T_seed] level-major: level h holds n_seeds*P_h
 *        slots starting at n_seeds*sum_{i<h} P_i; in a level the slot of seed m,
 *        path p is m*P_h + p; children of level-local slot q are q*f_h .. +f_h-1.
 * indptr DEVICE out [S+1], S = number of non-leaf slots, or NULL: children of
 *        slot r are ids[n_seeds + indptr[r] .. n_seeds + indptr[r+1]).
 * slot_idx DEVICE out [S - n_seeds] or NULL: for e below S - n_seeds (the
 *        children that are themselves non-leaf slots), n_seeds + e if
 *        ids[n_seeds + e] >= 0, else -1.  (indptr, slot_idx) is the CSR of the
 *        computation graph in slot numbering: the neighbour list a layer after
 *        the first aggregates over, whose input row of a slot is the slot number.
 * seeds  DEVICE [n_seeds], each in [0, n_vertices).
 * Errors: EINVAL (NULL, n_seeds < 0, bad fanouts), ERANGE (n_seeds*T_seed >= 2^31).
 * n_seeds == 0 is a no-op returning OK.
 */
hopgnn_status hopgnn_sample(const hopgnn_csr *g /*HOST struct*/, const int32_t *seeds,
                            int32_t n_seeds, const int32_t *fanouts /*HOST*/, int32_t n_layers,
                            uint64_t key, int32_t *ids, int32_t *indptr, int32_t *slot_idx,
                            void *stream);

/*
 * The micrographs of several batches of one shape in one launch (paper section 5.2 gathers for
 * the micrographs of several time steps at once; their sampling is independent work of the same
 * shape).  Exactly n_batches calls of hopgnn_sample: batch b reads seeds[b*n_seeds ..], uses
 * keys[b] (HOST array) and writes ids[b*T ..] (T = n_seeds * slots per seed) and, if slot_idx is
 * not NULL, slot_idx[b*slot_idx_stride ..] (stride >= T - n_seeds - last level, i.e. the entries
 * one batch writes); indptr is the same for every batch and is written once.
 * HOPGNN_ERANGE if n_batches * T does not fit the 32-bit slot arrays.
 */
/*
 * The same micrographs as hopgnn_sample_group, laid out as ONE level-major batch of n_seeds
 * micrographs in which micrograph m draws with keys[m / seeds_per_key] (HOST array of
 * ceil(n_seeds / seeds_per_key) keys): block b of seeds_per_key consecutive seeds is exactly the
 * batch hopgnn_sample(seeds + b*seeds_per_key, seeds_per_key, ..., keys[b]) would sample, only the
 * slots of all blocks share one level-major array, so that a layer runs once over all of them
 * (micrograph merging, paper section 5.3: fewer, fuller steps).  ids [n_seeds * slots per seed],
 * indptr and slot_idx as in hopgnn_sample for n_seeds seeds.
 */
hopgnn_status hopgnn_sample_merged(const hopgnn_csr *g /*HOST struct*/, const int32_t *seeds, int32_t n_seeds,
                                   int32_t seeds_per_key, const int32_t *fanouts /*HOST*/, int32_t n_layers,
                                   const uint64_t *keys /*HOST*/, int32_t *ids, int32_t *indptr,
                                   int32_t *slot_idx, void *stream);

hopgnn_status hopgnn_sample_group(const hopgnn_csr *g /*HOST struct*/, const int32_t *seeds, int32_t n_seeds,
                                  const int32_t *fanouts /*HOST*/, int32_t n_layers,
                                  const uint64_t *keys /*HOST*/, int32_t n_batches, int32_t *ids,
                                  int32_t *indptr, int32_t *slot_idx, int64_t slot_idx_stride, void *stream);

/*
 * Pre-gathering (paper section 5.2: merge the fetches of all micrographs a
 * worker trains in one iteration into one, each vertex once; implementation
 * section: duplicates are removed from the stored list of micrographs).
 *
 * ids        DEVICE [n_ids]; concatenation of one or more batches' slot arrays;
 *            negative entries are invalid slots and are skipped.
 * uniq       DEVICE out, capacity min(n_ids, n_vertices): valid IDs, strictly ascending.
 * n_uniq_dev DEVICE out, one int64: U = number of entries written to uniq.
 * remap      DEVICE out [n_ids]: position of ids[i] in uniq, -1 for invalid slots.
 * ws         DEVICE scratch of at least hopgnn_pregather_ws_bytes(...) bytes,
 *            256-byte aligned; contents on entry are irrelevant.
 * Errors: EINVAL, ENOMEM_WS, ERANGE (n_ids >= 2^31 or n_vertices > 2^31).
 */
size_t hopgnn_pregather_ws_bytes(int64_t n_ids, int64_t n_vertices, int32_t algo);

/*
 * k-hop sampling with per-micrograph deduplicated frontiers (paper section 4: a micrograph is the
 * set of vertices its sampling reaches, counted once each).  The same draws as hopgnn_sample - the
 * children of a vertex depend only on (key, root, vertex, hop, j), so equal vertices at one level of
 * one micrograph carry identical subtrees in the slot tree - but every (level, vertex) pair of a
 * micrograph is kept once, so the layers run over fewer rows and give the same rows for the roots.
 *
 * Nodes are numbered level-major: level 0 of every micrograph (the roots, in seed order), then level
 * 1 of every micrograph, ...; inside one micrograph's level the vertices ascend.
 *   node_vertex DEVICE out [T]     vertex of every node; entries past the node count are -1
 *                                  (T = n_seeds * hopgnn_slots_per_seed: the slot tree's size is the
 *                                  capacity), so the array can go to hopgnn_pregather as it is
 *   level_start DEVICE out int64 [n_layers + 2]   first node of level h; [n_layers + 1] = node count.
 *                                  Layer k (1-based) has level_start[n_layers - k + 1] destination rows
 *                                  (the nodes of levels 0 .. n_layers - k): pass its address as
 *                                  n_dst_dev of hopgnn_sage_fwd_dev
 *   indptr      DEVICE out [S + 1] S = T minus the last level; segment of node i = its children in
 *                                  draw order (fanout many, parallel edges kept); entries past the
 *                                  non-leaf node count equal the total, i.e. empty segments
 *   idx         DEVICE out [T - n_seeds]   child NODE index or -1 (the vertex has no neighbours);
 *                                  entries past the total are -1
 *   ws          DEVICE scratch, hopgnn_sample_dedup_ws_bytes, 256-byte aligned
 * Micrograph m draws with keys[m / seeds_per_key] (HOST array of ceil(n_seeds / seeds_per_key)
 * keys), as in hopgnn_sample_merged: one key for the whole batch is seeds_per_key = n_seeds.
 * One level of one micrograph may hold at most 4096 slots (product of the fanouts), else
 * HOPGNN_ERANGE.  Other errors as hopgnn_sample.
 *
 * hopgnn_compose_idx: out[e] = idx[e] >= 0 ? map[idx[e]] : -1 - the first layer reads the
 * pre-gathered rows, so its neighbour list is the node list's remap applied to the child indices.
 */
size_t hopgnn_sample_dedup_ws_bytes(int32_t n_seeds, const int32_t *fanouts /*HOST*/, int32_t n_layers);

hopgnn_status hopgnn_sample_dedup(const hopgnn_csr *g /*HOST struct*/, const int32_t *seeds, int32_t n_seeds,
                                  int32_t seeds_per_key, const int32_t *fanouts /*HOST*/, int32_t n_layers,
                                  const uint64_t *keys /*HOST*/, int32_t *node_vertex, int64_t *level_start, int32_t *indptr, int32_t *idx,
                                  void *ws, size_t ws_bytes, void *stream);

hopgnn_status hopgnn_compose_idx(const int32_t *idx, int64_t n, const int32_t *map, int32_t *out, void *stream);

/*
 * Layer-wise sampling of micrographs (paper section 4 measures micrograph locality under node-wise
 * and under layer-wise sampling; the paper gives no detail beyond naming the sampler, so this is the
 * reading taken).  Per micrograph and hop h a budget of budgets[h-1] draws is made for the whole
 * layer: position p_j = hash64(key, root, 0xFFFFFFFF, h, j) mod D in the concatenation of the
 * neighbour lists of the previous level's nodes (node order, list order; D = its length), with
 * replacement, so a vertex is drawn with probability proportional to the number of edges from the
 * previous level into it.  The level's nodes are the distinct drawn vertices, ascending (none if
 * D = 0).  Every edge between the two node sets is kept, each (node, node) pair once: the segment of
 * a previous-level node lists, in ascending order, the level's nodes adjacent to it.
 *
 * Output in the layout of hopgnn_sample_dedup (level-major node numbering, level_start, CSR of node
 * indices; the layers run through hopgnn_sage_fwd_dev in the same way), with segments of varying
 * length and no -1 entries.  Capacities per seed come from hopgnn_layerwise_caps:
 *   caps[0] nodes     = 1 + sum of the budgets           node_vertex [n_seeds * caps[0]], tail -1
 *   caps[1] non-leaf  = caps[0] - the last budget        indptr [n_seeds * caps[1] + 1], tail = total
 *   caps[2] entries   = sum of budgets[h-1] * budgets[h] (budgets[-1] = 1)
 *                                                        idx [n_seeds * caps[2]], tail -1
 * level_start DEVICE out int64 [n_layers + 2] as in hopgnn_sample_dedup; keys, seeds_per_key, ws
 * (hopgnn_sample_layerwise_ws_bytes, 256-byte aligned) likewise.
 * Limits: a budget is at most 1024 and the product of two consecutive budgets at most 65536, else
 * HOPGNN_ERANGE (hopgnn_layerwise_caps reports it too; the ws size is then 0).  Other errors as
 * hopgnn_sample.
 */
hopgnn_status hopgnn_layerwise_caps(const int32_t *budgets /*HOST*/, int32_t n_layers, int64_t *caps /*HOST out [3]*/);

size_t hopgnn_sample_layerwise_ws_bytes(int32_t n_seeds, const int32_t *budgets /*HOST*/, int32_t n_layers);

hopgnn_status hopgnn_sample_layerwise(const hopgnn_csr *g /*HOST struct*/, const int32_t *seeds, int32_t n_seeds,
                                      int32_t seeds_per_key, const int32_t *budgets /*HOST*/, int32_t n_layers,
                                      const uint64_t *keys /*HOST*/, int32_t *node_vertex, int64_t *level_start,
                                      int32_t *indptr, int32_t *idx, void *ws, size_t ws_bytes, void *stream);

/*
 * hopgnn_micrograph_locality (below) for the micrographs of a frontier structure, as written by
 * hopgnn_sample_dedup or hopgnn_sample_layerwise - the paper's locality table has rows for
 * node-wise and for layer-wise sampling.  The micrograph of seed m is every node reachable from node
 * m through the structure's entries:
 *   n_total[m] = its distinct vertices, n_coloc[m] = its distinct vertices other than the root
 *   whose home server owner[v] is the root's.
 * nodes_per_seed: the capacity of one micrograph (hopgnn_slots_per_seed or caps[0] of
 * hopgnn_layerwise_caps); it sizes the per-micrograph hash set in LDS (the next power of two at or
 * above 2 * nodes_per_seed cells), at most 16384, else ERANGE.  A micrograph that has more distinct
 * vertices than the set has cells cannot be counted: it reports n_total[m] = n_coloc[m] = -1
 * (never a wrong count); with the sampler's own capacity that cannot happen.
 * level_start is the DEVICE array the sampler wrote; owner DEVICE [n_vertices] int32; n_total,
 * n_coloc DEVICE out [n_seeds].
 */
hopgnn_status hopgnn_frontier_locality(const int32_t *node_vertex, const int64_t *level_start, const int32_t *indptr,
                                       const int32_t *idx, int32_t n_seeds, int32_t n_layers, int64_t nodes_per_seed,
                                       const int32_t *owner, int32_t *n_total, int32_t *n_coloc, void *stream);

/*
 * Prepares a pre-gather workspace once (zero presence map and counters; sizes and algo as in
 * hopgnn_pregather_ws_bytes).  hopgnn_pregather itself does not need it - it clears what it uses
 * - but every call of it, and every hopgnn_batch_fwd, leaves the workspace as this call does, so
 * a plan may promise a clean workspace (pg_ws_clean) and skip the clearing pass.  A call that
 * fails part-way may leave marks behind: call this again.
 */
hopgnn_status hopgnn_pregather_ws_init(void *ws, size_t ws_bytes, int64_t n_ids, int64_t n_vertices,
                                       int32_t algo, void *stream);

hopgnn_status hopgnn_pregather(const int32_t *ids, int64_t n_ids, int64_t n_vertices,
                               int32_t algo, int32_t *uniq, int64_t *n_uniq_dev, int32_t *remap,
                               void *ws, size_t ws_bytes, void *stream);

/*
 * hopgnn_pregather for callers that cannot allocate device memory or provide a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation): the same
 * kernels and the same results (bitmap path), with the scratch in a static device array of
 * 24 MiB that every GPU the library runs on holds until the process ends.  Calls no allocator.
 * Limit: n_vertices <= hopgnn_pregather_static_max_vertices() = 2^24, else HOPGNN_ERANGE;
 * other errors as hopgnn_pregather.  All calls on one GPU share that GPU's array: calls that
 * overlap in time on one GPU (different streams) race; the contents a call leaves behind are
 * cleared by the next call before use.  The first call on a device looks the array's address
 * up (hipGetSymbolAddress) with that device current.
 */
int64_t hopgnn_pregather_static_max_vertices(void);
hopgnn_status hopgnn_pregather_static(const int32_t *ids, int64_t n_ids, int64_t n_vertices, int32_t *uniq,
                                      int64_t *n_uniq_dev, int32_t *remap, void *stream);

/*
 * Data locality of micrographs (paper section 4, "data locality in micrographs": the
 * ratio R_micro = N_colocated / N_total of the locality table).
 * For every micrograph m of one batch (ids as written by hopgnn_sample):
 *   n_total[m] = number of distinct vertices among its valid slots,
 *   n_coloc[m] = number of distinct vertices other than the root whose home server
 *                owner[v] equals the root's, owner[ids[m]].
 * (The section's worked example also counts the root as local: n_coloc + 1.)
 * ids   DEVICE [n_seeds*T_seed]; owner DEVICE [n_vertices] int32;
 * n_total, n_coloc DEVICE out [n_seeds].
 * Errors: EINVAL; ERANGE if T_seed > 16384 (the per-micrograph hash set lives in LDS).
 */
hopgnn_status hopgnn_micrograph_locality(const int32_t *ids, int32_t n_seeds, const int32_t *fanouts /*HOST*/,
                                         int32_t n_layers, const int32_t *owner, int32_t *n_total,
                                         int32_t *n_coloc, void *stream);

/*
 * Owner split of a pre-gathered set (paper section 5.2: only vertices that are not stored
 * on the worker's own server are fetched; section 7.3: miss rate of feature gathering =
 * non-local requests / all requests).
 * remote       DEVICE out, capacity n_uniq: the entries of uniq with owner != server, in
 *              order (so still ascending);
 * n_remote_dev DEVICE out, one int64: their number; miss rate = n_remote / U.
 * n_uniq / n_uniq_dev as in hopgnn_gather (capacity + device count, or the count itself).
 * ws           DEVICE scratch, hopgnn_split_ws_bytes(n_uniq) bytes, 256-byte aligned.
 */
size_t hopgnn_split_ws_bytes(int64_t n_uniq);

hopgnn_status hopgnn_split_by_owner(const int32_t *uniq, int64_t n_uniq, const int64_t *n_uniq_dev,
                                    const int32_t *owner, int32_t server, int32_t *remote,
                                    int64_t *n_remote_dev, void *ws, size_t ws_bytes, void *stream);

/*
 * Gathering (paper section 2 "gathering": collect the feature vector of every
 * vertex of the sampled structure; section 3.1 names it the bottleneck).
 *
 *     Xu[i, :] = X[uniq[i], :]   for i < U, byte for byte.
 *
 * X          DEVICE [n_rows x dim] row-major, rows ld_elems elements apart.
 * uniq       DEVICE [U] row numbers in [0, n_rows).
 * n_uniq     if n_uniq_dev is NULL: U itself.  Otherwise the capacity of uniq/Xu
 *            (an upper bound of U used to size the launch) and U is read on the
 *            device from *n_uniq_dev, so no host synchronisation is needed.
 * Xu         DEVICE out [U x dim], packed.
 * Rows move as 128-bit words when base addresses, dim*size and ld*size are all
 * multiples of 16 bytes, else as 32-bit words, else as bytes.
 */
hopgnn_status hopgnn_gather(const void *X, hopgnn_dtype dt, int64_t n_rows, int32_t dim,
                            int64_t ld_elems, const int32_t *uniq, int64_t n_uniq,
                            const int64_t *n_uniq_dev, void *Xu, void *stream);

/*
 * GraphSAGE-mean layer forward (paper section 2 "computation": per layer an
 * aggregation over each vertex's neighbours, then a neural-network transform;
 * the aggregator is the mean of Hamilton et al.'s GraphSAGE):
 *
 *   c_r    = #{ e in [indptr[r], indptr[r+1]) : idx[e] >= 0 }
 *   m_r    = (1/c_r) * sum over those e of Hsrc[idx[e], :]      (0 if c_r = 0)
 *   out[r] = act( x_r W_self + m_r W_neigh + bias ),  x_r = Hsrc[self_idx[r], :]
 *
 * Hsrc     DEVICE [n_src x d_in], packed rows, dtype dt.
 * self_idx DEVICE [n_dst] or NULL (= identity: x_r = Hsrc[r], which needs n_src >= n_dst,
 *          else HOPGNN_EINVAL); a negative entry gives a zero self row.
 * indptr   DEVICE [n_dst+1], idx DEVICE [indptr[n_dst]]; negative idx = skip.
 * W_self, W_neigh DEVICE [d_in x d_out] row-major, dtype dt; bias DEVICE [d_out] or NULL.
 * relu     0: identity activation, else max(., 0).
 * out      DEVICE [n_dst x d_out], dtype dt (sums are fp32, rounded once on store;
 *          for 2-byte types the mean is rounded to dt before the projection).
 * ws       DEVICE scratch of at least hopgnn_sage_fwd_ws_bytes(...) bytes, 256-byte aligned.
 * The sum over a segment runs in entry order, so results are run-to-run stable.
 * Errors: EINVAL, ENOMEM_WS, ERANGE (n_dst or n_src >= 2^31).
 */
size_t hopgnn_sage_fwd_ws_bytes(hopgnn_dtype dt, int64_t n_dst, int32_t d_in, int32_t d_out);

hopgnn_status hopgnn_sage_fwd(const void *Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                              const int32_t *self_idx, const int32_t *indptr, const int32_t *idx,
                              int64_t n_dst, const void *W_self, const void *W_neigh,
                              const void *bias, int32_t d_out, int32_t relu, void *out, void *ws,
                              size_t ws_bytes, void *stream);

/*
 * hopgnn_sage_fwd with another neighbour aggregator (the paper's discussion of generality names
 * sum and max beside the mean):  m_r = mean, sum or element-wise maximum of Hsrc[idx[e]] over the
 * valid entries of row r (0 for an empty segment), out[r] = act(x_r W_self + m_r W_neigh + bias).
 * agg is a hopgnn_agg; HOPGNN_AGG_MEAN is hopgnn_sage_fwd itself.  Same arguments, workspace
 * (hopgnn_sage_fwd_ws_bytes) and errors; for 2-byte types m_r is rounded to dt before the product.
 */
hopgnn_status hopgnn_sage_fwd_agg(const void *Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                  const int32_t *self_idx, const int32_t *indptr, const int32_t *idx,
                                  int64_t n_dst, const void *W_self, const void *W_neigh, const void *bias,
                                  int32_t d_out, int32_t agg, int32_t relu, void *out, void *ws,
                                  size_t ws_bytes, void *stream);

/*
 * hopgnn_sage_fwd_agg for a row count that only the device knows: n_dst is the capacity the launch
 * is sized for and *n_dst_dev (DEVICE, NULL = n_dst) the number of destination rows that exist;
 * rows past it are neither read nor written.  Used with hopgnn_sample_dedup, whose level sizes
 * depend on the data.  The identity-self check (n_src >= n_dst) applies to the capacity.
 */
hopgnn_status hopgnn_sage_fwd_dev(const void *Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                  const int32_t *self_idx, const int32_t *indptr, const int32_t *idx,
                                  int64_t n_dst, const int64_t *n_dst_dev, const void *W_self,
                                  const void *W_neigh, const void *bias, int32_t d_out, int32_t agg,
                                  int32_t relu, void *out, void *ws, size_t ws_bytes, void *stream);

/*
 * The other two layer types the paper's evaluation trains (experimental setup: GCN, GraphSAGE,
 * GAT; section 2 describes a layer as an aggregation - addition or averaging - over the sampled
 * neighbours followed by a neural transform).  Same inputs as hopgnn_sage_fwd (Hsrc, self_idx,
 * indptr, idx: see there), one weight matrix W DEVICE [d_in x d_out] of type dt.
 *
 * hopgnn_gcn_fwd   out[r] = act( agg_r W + bias ),
 *     agg_r = x_r + sum of Hsrc[idx[e]] over the valid entries e of row r     (norm = 0)
 *     agg_r = that sum / (number of terms)                                     (norm = 1)
 *   i.e. (A+I) H W and D^-1 (A+I) H W on the sampled block, parallel edges counted.  A negative
 *   self index adds nothing and is not counted; no terms gives agg_r = 0.  For 2-byte types
 *   agg_r is rounded to dt before the product.
 *
 * hopgnn_gat_fwd   graph attention with n_heads heads (1..16, d_out divisible by it) of width
 *   d_head = d_out / n_heads, concatenated:  z_u = Hsrc[u] W (computed once per SOURCE row and
 *   kept in fp32 whatever dt is);  score(r,u,h) = LeakyReLU_0.2( <z_self(r)[h], a_dst[h]> + <z_u[h], a_src[h]> );
 *   alpha = softmax of the scores over {self(r)} + the valid entries of row r (parallel edges
 *   kept; a negative self index is left out and its a_dst term is 0);
 *   out[r,h] = act( sum alpha z_u[h] + bias[h] ); a row without entries gives act(bias).
 *   a_src, a_dst DEVICE [d_out] of type dt (head-major, like the columns of W).
 *   n_src_dev: DEVICE count of the source rows that exist (at most n_src), or NULL for n_src: when
 *   Hsrc is a pre-gathered buffer of capacity n_src whose row count hopgnn_pregather left on the
 *   device, only those rows are projected.
 *
 * bias DEVICE [d_out] or NULL; out DEVICE [n_dst x d_out] of type dt; ws DEVICE scratch of the
 * matching *_ws_bytes query (note that the attention layer's is sized by n_src), 256-byte
 * aligned.  Errors as for hopgnn_sage_fwd.
 */
size_t hopgnn_gcn_fwd_ws_bytes(hopgnn_dtype dt, int64_t n_dst, int32_t d_in, int32_t d_out);

hopgnn_status hopgnn_gcn_fwd(const void *Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                             const int32_t *self_idx, const int32_t *indptr, const int32_t *idx,
                             int64_t n_dst, const void *W, const void *bias, int32_t d_out, int32_t norm,
                             int32_t relu, void *out, void *ws, size_t ws_bytes, void *stream);

size_t hopgnn_gat_fwd_ws_bytes(hopgnn_dtype dt, int64_t n_src, int32_t d_in, int32_t d_out, int32_t n_heads);

hopgnn_status hopgnn_gat_fwd(const void *Hsrc, hopgnn_dtype dt, int64_t n_src, const int64_t *n_src_dev,
                             int32_t d_in, const int32_t *self_idx, const int32_t *indptr, const int32_t *idx,
                             int64_t n_dst, const void *W, const void *a_src, const void *a_dst,
                             const void *bias, int32_t d_out, int32_t n_heads, int32_t relu, void *out,
                             void *ws, size_t ws_bytes, void *stream);

/*
 * hopgnn_gcn_fwd and hopgnn_gat_fwd for a destination row count that only the device knows (the
 * layers over hopgnn_sample_dedup's or hopgnn_sample_layerwise's micrographs): n_dst is the
 * capacity, *n_dst_dev (DEVICE, NULL = n_dst) the rows that exist; rows past it are neither read nor
 * written.  Everything else as in the calls without _dev.
 */
hopgnn_status hopgnn_gcn_fwd_dev(const void *Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                 const int32_t *self_idx, const int32_t *indptr, const int32_t *idx, int64_t n_dst,
                                 const int64_t *n_dst_dev, const void *W, const void *bias, int32_t d_out,
                                 int32_t norm, int32_t relu, void *out, void *ws, size_t ws_bytes, void *stream);

hopgnn_status hopgnn_gat_fwd_dev(const void *Hsrc, hopgnn_dtype dt, int64_t n_src, const int64_t *n_src_dev,
                                 int32_t d_in, const int32_t *self_idx, const int32_t *indptr, const int32_t *idx,
                                 int64_t n_dst, const int64_t *n_dst_dev, const void *W, const void *a_src,
                                 const void *a_dst, const void *bias, int32_t d_out, int32_t n_heads, int32_t relu,
                                 void *out, void *ws, size_t ws_bytes, void *stream);

/*
 * GraphSAGE-mean layer backward with in-place gradient accumulation (paper section 5.1,
 * steps 3-4: every micrograph batch runs forward and backward on the server it sits on and
 * the gradients are accumulated until the subgraph is done; discussion section: the
 * accumulated partial gradients are updated in place).  With the forward call's Hsrc,
 * self_idx, indptr, idx, W_self, W_neigh and dOut = dL/d out:
 *
 *   dZ        = dOut where out_fwd > 0 (relu != 0), else dOut
 *   gW_self  += x_self^T dZ      gW_neigh += mean^T dZ      gbias += column sums of dZ
 *   dHsrc     = 0;  dHsrc[self_idx[r]] += dZ[r] W_self^T;
 *               dHsrc[idx[e]] += (dZ[r] W_neigh^T) / c_r  for every valid entry e of row r
 *
 * dt       type of Hsrc, W_self, W_neigh and out_fwd (fp32, bf16 or fp16).  Every gradient is
 *          fp32 in memory whatever dt is; the neighbour mean is rounded to dt as in the forward
 *          call.  With a 2-byte dt the two matrix products (weight gradient, input gradient) take
 *          the masked incoming gradient rounded to dt and accumulate in fp32 (2-byte matrix
 *          instructions; feature widths that are not multiples of 8 use fp32 products of the
 *          widened values instead); the bias gradient sums the fp32 values.
 * out_fwd  DEVICE [n_dst x d_out] of type dt, the stored forward output (decides the ReLU
 *          mask); may be NULL when relu == 0.
 * dOut     DEVICE [n_dst x d_out] fp32.
 * gW_self, gW_neigh DEVICE [d_in x d_out] fp32 accumulators, ADDED to (the caller zeroes them
 *          at the start of an iteration); gbias DEVICE [d_out] fp32 accumulator or NULL.
 *          Bit-stable from run to run (partial sums are combined in a fixed order).
 * dHsrc    DEVICE out [n_src x d_in] fp32 (overwritten), or NULL when the gradient of the
 *          layer input is not needed (the first layer: features are not trained).  Uses float
 *          atomic adds: bit-stable when every source row receives at most two contributions
 *          (true for hopgnn_sample's slot trees), else the rounding depends on arrival order.
 * ws       DEVICE scratch of hopgnn_sage_bwd_ws_bytes(dt, n_dst, d_in, d_out, dHsrc != NULL) bytes.
 */
size_t hopgnn_sage_bwd_ws_bytes(hopgnn_dtype dt, int64_t n_dst, int32_t d_in, int32_t d_out, int32_t want_dh);

hopgnn_status hopgnn_sage_bwd(const void *Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                              const int32_t *self_idx, const int32_t *indptr, const int32_t *idx,
                              int64_t n_dst, const void *W_self, const void *W_neigh, const void *out_fwd,
                              int32_t relu, const float *dOut, int32_t d_out, float *gW_self,
                              float *gW_neigh, float *gbias, float *dHsrc, void *ws, size_t ws_bytes,
                              void *stream);

/*
 * Backward of the other layer kinds the forward path offers (the aggregators the paper's
 * discussion of generality names next to the mean; the GCN-style layer of its evaluation), for
 * the same training loop (section 5.1, steps 3-4).  Gradient types, the rounding of the aggregate
 * and of the products, accumulation into gW / gbias, the meaning of dHsrc (overwritten, or NULL),
 * the workspace (hopgnn_sage_bwd_ws_bytes of the same sizes) and the errors are those of
 * hopgnn_sage_bwd.
 *
 * hopgnn_sage_bwd_agg   the layer of hopgnn_sage_fwd_agg; agg is a hopgnn_agg (MEAN is
 *     hopgnn_sage_bwd itself).  SUM hands every valid entry the whole of dZ[r] W_neigh^T; MAX
 *     hands each column of it to the entry that supplied the maximum, the first one in entry
 *     order among equal values (the one the forward pass keeps).  Other agg values: EINVAL.
 * hopgnn_gcn_bwd        the layer of hopgnn_gcn_fwd: gW += agg^T dZ, and the self row and every
 *     valid entry receive (dZ[r] W^T) / t with t the number of terms (norm = 1) or 1 (norm = 0);
 *     gW DEVICE [d_in x d_out] fp32 accumulator.  norm other than 0 or 1: EINVAL.
 * dHsrc is accumulated with float atomic adds after a clearing pass: bit-stable when a source row
 * receives at most two contributions, otherwise the rounding depends on arrival order.
 */
hopgnn_status hopgnn_sage_bwd_agg(const void *Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                  const int32_t *self_idx, const int32_t *indptr, const int32_t *idx,
                                  int64_t n_dst, const void *W_self, const void *W_neigh, const void *out_fwd,
                                  int32_t agg, int32_t relu, const float *dOut, int32_t d_out, float *gW_self,
                                  float *gW_neigh, float *gbias, float *dHsrc, void *ws, size_t ws_bytes,
                                  void *stream);

hopgnn_status hopgnn_gcn_bwd(const void *Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                             const int32_t *self_idx, const int32_t *indptr, const int32_t *idx, int64_t n_dst,
                             const void *W, const void *out_fwd, int32_t norm, int32_t relu, const float *dOut,
                             int32_t d_out, float *gW, float *gbias, float *dHsrc, void *ws, size_t ws_bytes,
                             void *stream);

/*
 * hopgnn_gat_bwd   backward of the layer of hopgnn_gat_fwd (the attention model of the paper's
 * evaluation, in the training loop of section 5.1, steps 3-4): the chain rule through the weighted
 * sum, the softmax over each destination row's entries, LeakyReLU_0.2, the two score products
 * and z = Hsrc W.
 * fwd_ws   DEVICE: the workspace of the hopgnn_gat_fwd call of this layer on the same inputs,
 *          untouched since (z and the attention scores are read from its first
 *          hopgnn_gat_fwd_ws_bytes(...) bytes); 256-byte aligned.
 * n_src_dev DEVICE, or NULL = n_src: the number of source rows that exist when only the device
 *          knows it (layer 1 reads the pre-gathered rows; n_src is then their capacity), as in
 *          hopgnn_gat_fwd; rows past it are neither read nor written.
 * out_fwd  the stored forward output (ReLU mask; may be NULL when relu == 0); dOut fp32.
 * gW [d_in x d_out], ga_src [d_out], ga_dst [d_out], gbias [d_out] (or NULL): DEVICE fp32
 *          accumulators, ADDED to.  dHsrc DEVICE out [n_src x d_in] fp32, overwritten, or NULL.
 * ws       DEVICE scratch of hopgnn_gat_bwd_ws_bytes(dt, n_src, n_dst, d_in, d_out, n_heads)
 *          bytes (0 for invalid arguments), 256-byte aligned.
 * Arithmetic is fp32; with a 2-byte dt the gradient with respect to z is rounded to dt before the
 * two matrix products (gW, dHsrc) as in hopgnn_sage_bwd.  The sums over destination rows into a
 * source row (dz, score gradients) are float atomic adds: their rounding depends on arrival order.
 * gbias, ga_src and ga_dst are summed in a fixed order.  Errors as hopgnn_gat_fwd, plus EINVAL for
 * a NULL fwd_ws or a ReLU without out_fwd, ENOMEM_WS for a short workspace.
 */
size_t hopgnn_gat_bwd_ws_bytes(hopgnn_dtype dt, int64_t n_src, int64_t n_dst, int32_t d_in, int32_t d_out,
                               int32_t n_heads);

hopgnn_status hopgnn_gat_bwd(const void *Hsrc, hopgnn_dtype dt, int64_t n_src, const int64_t *n_src_dev,
                             int32_t d_in, const int32_t *self_idx, const int32_t *indptr, const int32_t *idx, int64_t n_dst,
                             const void *W, const void *a_src, const void *a_dst, const void *out_fwd,
                             const void *fwd_ws, int32_t relu, const float *dOut, int32_t d_out, int32_t n_heads,
                             float *gW, float *ga_src, float *ga_dst, float *gbias, float *dHsrc, void *ws,
                             size_t ws_bytes, void *stream);

/*
 * hopgnn_sage_bwd for neighbour lists in slot order, the layers k >= 2 of hopgnn_sample's trees:
 * self rows are the rows themselves and entry e of the segments is source row first_child_row + e
 * (idx[e] holds that number, or -1 for an invalid slot: what hopgnn_sample writes as slot_idx, with
 * first_child_row = n_seeds).  Every source row then has at most one parent, so dHsrc is written
 * row by row without atomic adds and without a clearing pass: bit-stable, and about four times
 * faster than the general scatter.  n_src must be at least first_child_row + the number of entries;
 * source rows past that are zeroed.  0 <= first_child_row <= n_dst, else EINVAL.  Other arguments,
 * workspace and errors as hopgnn_sage_bwd; the weight gradients are computed by the same kernels.
 *
 * mean_fwd (here and in hopgnn_sage_bwd_dev): DEVICE [n_dst x d_in] of type dt, the neighbour means of
 * the forward call, or NULL to compute them again.  hopgnn_sage_fwd, _agg (mean) and _dev leave them
 * in the first n_dst * d_in elements of their workspace, which stay valid until that workspace is
 * used again: a caller that gives every layer its own forward workspace passes that pointer here.
 */
hopgnn_status hopgnn_sage_bwd_slots(const void *Hsrc, hopgnn_dtype dt, int64_t n_src, int32_t d_in,
                                    const int32_t *indptr, const int32_t *idx, int64_t n_dst, int64_t first_child_row,
                                    const void *W_self, const void *W_neigh, const void *out_fwd,
                                    const void *mean_fwd, int32_t relu,
                                    const float *dOut, int32_t d_out, float *gW_self, float *gW_neigh, float *gbias,
                                    float *dHsrc, void *ws, size_t ws_bytes, void *stream);

/*
 * hopgnn_sage_bwd for row counts that only the device knows (the layers over hopgnn_sample_dedup's
 * or hopgnn_sample_layerwise's micrographs, as hopgnn_sage_fwd_dev in the forward pass): n_dst and
 * n_src are the capacities the launches and the workspace are sized for, *n_dst_dev and *n_src_dev
 * (DEVICE, NULL = the capacity) the rows that exist.  Destination rows past *n_dst_dev contribute
 * nothing and their out_fwd / dOut / Hsrc entries are not used; of dHsrc only the first *n_src_dev
 * rows are written.  A source row may have many parents here, so the float atomic adds into dHsrc
 * arrive in varying order (gradients agree to rounding, not bit for bit).
 */
hopgnn_status hopgnn_sage_bwd_dev(const void *Hsrc, hopgnn_dtype dt, int64_t n_src, const int64_t *n_src_dev,
                                  int32_t d_in, const int32_t *self_idx, const int32_t *indptr, const int32_t *idx,
                                  int64_t n_dst, const int64_t *n_dst_dev, const void *W_self, const void *W_neigh,
                                  const void *out_fwd, const void *mean_fwd, int32_t relu, const float *dOut,
                                  int32_t d_out,
                                  float *gW_self, float *gW_neigh, float *gbias, float *dHsrc, void *ws,
                                  size_t ws_bytes, void *stream);

/*
 * One call per group of batches: the whole hot path in the order of paper sections 2, 4
 * and 5.2 - sample the micrographs of each batch's seeds, pre-gather the group's merged slot
 * list once, fetch every distinct row once, then run the L layers of each batch on the
 * fetched rows.  It issues exactly the calls above (hopgnn_sample_group, hopgnn_pregather,
 * hopgnn_gather, hopgnn_sage_fwd x n_batches x L) from C on one stream; it exists because at
 * a few microseconds per kernel the launch sequence itself is the bottleneck when it is driven
 * call by call from an interpreter.  No host synchronisation, no allocation.
 *
 * The plan is a HOST struct the caller fills once; every pointer in it is DEVICE memory the
 * caller owns (T = n_seeds * hopgnn_slots_per_seed, S = T minus the leaf level):
 *   graph, X/dt/dim/ld_elems    as in hopgnn_sample and hopgnn_gather
 *   n_seeds, n_layers, fanouts  shape of every batch
 *   d_out[k], W_self[k], W_neigh[k], bias[k]   layer k+1; d_in of layer 1 is dim, of layer
 *                               k+1 it is d_out[k-1]; ReLU after every layer but the last
 *   group                       most batches one call may carry (buffers are sized for it)
 *   ids, remap                  [group*T];  indptr [S+1];  slot_idx [group*max(S-n_seeds,1)]
 *   uniq [uniq_capacity], n_uniq (1 x int64), Xu [uniq_capacity x dim]; uniq_capacity >=
 *                               min(group*T, n_vertices)
 *   H[k]                        [n_dst(k+1) x d_out[k]] for k < n_layers-1 (the last layer writes
 *                               to `out`); reused by every batch of the group
 *   pg_ws, sage_ws              scratch of hopgnn_pregather_ws_bytes(group*T, ..) and the largest
 *                               hopgnn_sage_fwd_ws_bytes over the layers
 *   mark_begin/_end, mark_stage optional hipEvent_t pair (NULL: none) recorded on `stream` around
 *                               one stage of the sequence, so that a harness can time a kernel
 *                               inside its timed region.  mark_stage: HOPGNN_MARK_GATHER (0) the
 *                               gather launch; HOPGNN_MARK_EMPTY nothing (the pair is recorded
 *                               back to back after the gather: what two markers cost by
 *                               themselves); HOPGNN_MARK_SAMPLE, HOPGNN_MARK_PREGATHER those calls;
 *                               HOPGNN_MARK_AGGREGATE + k / HOPGNN_MARK_PROJECT + k the segmented
 *                               aggregation / the projection kernel of layer k (1-based) of the
 *                               call's first batch (layer_kind 0 without dedup only; otherwise
 *                               HOPGNN_EINVAL).
 *   layer_kind                  0: GraphSAGE-mean layers (hopgnn_sage_fwd, W_self/W_neigh);
 *                               1: GCN-style layers (hopgnn_gcn_fwd with W_self as the one weight
 *                               matrix and norm = gcn_norm); 2: attention layers (hopgnn_gat_fwd
 *                               with W_self, a_src[k], a_dst[k], gat_heads heads; the first layer
 *                               projects only the rows the pre-gather found).  sage_ws must be
 *                               large enough for the chosen layer type's *_ws_bytes.
 *   dedup                       nonzero: per-micrograph deduplicated frontiers - hopgnn_sample_dedup
 *                               (into node_vertex / level_start / indptr / dd_idx with dd_ws),
 *                               hopgnn_pregather over node_vertex, hopgnn_gather, hopgnn_compose_idx
 *                               (into dd_idx_l1) and the layers through hopgnn_sage_fwd_dev with
 *                               their row counts read from level_start.  The n_batches batches of
 *                               a call form one merged batch (batch b draws with keys[b]) and
 *                               every layer is one launch (layer_kind 1 / 2: hopgnn_gcn_fwd_dev /
 *                               hopgnn_gat_fwd_dev); ids, slot_idx and merge_layers are not used; remap holds the node list's
 *                               positions.  With G = group and T the slots of G*n_seeds seeds:
 *                               node_vertex and remap [T], level_start int64 [n_layers+2], indptr
 *                               [T - last level + 1], dd_idx and dd_idx_l1 [T - G*n_seeds], H[k] and
 *                               sage_ws for G times the rows, dd_ws of
 *                               hopgnn_sample_dedup_ws_bytes(G*n_seeds, ..).
 *                               dedup = 2: the same sequence over layer-wise sampled micrographs
 *                               (hopgnn_sample_layerwise, fanouts read as the budgets); with
 *                               caps = hopgnn_layerwise_caps: node_vertex and remap [G*n_seeds*caps[0]],
 *                               indptr [G*n_seeds*caps[1] + 1], dd_idx and dd_idx_l1
 *                               [G*n_seeds*caps[2]], dd_ws of hopgnn_sample_layerwise_ws_bytes.
 *   merge_layers                nonzero: the group's micrographs are sampled as one level-major
 *                               batch (hopgnn_sample_merged, seeds_per_key = n_seeds) and every
 *                               layer is ONE hopgnn_sage_fwd over the whole group instead of one
 *                               per batch - the same rows per seed, far fewer and fuller launches.
 *                               Then indptr holds group*S+1 entries, H[k] group times the rows,
 *                               sage_ws is sized for group times the rows, and ids / remap /
 *                               slot_idx are in the merged layout.
 *   fuse_tree, tree_ws          nonzero fuse_tree (GraphSAGE-mean layers over slot trees only: layer_kind 0,
 *                               dedup 0, at least two layers, every fanout but the last at most 64,
 *                               dim and every d_out whole 16-byte words (multiples of 4 for fp32, of 8 for
 *                               2-byte types); otherwise the flag is ignored): the
 *                               slot tree's shape is used to leave work out.  A parent's children are
 *                               consecutive slots, so layer k's projection also averages every group
 *                               of siblings of the rows it has just produced (stored values, child
 *                               order, invalid slots skipped: the segmented mean's arithmetic) and
 *                               hands layer k+1 its neighbour means; layers >= 2 then run no
 *                               aggregation kernel, and the rows of layer k's deepest level - which
 *                               layer k+1 reads through those means only - are never written (H[k]
 *                               holds the rows of layer k+1's destinations).  Same last-layer bits as
 *                               without the flag.  tree_ws: scratch of hopgnn_batch_tree_ws_bytes(plan)
 *                               (transposed weights, a zero row, two mean buffers), 256-byte aligned,
 *                               filled by hopgnn_batch_prepare(plan) once and again whenever the
 *                               weights change; sage_ws is then not used.
 *   pg_ws_clean                 nonzero: pg_ws was prepared by hopgnn_pregather_ws_init (sizes
 *                               group*T, n_vertices, pg_algo) and has since only been used by
 *                               this library's calls, all of which leave it clean.  Then the
 *                               sampler marks the pre-gather's presence map as it writes the
 *                               ids and the clearing and marking passes are skipped (same
 *                               results).  Zero: no assumption about pg_ws.
 *
 * seeds  DEVICE [n_batches*n_seeds]; keys HOST [n_batches]; out DEVICE
 *        [n_batches*n_seeds x d_out[n_layers-1]] in X's element type.
 * Returns the first failing call's status (nothing later is launched); HOPGNN_EINVAL if
 * n_batches is outside 1..group or a pointer is NULL.
 */
typedef struct {
    hopgnn_csr graph;
    const void *X;
    hopgnn_dtype dt;
    int32_t dim;
    int64_t ld_elems;
    int32_t n_seeds, n_layers;
    int32_t fanouts[8];
    int32_t d_out[8];
    const void *W_self[8];
    const void *W_neigh[8];
    const void *bias[8];
    int32_t pg_algo, group;
    int32_t *ids, *indptr, *slot_idx, *uniq;
    int64_t uniq_capacity;
    int64_t *n_uniq;
    int32_t *remap;
    void *Xu;
    void *H[8];
    void *pg_ws;
    size_t pg_ws_bytes;
    void *sage_ws;
    size_t sage_ws_bytes;
    void *mark_begin, *mark_end;
    int32_t pg_ws_clean;
    int32_t merge_layers;
    int32_t layer_kind, gcn_norm, gat_heads;
    const void *a_src[8];
    const void *a_dst[8];
    int32_t dedup;
    int32_t *node_vertex;
    int64_t *level_start;
    int32_t *dd_idx, *dd_idx_l1;
    void *dd_ws;
    size_t dd_ws_bytes;
    int32_t mark_stage;
    int32_t fuse_tree;
    void *tree_ws;
    size_t tree_ws_bytes;
} hopgnn_batch_plan;

enum { HOPGNN_MARK_GATHER = 0, HOPGNN_MARK_EMPTY = 1, HOPGNN_MARK_SAMPLE = 2, HOPGNN_MARK_PREGATHER = 3,
       HOPGNN_MARK_AGGREGATE = 16, HOPGNN_MARK_PROJECT = 32 };

size_t hopgnn_batch_tree_ws_bytes(const hopgnn_batch_plan *plan /*HOST*/);
hopgnn_status hopgnn_batch_prepare(const hopgnn_batch_plan *plan /*HOST*/, void *stream);

hopgnn_status hopgnn_batch_fwd(const hopgnn_batch_plan *plan /*HOST*/, const int32_t *seeds,
                               const uint64_t *keys /*HOST*/, int32_t n_batches, void *out, void *stream);

/*
 * End of an iteration (paper section 5.1, step 5, and the discussion: the accumulated partial
 * gradients are cleared at the end of each iteration).  The optimiser is not named; reading:
 * plain SGD.  W[i] <- W[i] - lr * grad[i], computed in fp32 and rounded once to W's type; with
 * zero_grad != 0 the accumulator is cleared in the same pass.
 * W DEVICE [n] of type dt (in/out), grad DEVICE [n] fp32 (in, cleared if asked).
 */
hopgnn_status hopgnn_sgd_update(void *W, hopgnn_dtype dt, float *grad, int64_t n, float lr, int32_t zero_grad,
                                void *stream);

/*
 * hopgnn_sgd_update for all of a model's parameter arrays in one launch: W[t] (DEVICE, type dt,
 * n[t] elements) takes grad[t] (DEVICE fp32), t < n_tensors <= 32.  W, grad and n are HOST arrays
 * of n_tensors entries; arrays of length 0 are skipped.  Same arithmetic, element by element.
 */
hopgnn_status hopgnn_sgd_update_multi(void *const *W /*HOST*/, hopgnn_dtype dt, float *const *grad /*HOST*/,
                                      const int64_t *n /*HOST*/, int32_t n_tensors, float lr, int32_t zero_grad,
                                      void *stream);

/*
 * Micrograph merging (paper section 5.3).  HOST-only bookkeeping, no device work.
 *
 * counts is a HOST matrix [n_models x n_steps], row-major: root vertices model m trains at
 * time step t of one iteration.
 *
 * hopgnn_merge_min_step  "which micrographs to merge": the time step with the fewest root
 *     vertices over all models (the paper's stand-in for the number of vertex features a
 *     step needs); ties go to the earliest step.  -1 on bad input.
 * hopgnn_merge_apply     merges step ts away: each model's roots of step ts are dealt to that
 *     model's other steps as evenly as possible (floor share each, the remainder one apiece to
 *     the earliest steps), then column ts is removed in place (rows become n_steps-1 long).
 *     Every model keeps its total.  Returns the new number of steps, -1 on bad input.
 *     Worked example of the section: a model with 4, 2, 2 roots at t0, t1, t2 and ts = t1
 *     ends with 5 and 3.
 * hopgnn_merge_ctl_*     "how many to merge": the examination period.  _init starts with one
 *     step per server.  _report is called once per epoch with that epoch's run time and
 *     returns the number of steps to use in the next epoch: after the first epoch one step is
 *     merged; while an epoch gets faster another is merged; the first epoch that does not get
 *     faster undoes its merge and the pattern is kept from then on (the paper's run goes
 *     4 -> 3 -> 2 -> 3).
 */
typedef struct {
    int32_t n_steps;     /* steps per iteration to use now                */
    int32_t settled;     /* 1 once the examination period is over         */
    int32_t epochs_seen;
    double prev_time;    /* run time of the last epoch that was kept      */
} hopgnn_merge_ctl;

int32_t hopgnn_merge_min_step(const int64_t *counts /*HOST*/, int32_t n_models, int32_t n_steps);
int32_t hopgnn_merge_apply(int64_t *counts /*HOST, in/out*/, int32_t n_models, int32_t n_steps, int32_t ts);
hopgnn_status hopgnn_merge_ctl_init(hopgnn_merge_ctl *ctl /*HOST*/, int32_t n_servers);
int32_t hopgnn_merge_ctl_report(hopgnn_merge_ctl *ctl /*HOST*/, double epoch_time);

#ifdef __cplusplus
}
#endif
#endif /* HOPGNN_H */
