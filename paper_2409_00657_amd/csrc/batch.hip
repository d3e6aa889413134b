// Whole groups of batches from one C call: the launch sequence of the hot path (paper sections
// 2, 4 and 5.2) issued from C, because the kernels of a mid-sized batch take a few microseconds
// each and an interpreter cannot issue them that fast.  Only sequencing: every step is one of
// the library's own entry points.
#include <hip/hip_runtime.h>

#include "pregather_internal.hpp"
#include "sage_common.hpp"

using namespace hopgnn;

namespace {

// Scratch of the fused slot-tree path: per layer the transposed weights (2-byte types), one zero
// row, and two neighbour-mean buffers that consecutive layers alternate between (layer k reads
// mean[(k-1)&1], its projection writes layer k+1's means into mean[k&1]).
struct TreeWs {
    size_t wt_off[kMaxLayers], zero_off, zero_bytes, mean_off[2], total;
    int32_t KP[kMaxLayers], NP[kMaxLayers];
    bool ok;
};

bool tree_applies(const hopgnn_batch_plan* p) {
    const int32_t L = p->n_layers;
    if (!p->fuse_tree || p->layer_kind != 0 || p->dedup || L < 2 || L > kMaxLayers) return false;
    const int32_t per16 = p->dt == HOPGNN_F32 ? 4 : 8;        // elements per 16-byte word: rows move as whole words
    if (p->dim % per16 != 0) return false;
    for (int32_t k = 0; k < L; ++k)
        if (p->d_out[k] < 1 || p->d_out[k] % per16 != 0) return false;
    for (int32_t h = 0; h + 1 < L; ++h)           // groups of siblings on the levels that some layer averages
        if (p->fanouts[h] < 1 || p->fanouts[h] > kTreeMaxFan) return false;
    return true;
}

TreeWs tree_ws_layout(const hopgnn_batch_plan* p) {
    TreeWs W{};
    const int32_t L = p->n_layers, B = p->n_seeds;
    W.ok = tree_applies(p) && B >= 1;
    if (!W.ok) return W;
    const size_t es = dtype_size(p->dt);
    const int64_t scale = p->merge_layers ? p->group : 1;
    int64_t level[kMaxLayers + 1];
    level[0] = (int64_t)B * scale;
    for (int h = 1; h <= L; ++h) level[h] = level[h - 1] * p->fanouts[h - 1];
    size_t o = 0, mean_bytes[2] = {0, 0};
    int32_t d_in = p->dim, d_max = p->dim;
    for (int32_t k = 1; k <= L; ++k) {
        const ProjWs P = proj_ws_layout(p->dt, 0, d_in, 2 * d_in, p->d_out[k - 1]);
        W.KP[k - 1] = P.KP;
        W.NP[k - 1] = P.NP;
        W.wt_off[k - 1] = o;
        o += P.wt_bytes;
        int64_t n_dst = 0;
        for (int h = 0; h <= L - k; ++h) n_dst += level[h];
        const size_t mb = align_up((size_t)n_dst * (size_t)d_in * es, 256);
        if (mb > mean_bytes[(k - 1) & 1]) mean_bytes[(k - 1) & 1] = mb;
        d_max = d_in > d_max ? d_in : d_max;
        d_in = p->d_out[k - 1];
    }
    W.zero_off = o;
    W.zero_bytes = align_up(((size_t)2 * d_max + 64) * es, 256);
    o += W.zero_bytes;
    W.mean_off[0] = o;
    o += mean_bytes[0];
    W.mean_off[1] = o;
    o += mean_bytes[1];
    W.total = o;
    return W;
}

}  // namespace

extern "C" size_t hopgnn_batch_tree_ws_bytes(const hopgnn_batch_plan* p) {
    if (p == nullptr) return 0;
    const TreeWs W = tree_ws_layout(p);
    return W.ok ? W.total : 0;
}

extern "C" hopgnn_status hopgnn_batch_prepare(const hopgnn_batch_plan* p, void* stream) {
    if (p == nullptr) return HOPGNN_EINVAL;
    const TreeWs W = tree_ws_layout(p);
    if (!W.ok) return HOPGNN_OK;                   // the flag does not apply to this plan: nothing to prepare
    if (p->tree_ws == nullptr || !aligned(p->tree_ws, 256)) return HOPGNN_EINVAL;
    if (p->tree_ws_bytes < W.total) return HOPGNN_ENOMEM_WS;
    char* ws = static_cast<char*>(p->tree_ws);
    int32_t d_in = p->dim;
    for (int32_t k = 1; k <= p->n_layers; ++k) {
        if (p->W_self[k - 1] == nullptr || p->W_neigh[k - 1] == nullptr) return HOPGNN_EINVAL;
        TransposeJob job{};
        if (p->dt != HOPGNN_F32)
            job = TransposeJob{static_cast<const uint16_t*>(p->W_self[k - 1]), static_cast<const uint16_t*>(p->W_neigh[k - 1]),
                               reinterpret_cast<uint16_t*>(ws + W.wt_off[k - 1]), d_in, p->d_out[k - 1], W.KP[k - 1],
                               W.NP[k - 1], 0u, 2 * d_in};
        const hopgnn_status rc = launch_prep_weights(job, k == 1 ? ws + W.zero_off : nullptr, k == 1 ? W.zero_bytes : 0,
                                                     static_cast<hipStream_t>(stream));
        if (rc != HOPGNN_OK) return rc;
        d_in = p->d_out[k - 1];
    }
    return HOPGNN_OK;
}

extern "C" hopgnn_status hopgnn_batch_fwd(const hopgnn_batch_plan* p, const int32_t* seeds, const uint64_t* keys,
                                          int32_t n_batches, void* out, void* stream) {
    if (p == nullptr || seeds == nullptr || keys == nullptr || out == nullptr) return HOPGNN_EINVAL;
    if (n_batches < 1 || n_batches > p->group) return HOPGNN_EINVAL;
    const int32_t L = p->n_layers, B = p->n_seeds;
    if (L < 1 || L > kMaxLayers || B < 1) return HOPGNN_EINVAL;
    if ((p->mark_begin == nullptr) != (p->mark_end == nullptr)) return HOPGNN_EINVAL;
    const bool marked = p->mark_begin != nullptr;
    const int32_t mstage = marked ? p->mark_stage : -1;
    int32_t mark_layer = 0;           // layer whose aggregation (mark_agg) or projection kernel is bracketed
    bool mark_agg = false;
    if (marked) {
        if (mstage >= HOPGNN_MARK_PROJECT) mark_layer = mstage - HOPGNN_MARK_PROJECT;
        else if (mstage >= HOPGNN_MARK_AGGREGATE) mark_layer = mstage - HOPGNN_MARK_AGGREGATE, mark_agg = true;
        else if (mstage < 0 || mstage > HOPGNN_MARK_PREGATHER) return HOPGNN_EINVAL;
        if (mstage >= HOPGNN_MARK_AGGREGATE && (mark_layer < 1 || mark_layer > p->n_layers || p->layer_kind != 0))
            return HOPGNN_EINVAL;
        if (p->dedup && mstage > HOPGNN_MARK_EMPTY) return HOPGNN_EINVAL;   // only the gather is bracketed there
    }
    hipEvent_t ev_a = (hipEvent_t)p->mark_begin, ev_b = (hipEvent_t)p->mark_end;
    auto rec = [&](int32_t stage, bool begin) -> bool {     // record the marker of `stage`, if it is the marked one
        if (mstage != stage) return true;
        return hipEventRecord(begin ? ev_a : ev_b, (hipStream_t)stream) == hipSuccess;
    };
    if (p->layer_kind < 0 || p->layer_kind > 2) return HOPGNN_EINVAL;
    const int64_t t_seed = hopgnn_slots_per_seed(p->fanouts, L);
    if (t_seed < 0) return HOPGNN_EINVAL;
    int64_t level[kMaxLayers + 1];
    level[0] = B;
    for (int h = 1; h <= L; ++h) level[h] = level[h - 1] * p->fanouts[h - 1];
    const int64_t T = t_seed * B, S = T - level[L];
    const int64_t slot_idx_stride = S - B > 1 ? S - B : 1;
    const size_t es = dtype_size(p->dt);
    hipStream_t st = (hipStream_t)stream;
    if (p->dedup) {
        // per-micrograph frontiers (1: node-wise draws kept once per level, 2: layer-wise sampling):
        // node counts depend on the data, so everything is sized for the capacity and the layers
        // read their row counts from level_start
        if (p->dedup > 2) return HOPGNN_EINVAL;
        if (p->node_vertex == nullptr || p->level_start == nullptr || p->dd_idx == nullptr || p->dd_idx_l1 == nullptr)
            return HOPGNN_EINVAL;
        const bool layerwise = p->dedup == 2;
        const int32_t B_all = n_batches * B;          // the call's batches form one merged batch
        int64_t cap_level[kMaxLayers + 1];            // node capacity of level h, per seed
        int64_t nodes_seed = 0, entries_seed = 0;
        if (layerwise) {
            int64_t caps[3];
            const hopgnn_status rc_caps = hopgnn_layerwise_caps(p->fanouts, L, caps);
            if (rc_caps != HOPGNN_OK) return rc_caps;
            cap_level[0] = 1;
            for (int h = 1; h <= L; ++h) cap_level[h] = p->fanouts[h - 1];
            nodes_seed = caps[0];
            entries_seed = caps[2];
        } else {
            for (int h = 0; h <= L; ++h) cap_level[h] = level[h] / B;
            nodes_seed = t_seed;
            entries_seed = t_seed - 1;
        }
        const int64_t T_all = nodes_seed * B_all;
        if (T_all + (layerwise ? entries_seed * B_all : 0) >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;
        // with a workspace the caller keeps clean the compaction marks the presence map itself
        uint8_t* dd_marks = p->pg_ws_clean ? pregather_marks_map(p->pg_ws, p->pg_ws_bytes,
                                                                 (int64_t)p->group * B * nodes_seed,
                                                                 p->graph.n_vertices, p->pg_algo)
                                           : nullptr;
        hopgnn_status rc =
            layerwise ? sample_layerwise(&p->graph, seeds, B_all, B, p->fanouts, L, keys, p->node_vertex, p->level_start,
                                         p->indptr, p->dd_idx, p->dd_ws, p->dd_ws_bytes, dd_marks, stream)
                      : sample_dedup(&p->graph, seeds, B_all, B, p->fanouts, L, keys, p->node_vertex, p->level_start,
                                     p->indptr, p->dd_idx, p->dd_ws, p->dd_ws_bytes, dd_marks, stream);
        if (rc != HOPGNN_OK) return rc;
        if (dd_marks != nullptr)
            rc = pregather_from_marks(p->node_vertex, T_all, p->graph.n_vertices, p->uniq, p->n_uniq, p->remap, p->pg_ws,
                                      p->pg_ws_bytes, st);
        else
            rc = hopgnn_pregather(p->node_vertex, T_all, p->graph.n_vertices, p->pg_algo, p->uniq, p->n_uniq, p->remap,
                                  p->pg_ws, p->pg_ws_bytes, stream);
        if (rc != HOPGNN_OK) return rc;
        if (!rec(HOPGNN_MARK_GATHER, true)) return HOPGNN_EHIP;
        rc = hopgnn_gather(p->X, p->dt, p->graph.n_vertices, p->dim, p->ld_elems, p->uniq, p->uniq_capacity, p->n_uniq,
                           p->Xu, stream);
        if (rc != HOPGNN_OK) return rc;
        if (!rec(HOPGNN_MARK_GATHER, false) || !rec(HOPGNN_MARK_EMPTY, true) || !rec(HOPGNN_MARK_EMPTY, false))
            return HOPGNN_EHIP;
        rc = hopgnn_compose_idx(p->dd_idx, entries_seed * B_all, p->remap, p->dd_idx_l1, stream);
        if (rc != HOPGNN_OK) return rc;
        const void* src = p->Xu;
        int64_t n_src = p->uniq_capacity;
        int32_t d_in = p->dim;
        for (int32_t k = 1; k <= L; ++k) {
            int64_t n_dst = 0;                      // capacity: levels 0 .. L-k
            for (int h = 0; h <= L - k; ++h) n_dst += cap_level[h] * B_all;
            void* dst = k == L ? out : p->H[k - 1];
            if (dst == nullptr) return HOPGNN_EINVAL;
            const int32_t* self_idx = k == 1 ? p->remap : nullptr;
            const int32_t* idx = k == 1 ? p->dd_idx_l1 : p->dd_idx;
            const int64_t* n_dst_dev = p->level_start + (L - k + 1);
            if (p->layer_kind == 0)
                rc = hopgnn_sage_fwd_dev(src, p->dt, n_src, d_in, self_idx, p->indptr, idx, n_dst, n_dst_dev,
                                         p->W_self[k - 1], p->W_neigh[k - 1], p->bias[k - 1], p->d_out[k - 1],
                                         HOPGNN_AGG_MEAN, k < L ? 1 : 0, dst, p->sage_ws, p->sage_ws_bytes, stream);
            else if (p->layer_kind == 1)
                rc = hopgnn_gcn_fwd_dev(src, p->dt, n_src, d_in, self_idx, p->indptr, idx, n_dst, n_dst_dev,
                                        p->W_self[k - 1], p->bias[k - 1], p->d_out[k - 1], p->gcn_norm, k < L ? 1 : 0, dst,
                                        p->sage_ws, p->sage_ws_bytes, stream);
            else        // the source rows that exist: the pre-gathered rows, then the previous layer's rows
                rc = hopgnn_gat_fwd_dev(src, p->dt, n_src, k == 1 ? p->n_uniq : p->level_start + (L - k + 2), d_in,
                                        self_idx, p->indptr, idx, n_dst, n_dst_dev, p->W_self[k - 1], p->a_src[k - 1],
                                        p->a_dst[k - 1], p->bias[k - 1], p->d_out[k - 1], p->gat_heads, k < L ? 1 : 0, dst,
                                        p->sage_ws, p->sage_ws_bytes, stream);
            if (rc != HOPGNN_OK) return rc;
            src = dst;
            n_src = n_dst;
            d_in = p->d_out[k - 1];
        }
        return HOPGNN_OK;
    }
    // merge_layers: the group is laid out as ONE level-major batch of n_batches * B micrographs
    // (each block of B seeds with its own key), so every layer is one launch over the whole group
    const bool merged = p->merge_layers != 0;
    const int32_t B_run = merged ? n_batches * B : B;          // micrographs per layer launch
    const int32_t n_runs = merged ? 1 : n_batches;
    if ((int64_t)n_batches * T >= ((int64_t)1 << 31)) return HOPGNN_ERANGE;

    // With a workspace the caller keeps clean (hopgnn_pregather_ws_init once, then only calls that
    // leave it clean) the sampler marks the presence map itself: no clearing pass, no marking pass.
    uint8_t* marks = p->pg_ws_clean ? pregather_marks_map(p->pg_ws, p->pg_ws_bytes, (int64_t)p->group * T,
                                                          p->graph.n_vertices, p->pg_algo)
                                    : nullptr;
    if (!rec(HOPGNN_MARK_SAMPLE, true)) return HOPGNN_EHIP;
    hopgnn_status rc =
        merged ? sample_merged(&p->graph, seeds, B_run, B, p->fanouts, L, keys, p->ids, p->indptr,
                               L > 1 ? p->slot_idx : nullptr, marks, stream)
               : sample_batches(&p->graph, seeds, B, p->fanouts, L, keys, n_batches, p->ids, p->indptr,
                                L > 1 ? p->slot_idx : nullptr, slot_idx_stride, marks, stream);
    if (rc != HOPGNN_OK) return rc;
    if (!rec(HOPGNN_MARK_SAMPLE, false) || !rec(HOPGNN_MARK_PREGATHER, true)) return HOPGNN_EHIP;
    if (marks != nullptr)
        rc = pregather_from_marks(p->ids, n_batches * T, p->graph.n_vertices, p->uniq, p->n_uniq, p->remap, p->pg_ws,
                                  p->pg_ws_bytes, st);
    else
        rc = hopgnn_pregather(p->ids, n_batches * T, p->graph.n_vertices, p->pg_algo, p->uniq, p->n_uniq, p->remap,
                              p->pg_ws, p->pg_ws_bytes, stream);
    if (rc != HOPGNN_OK) return rc;
    if (!rec(HOPGNN_MARK_PREGATHER, false) || !rec(HOPGNN_MARK_GATHER, true)) return HOPGNN_EHIP;
    rc = hopgnn_gather(p->X, p->dt, p->graph.n_vertices, p->dim, p->ld_elems, p->uniq, p->uniq_capacity, p->n_uniq,
                       p->Xu, stream);
    if (rc != HOPGNN_OK) return rc;
    if (!rec(HOPGNN_MARK_GATHER, false) || !rec(HOPGNN_MARK_EMPTY, true) || !rec(HOPGNN_MARK_EMPTY, false))
        return HOPGNN_EHIP;

    const int32_t d_last = p->d_out[L - 1];
    const int64_t rows_scale = merged ? n_batches : 1;         // level sizes of one run = B_run / B times a batch's
    const TreeWs TW = tree_ws_layout(p);
    if (TW.ok) {
        // The slot tree's shape leaves work out: see fuse_tree in the header.  Layer 1 aggregates with the
        // segmented-mean kernel (its neighbours are scattered rows of Xu); every projection but the last
        // also writes the next layer's neighbour means and skips the rows only those means read.
        if (p->tree_ws == nullptr || !aligned(p->tree_ws, 256)) return HOPGNN_EINVAL;
        if (p->tree_ws_bytes < TW.total) return HOPGNN_ENOMEM_WS;
        if (mstage >= HOPGNN_MARK_AGGREGATE + 2 && mstage < HOPGNN_MARK_PROJECT) return HOPGNN_EINVAL;   // no such kernel
        char* tws = static_cast<char*>(p->tree_ws);
        const void* zero = tws + TW.zero_off;
        for (int32_t b = 0; b < n_runs; ++b) {
            const int32_t* rb = p->remap + b * T;
            const void* src = p->Xu;
            int64_t n_src = p->uniq_capacity;
            int32_t d_in = p->dim;
            for (int32_t k = 1; k <= L; ++k) {
                int64_t n_dst = 0;
                for (int h = 0; h <= L - k; ++h) n_dst += level[h] * rows_scale;
                void* dst = k == L ? (void*)((char*)out + (size_t)b * B * d_last * es) : p->H[k - 1];
                if (dst == nullptr) return HOPGNN_EINVAL;
                void* mean = tws + TW.mean_off[(k - 1) & 1];
                const uint16_t* Wt = reinterpret_cast<const uint16_t*>(tws + TW.wt_off[k - 1]);
                const bool mk = b == 0 && k == mark_layer;
                if (k == 1) {
                    if (mk && mark_agg && hipEventRecord(ev_a, st) != hipSuccess) return HOPGNN_EHIP;
                    const AggSpec spec{nullptr, 0, kAggOpMean};
                    void* zr = const_cast<void*>(zero);
                    if (p->dt == HOPGNN_F32) rc = launch_mean<TrF32>(src, p->indptr, rb + B_run, n_dst, d_in, mean, zr, TW.zero_bytes, TransposeJob{}, 0, st, spec, nullptr);
                    else if (p->dt == HOPGNN_BF16) rc = launch_mean<TrBF16>(src, p->indptr, rb + B_run, n_dst, d_in, mean, zr, TW.zero_bytes, TransposeJob{}, 0, st, spec, nullptr);
                    else rc = launch_mean<TrF16>(src, p->indptr, rb + B_run, n_dst, d_in, mean, zr, TW.zero_bytes, TransposeJob{}, 0, st, spec, nullptr);
                    if (rc != HOPGNN_OK) return rc;
                    if (mk && mark_agg && hipEventRecord(ev_b, st) != hipSuccess) return HOPGNN_EHIP;
                }
                TreeLayer tree{};
                tree.n_levels = L - k + 1;
                for (int h = 0; h < tree.n_levels; ++h) {
                    tree.level_rows[h] = level[h] * rows_scale;
                    tree.fan[h] = h ? p->fanouts[h - 1] : 1;
                }
                tree.ids = p->ids + (merged ? 0 : (int64_t)b * T);
                tree.mean_next = tws + TW.mean_off[k & 1];
                tree.n_src = n_src;
                if (mk && !mark_agg && hipEventRecord(ev_a, st) != hipSuccess) return HOPGNN_EHIP;
                rc = project_dispatch(p->dt, st, src, k == 1 ? rb : nullptr, mean, p->W_self[k - 1], p->W_neigh[k - 1], Wt,
                                      TW.KP[k - 1], p->bias[k - 1], n_dst, d_in, 2 * d_in, p->d_out[k - 1], k < L ? 1 : 0,
                                      zero, dst, 0, nullptr, k < L ? &tree : nullptr);
                if (rc != HOPGNN_OK) return rc;
                if (mk && !mark_agg && hipEventRecord(ev_b, st) != hipSuccess) return HOPGNN_EHIP;
                src = dst;
                n_src = n_dst;
                d_in = p->d_out[k - 1];
            }
        }
        return HOPGNN_OK;
    }
    for (int32_t b = 0; b < n_runs; ++b) {
        const int32_t* rb = p->remap + b * T;
        const void* src = p->Xu;
        int64_t n_src = p->uniq_capacity;
        int32_t d_in = p->dim;
        for (int32_t k = 1; k <= L; ++k) {
            int64_t n_dst = 0;                      // slots of levels 0 .. L-k
            for (int h = 0; h <= L - k; ++h) n_dst += level[h] * rows_scale;
            void* dst = k == L ? (void*)((char*)out + (size_t)b * B * d_last * es) : p->H[k - 1];
            if (dst == nullptr) return HOPGNN_EINVAL;
            const int32_t* self_idx = k == 1 ? rb : nullptr;
            const int32_t* nbr = k == 1 ? rb + B_run : p->slot_idx + b * slot_idx_stride;
            const int32_t relu = k < L ? 1 : 0;
            if (p->layer_kind == 0) {
                LayerMarks lm{};
                if (b == 0 && k == mark_layer) {
                    if (mark_agg) lm.agg_begin = ev_a, lm.agg_end = ev_b;
                    else lm.proj_begin = ev_a, lm.proj_end = ev_b;
                }
                rc = sage_fwd_marked(src, p->dt, n_src, d_in, self_idx, p->indptr, nbr, n_dst, nullptr, p->W_self[k - 1],
                                     p->W_neigh[k - 1], p->bias[k - 1], p->d_out[k - 1], HOPGNN_AGG_MEAN, relu, dst,
                                     p->sage_ws, p->sage_ws_bytes, stream, b == 0 && k == mark_layer ? &lm : nullptr);
            }
            else if (p->layer_kind == 1)
                rc = hopgnn_gcn_fwd(src, p->dt, n_src, d_in, self_idx, p->indptr, nbr, n_dst, p->W_self[k - 1],
                                    p->bias[k - 1], p->d_out[k - 1], p->gcn_norm, relu, dst, p->sage_ws, p->sage_ws_bytes,
                                    stream);
            else
                rc = hopgnn_gat_fwd(src, p->dt, n_src, k == 1 ? p->n_uniq : nullptr, d_in, self_idx, p->indptr, nbr,
                                    n_dst, p->W_self[k - 1], p->a_src[k - 1], p->a_dst[k - 1], p->bias[k - 1],
                                    p->d_out[k - 1], p->gat_heads, relu, dst, p->sage_ws, p->sage_ws_bytes, stream);
            if (rc != HOPGNN_OK) return rc;
            src = dst;
            n_src = n_dst;
            d_in = p->d_out[k - 1];
        }
    }
    return HOPGNN_OK;
}
