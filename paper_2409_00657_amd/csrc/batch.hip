// Whole groups of batches from one C call: the launch sequence of the hot path (paper sections
// 2, 4 and 5.2) issued from C, because the kernels of a mid-sized batch take a few microseconds
// each and an interpreter cannot issue them that fast.  Only sequencing: every step is one of
// the library's own entry points.
#include <hip/hip_runtime.h>

#include "pregather_internal.hpp"
#include "sage_common.hpp"

using namespace hopgnn;

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
