// Calls between the library's own translation units (not part of the C ABI): the single-call
// batch path samples straight into the pre-gather's presence map.
#pragma once
#include <hip/hip_runtime.h>

#include "common.hpp"

namespace hopgnn {

// The presence map (one byte per vertex) inside a pre-gather workspace, or nullptr when the
// bitmap path does not apply to these sizes / this algo or the workspace is too small.
uint8_t* pregather_marks_map(void* ws, size_t ws_bytes, int64_t n_ids, int64_t n_vertices, int32_t algo);

// The pre-gather of `ids` from a presence map that already holds exactly their marks (and was
// clean before them); leaves the map clean again.
hopgnn_status pregather_from_marks(const int32_t* ids, int64_t n_ids, int64_t n_vertices, int32_t* uniq,
                                   int64_t* n_uniq_dev, int32_t* remap, void* ws, size_t ws_bytes, hipStream_t s);

// hopgnn_sample_group, optionally storing a 1 into present[v] for every valid vertex it writes.
hopgnn_status sample_batches(const hopgnn_csr* g, const int32_t* seeds, int32_t n_seeds, const int32_t* fanouts,
                             int32_t n_layers, const uint64_t* keys, int32_t n_batches, int32_t* ids, int32_t* indptr,
                             int32_t* slot_idx, int64_t slot_idx_stride, uint8_t* present, void* stream);

// hopgnn_sample_merged with the same optional marking.
hopgnn_status sample_merged(const hopgnn_csr* g, const int32_t* seeds, int32_t n_seeds, int32_t seeds_per_key,
                            const int32_t* fanouts, int32_t n_layers, const uint64_t* keys, int32_t* ids,
                            int32_t* indptr, int32_t* slot_idx, uint8_t* present, void* stream);

// hopgnn_sample_dedup with the same optional marking (every node's vertex).
hopgnn_status sample_dedup(const hopgnn_csr* g, const int32_t* seeds, int32_t n_seeds, int32_t seeds_per_key,
                           const int32_t* fanouts, int32_t n_layers, const uint64_t* keys, int32_t* node_vertex,
                           int64_t* level_start, int32_t* indptr, int32_t* idx, void* ws, size_t ws_bytes,
                           uint8_t* present, void* stream);

// hopgnn_sample_layerwise with the same optional marking.
hopgnn_status sample_layerwise(const hopgnn_csr* g, const int32_t* seeds, int32_t n_seeds, int32_t seeds_per_key,
                               const int32_t* budgets, int32_t n_layers, const uint64_t* keys, int32_t* node_vertex,
                               int64_t* level_start, int32_t* indptr, int32_t* idx, void* ws, size_t ws_bytes,
                               uint8_t* present, void* stream);

}  // namespace hopgnn
