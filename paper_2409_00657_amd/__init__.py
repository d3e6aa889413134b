"""MI355X-native micrograph hot path of HopGNN (arxiv 2409.00657).

``binding`` is the thin ctypes layer over the C-ABI library built from
``csrc/`` (hand-written HIP for gfx950); ``synth`` produces seeded inputs.
"""
from . import synth  # noqa: F401
from .binding import (  # noqa: F401
    DTYPE_OF, hopgnn_batch_fwd, hopgnn_gat_fwd, hopgnn_gat_fwd_ws_bytes, hopgnn_gather,
    hopgnn_gcn_fwd, hopgnn_gcn_fwd_ws_bytes, hopgnn_micrograph_locality, hopgnn_pregather, hopgnn_pregather_ws_bytes, hopgnn_pregather_ws_init,
    hopgnn_sage_bwd, hopgnn_sage_bwd_ws_bytes, hopgnn_sage_fwd, hopgnn_sage_fwd_agg, hopgnn_sage_fwd_ws_bytes, hopgnn_sample, hopgnn_sample_dedup, hopgnn_sample_dedup_ws_bytes, hopgnn_compose_idx,
    hopgnn_sage_fwd_dev, hopgnn_sgd_update, hopgnn_sample_group, hopgnn_sample_merged,
    hopgnn_slots_per_seed, hopgnn_split_by_owner, hopgnn_split_ws_bytes, library_path, load_library,
)
