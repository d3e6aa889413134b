"""Thin ctypes binding over libhopgnn.so: argument marshalling only.

Every function has the name and meaning of the C entry point in
``include/hopgnn.h``; tensors are torch CUDA(HIP) tensors whose storage the
caller owns, and work is enqueued on torch's current stream.  There is no CPU
path: if the library has not been built the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libhopgnn.so")
_lib: Optional[ctypes.CDLL] = None

F32, BF16, F16 = 0, 1, 2
DTYPE_OF = {torch.float32: F32, torch.bfloat16: BF16, torch.float16: F16}
PG_AUTO, PG_BITMAP, PG_RADIX = 0, 1, 2
MARK_GATHER, MARK_EMPTY, MARK_SAMPLE, MARK_PREGATHER, MARK_AGGREGATE, MARK_PROJECT = 0, 1, 2, 3, 16, 32

EXPORTS = ["hopgnn_status_str", "hopgnn_slots_per_seed", "hopgnn_sample",
           "hopgnn_pregather_ws_bytes", "hopgnn_pregather", "hopgnn_gather",
           "hopgnn_sage_fwd_ws_bytes", "hopgnn_sage_fwd", "hopgnn_sage_bwd_ws_bytes", "hopgnn_sage_bwd",
           "hopgnn_micrograph_locality",
           "hopgnn_split_ws_bytes", "hopgnn_split_by_owner", "hopgnn_merge_min_step", "hopgnn_merge_apply",
           "hopgnn_merge_ctl_init", "hopgnn_merge_ctl_report", "hopgnn_batch_fwd",
           "hopgnn_sgd_update", "hopgnn_sgd_update_multi", "hopgnn_sage_fwd_dev", "hopgnn_sage_bwd_dev", "hopgnn_sage_bwd_slots", "hopgnn_sage_bwd_agg", "hopgnn_gcn_bwd", "hopgnn_gat_bwd_ws_bytes", "hopgnn_gat_bwd", "hopgnn_sample_dedup_ws_bytes", "hopgnn_sample_dedup",
           "hopgnn_compose_idx", "hopgnn_frontier_locality", "hopgnn_layerwise_caps", "hopgnn_sample_layerwise_ws_bytes",
           "hopgnn_sample_layerwise", "hopgnn_sample_group", "hopgnn_sample_merged", "hopgnn_pregather_ws_init", "hopgnn_pregather_static", "hopgnn_batch_tree_ws_bytes", "hopgnn_batch_prepare", "hopgnn_pregather_static_max_vertices", "hopgnn_sage_fwd_agg", "hopgnn_gcn_fwd_ws_bytes", "hopgnn_gcn_fwd", "hopgnn_gat_fwd_ws_bytes", "hopgnn_gat_fwd",
           "hopgnn_gcn_fwd_dev", "hopgnn_gat_fwd_dev"]


class HopgnnError(RuntimeError):
    pass


class MergeCtl(ctypes.Structure):
    _fields_ = [("n_steps", ctypes.c_int32), ("settled", ctypes.c_int32), ("epochs_seen", ctypes.c_int32),
                ("prev_time", ctypes.c_double)]


class _Csr(ctypes.Structure):
    _fields_ = [("n_vertices", ctypes.c_int64), ("n_edges", ctypes.c_int64),
                ("offsets", ctypes.c_void_p), ("offsets_i64", ctypes.c_int32),
                ("indices", ctypes.c_void_p)]


class BatchPlan(ctypes.Structure):
    """hopgnn_batch_plan: field for field the C struct."""
    _fields_ = [("graph", _Csr), ("X", ctypes.c_void_p), ("dt", ctypes.c_int), ("dim", ctypes.c_int32),
                ("ld_elems", ctypes.c_int64), ("n_seeds", ctypes.c_int32), ("n_layers", ctypes.c_int32),
                ("fanouts", ctypes.c_int32 * 8), ("d_out", ctypes.c_int32 * 8),
                ("W_self", ctypes.c_void_p * 8), ("W_neigh", ctypes.c_void_p * 8), ("bias", ctypes.c_void_p * 8),
                ("pg_algo", ctypes.c_int32), ("group", ctypes.c_int32),
                ("ids", ctypes.c_void_p), ("indptr", ctypes.c_void_p), ("slot_idx", ctypes.c_void_p),
                ("uniq", ctypes.c_void_p), ("uniq_capacity", ctypes.c_int64), ("n_uniq", ctypes.c_void_p),
                ("remap", ctypes.c_void_p), ("Xu", ctypes.c_void_p), ("H", ctypes.c_void_p * 8),
                ("pg_ws", ctypes.c_void_p), ("pg_ws_bytes", ctypes.c_size_t),
                ("sage_ws", ctypes.c_void_p), ("sage_ws_bytes", ctypes.c_size_t),
                ("mark_begin", ctypes.c_void_p), ("mark_end", ctypes.c_void_p),
                ("pg_ws_clean", ctypes.c_int32), ("merge_layers", ctypes.c_int32),
                ("layer_kind", ctypes.c_int32), ("gcn_norm", ctypes.c_int32), ("gat_heads", ctypes.c_int32),
                ("a_src", ctypes.c_void_p * 8), ("a_dst", ctypes.c_void_p * 8),
                ("dedup", ctypes.c_int32), ("node_vertex", ctypes.c_void_p), ("level_start", ctypes.c_void_p),
                ("dd_idx", ctypes.c_void_p), ("dd_idx_l1", ctypes.c_void_p), ("dd_ws", ctypes.c_void_p),
                ("dd_ws_bytes", ctypes.c_size_t), ("mark_stage", ctypes.c_int32), ("fuse_tree", ctypes.c_int32),
                ("tree_ws", ctypes.c_void_p), ("tree_ws_bytes", ctypes.c_size_t)]


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load the built library; never falls back to anything else."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise HopgnnError("libhopgnn.so is not built: run `python -m paper_2409_00657_amd.build` "
                          "(there is no CPU fallback)")
    L = ctypes.CDLL(_LIB_PATH)
    c = ctypes
    L.hopgnn_status_str.restype = c.c_char_p
    L.hopgnn_status_str.argtypes = [c.c_int]
    L.hopgnn_slots_per_seed.restype = c.c_int64
    L.hopgnn_slots_per_seed.argtypes = [c.POINTER(c.c_int32), c.c_int32]
    L.hopgnn_sample.restype = c.c_int
    L.hopgnn_sample.argtypes = [c.POINTER(_Csr), c.c_void_p, c.c_int32, c.POINTER(c.c_int32),
                                c.c_int32, c.c_uint64, c.c_void_p, c.c_void_p, c.c_void_p,
                                c.c_void_p]
    L.hopgnn_pregather_ws_bytes.restype = c.c_size_t
    L.hopgnn_pregather_ws_bytes.argtypes = [c.c_int64, c.c_int64, c.c_int32]
    L.hopgnn_pregather.restype = c.c_int
    L.hopgnn_pregather.argtypes = [c.c_void_p, c.c_int64, c.c_int64, c.c_int32, c.c_void_p,
                                   c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    L.hopgnn_gather.restype = c.c_int
    L.hopgnn_gather.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_int64, c.c_void_p,
                                c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p]
    L.hopgnn_sage_fwd_ws_bytes.restype = c.c_size_t
    L.hopgnn_sage_fwd_ws_bytes.argtypes = [c.c_int, c.c_int64, c.c_int32, c.c_int32]
    L.hopgnn_sage_fwd.restype = c.c_int
    L.hopgnn_sage_fwd.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p,
                                  c.c_void_p, c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p,
                                  c.c_void_p, c.c_int32, c.c_int32, c.c_void_p, c.c_void_p,
                                  c.c_size_t, c.c_void_p]
    L.hopgnn_sage_bwd_ws_bytes.restype = c.c_size_t
    L.hopgnn_sage_bwd_ws_bytes.argtypes = [c.c_int, c.c_int64, c.c_int32, c.c_int32, c.c_int32]
    L.hopgnn_sage_bwd.restype = c.c_int
    L.hopgnn_sage_bwd.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                  c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_void_p, c.c_int32,
                                  c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    L.hopgnn_sgd_update_multi.restype = c.c_int
    L.hopgnn_sgd_update_multi.argtypes = [c.POINTER(c.c_void_p), c.c_int, c.POINTER(c.c_void_p), c.POINTER(c.c_int64),
                                          c.c_int32, c.c_float, c.c_int32, c.c_void_p]
    L.hopgnn_sage_bwd_agg.restype = c.c_int
    L.hopgnn_sage_bwd_agg.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                      c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, c.c_void_p,
                                      c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t,
                                      c.c_void_p]
    L.hopgnn_gcn_bwd.restype = c.c_int
    L.hopgnn_gcn_bwd.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                 c.c_int64, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, c.c_void_p, c.c_int32,
                                 c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    L.hopgnn_gat_bwd_ws_bytes.restype = c.c_size_t
    L.hopgnn_gat_bwd_ws_bytes.argtypes = [c.c_int, c.c_int64, c.c_int64, c.c_int32, c.c_int32, c.c_int32]
    L.hopgnn_gat_bwd.restype = c.c_int
    L.hopgnn_gat_bwd.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_void_p, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                 c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32,
                                 c.c_void_p, c.c_int32, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
                                 c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    L.hopgnn_sage_bwd_slots.restype = c.c_int
    L.hopgnn_sage_bwd_slots.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_int64,
                                        c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_void_p,
                                        c.c_int32,
                                        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t,
                                        c.c_void_p]
    L.hopgnn_sage_bwd_dev.restype = c.c_int
    L.hopgnn_sage_bwd_dev.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_void_p, c.c_int32, c.c_void_p, c.c_void_p,
                                      c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
                                      c.c_int32, c.c_void_p, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
                                      c.c_void_p, c.c_size_t, c.c_void_p]
    L.hopgnn_micrograph_locality.restype = c.c_int
    L.hopgnn_micrograph_locality.argtypes = [c.c_void_p, c.c_int32, c.POINTER(c.c_int32), c.c_int32,
                                             c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    L.hopgnn_split_ws_bytes.restype = c.c_size_t
    L.hopgnn_split_ws_bytes.argtypes = [c.c_int64]
    L.hopgnn_split_by_owner.restype = c.c_int
    L.hopgnn_split_by_owner.argtypes = [c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p, c.c_int32,
                                        c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    L.hopgnn_merge_min_step.restype = c.c_int32
    L.hopgnn_merge_min_step.argtypes = [c.POINTER(c.c_int64), c.c_int32, c.c_int32]
    L.hopgnn_merge_apply.restype = c.c_int32
    L.hopgnn_merge_apply.argtypes = [c.POINTER(c.c_int64), c.c_int32, c.c_int32, c.c_int32]
    L.hopgnn_merge_ctl_init.restype = c.c_int
    L.hopgnn_merge_ctl_init.argtypes = [c.POINTER(MergeCtl), c.c_int32]
    L.hopgnn_merge_ctl_report.restype = c.c_int32
    L.hopgnn_merge_ctl_report.argtypes = [c.POINTER(MergeCtl), c.c_double]
    L.hopgnn_sage_fwd_dev.restype = c.c_int
    L.hopgnn_sage_fwd_dev.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                      c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32,
                                      c.c_int32, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    L.hopgnn_sample_dedup_ws_bytes.restype = c.c_size_t
    L.hopgnn_sample_dedup_ws_bytes.argtypes = [c.c_int32, c.POINTER(c.c_int32), c.c_int32]
    L.hopgnn_frontier_locality.restype = c.c_int
    L.hopgnn_frontier_locality.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32,
                                           c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    L.hopgnn_layerwise_caps.restype = c.c_int
    L.hopgnn_layerwise_caps.argtypes = [c.POINTER(c.c_int32), c.c_int32, c.POINTER(c.c_int64)]
    L.hopgnn_sample_layerwise_ws_bytes.restype = c.c_size_t
    L.hopgnn_sample_layerwise_ws_bytes.argtypes = [c.c_int32, c.POINTER(c.c_int32), c.c_int32]
    L.hopgnn_sample_layerwise.restype = c.c_int
    L.hopgnn_sample_layerwise.argtypes = [c.POINTER(_Csr), c.c_void_p, c.c_int32, c.c_int32, c.POINTER(c.c_int32),
                                          c.c_int32, c.POINTER(c.c_uint64), c.c_void_p, c.c_void_p, c.c_void_p,
                                          c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    L.hopgnn_sample_dedup.restype = c.c_int
    L.hopgnn_sample_dedup.argtypes = [c.POINTER(_Csr), c.c_void_p, c.c_int32, c.c_int32, c.POINTER(c.c_int32), c.c_int32,
                                      c.POINTER(c.c_uint64), c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
                                      c.c_size_t, c.c_void_p]
    L.hopgnn_compose_idx.restype = c.c_int
    L.hopgnn_compose_idx.argtypes = [c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p]
    L.hopgnn_sgd_update.restype = c.c_int
    L.hopgnn_sgd_update.argtypes = [c.c_void_p, c.c_int, c.c_void_p, c.c_int64, c.c_float, c.c_int32, c.c_void_p]
    L.hopgnn_sample_merged.restype = c.c_int
    L.hopgnn_sample_merged.argtypes = [c.POINTER(_Csr), c.c_void_p, c.c_int32, c.c_int32, c.POINTER(c.c_int32),
                                       c.c_int32, c.POINTER(c.c_uint64), c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    L.hopgnn_sage_fwd_agg.restype = c.c_int
    L.hopgnn_sage_fwd_agg.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                      c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, c.c_int32,
                                      c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    L.hopgnn_pregather_static_max_vertices.restype = c.c_int64
    L.hopgnn_pregather_static_max_vertices.argtypes = []
    L.hopgnn_pregather_static.restype = c.c_int
    L.hopgnn_pregather_static.argtypes = [c.c_void_p, c.c_int64, c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    L.hopgnn_pregather_ws_init.restype = c.c_int
    L.hopgnn_pregather_ws_init.argtypes = [c.c_void_p, c.c_size_t, c.c_int64, c.c_int64, c.c_int32, c.c_void_p]
    L.hopgnn_sample_group.restype = c.c_int
    L.hopgnn_sample_group.argtypes = [c.POINTER(_Csr), c.c_void_p, c.c_int32, c.POINTER(c.c_int32), c.c_int32,
                                      c.POINTER(c.c_uint64), c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64,
                                      c.c_void_p]
    L.hopgnn_gcn_fwd_ws_bytes.restype = c.c_size_t
    L.hopgnn_gcn_fwd_ws_bytes.argtypes = [c.c_int, c.c_int64, c.c_int32, c.c_int32]
    L.hopgnn_gcn_fwd.restype = c.c_int
    L.hopgnn_gcn_fwd.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                 c.c_int64, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, c.c_int32, c.c_void_p,
                                 c.c_void_p, c.c_size_t, c.c_void_p]
    L.hopgnn_gcn_fwd_dev.restype = c.c_int
    L.hopgnn_gcn_fwd_dev.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                     c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, c.c_int32,
                                     c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    L.hopgnn_gat_fwd_dev.restype = c.c_int
    L.hopgnn_gat_fwd_dev.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_void_p, c.c_int32, c.c_void_p, c.c_void_p,
                                     c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
                                     c.c_int32, c.c_int32, c.c_int32, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    L.hopgnn_gat_fwd_ws_bytes.restype = c.c_size_t
    L.hopgnn_gat_fwd_ws_bytes.argtypes = [c.c_int, c.c_int64, c.c_int32, c.c_int32, c.c_int32]
    L.hopgnn_gat_fwd.restype = c.c_int
    L.hopgnn_gat_fwd.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_void_p, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                 c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32,
                                 c.c_int32, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    L.hopgnn_batch_tree_ws_bytes.restype = c.c_size_t
    L.hopgnn_batch_tree_ws_bytes.argtypes = [c.POINTER(BatchPlan)]
    L.hopgnn_batch_prepare.restype = c.c_int
    L.hopgnn_batch_prepare.argtypes = [c.POINTER(BatchPlan), c.c_void_p]
    L.hopgnn_batch_fwd.restype = c.c_int
    L.hopgnn_batch_fwd.argtypes = [c.POINTER(BatchPlan), c.c_void_p, c.POINTER(c.c_uint64), c.c_int32, c.c_void_p,
                                   c.c_void_p]
    _lib = L
    return L


def _check(rc: int, what: str) -> None:
    if rc != 0:
        msg = load_library().hopgnn_status_str(rc).decode()
        raise HopgnnError("%s: %s (status %d)" % (what, msg, rc))


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise HopgnnError("expected a device tensor")
    if not t.is_contiguous():
        raise HopgnnError("expected a contiguous tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _fan(fanouts: Sequence[int]):
    return (ctypes.c_int32 * len(fanouts))(*[int(f) for f in fanouts])


def hopgnn_slots_per_seed(fanouts: Sequence[int]) -> int:
    return int(load_library().hopgnn_slots_per_seed(_fan(fanouts), len(fanouts)))


def hopgnn_sample(offsets: torch.Tensor, indices: torch.Tensor, seeds: torch.Tensor,
                  fanouts: Sequence[int], key: int, ids: torch.Tensor,
                  indptr: Optional[torch.Tensor] = None,
                  slot_idx: Optional[torch.Tensor] = None) -> None:
    g = _Csr(offsets.numel() - 1, indices.numel(), offsets.data_ptr(),
             1 if offsets.dtype == torch.int64 else 0, indices.data_ptr())
    if offsets.dtype not in (torch.int32, torch.int64) or indices.dtype != torch.int32:
        raise HopgnnError("offsets must be int32/int64 and indices int32")
    _ptr(offsets), _ptr(indices)
    rc = load_library().hopgnn_sample(ctypes.byref(g), _ptr(seeds), seeds.numel(), _fan(fanouts),
                                      len(fanouts), ctypes.c_uint64(key & 0xFFFFFFFFFFFFFFFF),
                                      _ptr(ids), _ptr(indptr), _ptr(slot_idx), _stream())
    _check(rc, "hopgnn_sample")


def hopgnn_sample_group(offsets: torch.Tensor, indices: torch.Tensor, seeds: torch.Tensor, n_seeds: int,
                        fanouts: Sequence[int], keys: Sequence[int], ids: torch.Tensor,
                        indptr: Optional[torch.Tensor] = None, slot_idx: Optional[torch.Tensor] = None,
                        slot_idx_stride: int = 0) -> None:
    """len(keys) batches of n_seeds seeds each (seeds back to back) in one launch."""
    g = _Csr(offsets.numel() - 1, indices.numel(), offsets.data_ptr(),
             1 if offsets.dtype == torch.int64 else 0, indices.data_ptr())
    if offsets.dtype not in (torch.int32, torch.int64) or indices.dtype != torch.int32:
        raise HopgnnError("offsets must be int32/int64 and indices int32")
    n = len(keys)
    if seeds.numel() != n * n_seeds or seeds.dtype != torch.int32:
        raise HopgnnError("seeds must hold n_batches * n_seeds int32 values")
    karr = (ctypes.c_uint64 * max(n, 1))(*[k & 0xFFFFFFFFFFFFFFFF for k in keys])
    rc = load_library().hopgnn_sample_group(ctypes.byref(g), _ptr(seeds), n_seeds, _fan(fanouts), len(fanouts), karr, n,
                                            _ptr(ids), _ptr(indptr), _ptr(slot_idx), slot_idx_stride, _stream())
    _check(rc, "hopgnn_sample_group")


def hopgnn_sample_merged(offsets: torch.Tensor, indices: torch.Tensor, seeds: torch.Tensor, seeds_per_key: int,
                         fanouts: Sequence[int], keys: Sequence[int], ids: torch.Tensor,
                         indptr: Optional[torch.Tensor] = None, slot_idx: Optional[torch.Tensor] = None) -> None:
    """One level-major batch of seeds.numel() micrographs; block b of seeds_per_key seeds uses keys[b]."""
    g = _Csr(offsets.numel() - 1, indices.numel(), offsets.data_ptr(),
             1 if offsets.dtype == torch.int64 else 0, indices.data_ptr())
    if offsets.dtype not in (torch.int32, torch.int64) or indices.dtype != torch.int32:
        raise HopgnnError("offsets must be int32/int64 and indices int32")
    n = seeds.numel()
    if seeds.dtype != torch.int32 or len(keys) != -(-n // max(seeds_per_key, 1)):
        raise HopgnnError("seeds must be int32 and keys hold one key per block of seeds_per_key seeds")
    karr = (ctypes.c_uint64 * max(len(keys), 1))(*[k & 0xFFFFFFFFFFFFFFFF for k in keys])
    rc = load_library().hopgnn_sample_merged(ctypes.byref(g), _ptr(seeds), n, seeds_per_key, _fan(fanouts), len(fanouts),
                                             karr, _ptr(ids), _ptr(indptr), _ptr(slot_idx), _stream())
    _check(rc, "hopgnn_sample_merged")


def hopgnn_pregather_ws_bytes(n_ids: int, n_vertices: int, algo: int = PG_AUTO) -> int:
    return int(load_library().hopgnn_pregather_ws_bytes(n_ids, n_vertices, algo))


def hopgnn_pregather_static(ids: torch.Tensor, n_vertices: int, uniq: torch.Tensor, n_uniq: torch.Tensor,
                            remap: torch.Tensor) -> None:
    """hopgnn_pregather with the library's static scratch: no workspace, no allocation."""
    _check(load_library().hopgnn_pregather_static(_ptr(ids), ids.numel(), n_vertices, _ptr(uniq), _ptr(n_uniq),
                                                  _ptr(remap), _stream()), "hopgnn_pregather_static")


def hopgnn_pregather_ws_init(ws: torch.Tensor, n_ids: int, n_vertices: int, algo: int = PG_AUTO) -> None:
    _check(load_library().hopgnn_pregather_ws_init(_ptr(ws), ws.numel() * ws.element_size(), n_ids, n_vertices, algo,
                                                   _stream()), "hopgnn_pregather_ws_init")


def hopgnn_pregather(ids: torch.Tensor, n_vertices: int, uniq: torch.Tensor,
                     n_uniq_dev: torch.Tensor, remap: torch.Tensor, ws: torch.Tensor,
                     algo: int = PG_AUTO) -> None:
    rc = load_library().hopgnn_pregather(_ptr(ids), ids.numel(), n_vertices, algo, _ptr(uniq),
                                         _ptr(n_uniq_dev), _ptr(remap), _ptr(ws),
                                         ws.numel() * ws.element_size(), _stream())
    _check(rc, "hopgnn_pregather")


def hopgnn_gather(X: torch.Tensor, uniq: torch.Tensor, n_uniq: int,
                  n_uniq_dev: Optional[torch.Tensor], Xu: torch.Tensor) -> None:
    if X.dim() != 2 or X.stride(1) != 1:
        raise HopgnnError("X must be 2-D with unit column stride")
    rc = load_library().hopgnn_gather(ctypes.c_void_p(X.data_ptr()), DTYPE_OF[X.dtype], X.shape[0],
                                      X.shape[1], X.stride(0), _ptr(uniq), n_uniq,
                                      _ptr(n_uniq_dev), _ptr(Xu), _stream())
    _check(rc, "hopgnn_gather")


def hopgnn_sage_fwd_ws_bytes(dtype: torch.dtype, n_dst: int, d_in: int, d_out: int) -> int:
    return int(load_library().hopgnn_sage_fwd_ws_bytes(DTYPE_OF[dtype], n_dst, d_in, d_out))


def hopgnn_sage_fwd(Hsrc: torch.Tensor, n_src: int, self_idx: Optional[torch.Tensor],
                    indptr: torch.Tensor, idx: torch.Tensor, n_dst: int, W_self: torch.Tensor,
                    W_neigh: torch.Tensor, bias: Optional[torch.Tensor], relu: bool,
                    out: torch.Tensor, ws: torch.Tensor) -> None:
    d_in, d_out = W_self.shape
    rc = load_library().hopgnn_sage_fwd(_ptr(Hsrc), DTYPE_OF[Hsrc.dtype], n_src, d_in,
                                        _ptr(self_idx), _ptr(indptr), _ptr(idx), n_dst,
                                        _ptr(W_self), _ptr(W_neigh), _ptr(bias), d_out,
                                        1 if relu else 0, _ptr(out), _ptr(ws),
                                        ws.numel() * ws.element_size(), _stream())
    _check(rc, "hopgnn_sage_fwd")


def hopgnn_micrograph_locality(ids: torch.Tensor, n_seeds: int, fanouts: Sequence[int], owner: torch.Tensor,
                               n_total: torch.Tensor, n_coloc: torch.Tensor) -> None:
    rc = load_library().hopgnn_micrograph_locality(_ptr(ids), n_seeds, _fan(fanouts), len(fanouts),
                                                   _ptr(owner), _ptr(n_total), _ptr(n_coloc), _stream())
    _check(rc, "hopgnn_micrograph_locality")


def hopgnn_split_ws_bytes(n_uniq: int) -> int:
    return int(load_library().hopgnn_split_ws_bytes(n_uniq))


def hopgnn_split_by_owner(uniq: torch.Tensor, n_uniq: int, n_uniq_dev: Optional[torch.Tensor],
                          owner: torch.Tensor, server: int, remote: torch.Tensor, n_remote_dev: torch.Tensor,
                          ws: torch.Tensor) -> None:
    rc = load_library().hopgnn_split_by_owner(_ptr(uniq), n_uniq, _ptr(n_uniq_dev), _ptr(owner), server,
                                              _ptr(remote), _ptr(n_remote_dev), _ptr(ws),
                                              ws.numel() * ws.element_size(), _stream())
    _check(rc, "hopgnn_split_by_owner")


def hopgnn_merge_min_step(counts) -> int:
    """counts: list of rows (models) of per-step root counts (host)."""
    n_models, n_steps = len(counts), len(counts[0])
    flat = (ctypes.c_int64 * (n_models * n_steps))(*[int(x) for r in counts for x in r])
    return int(load_library().hopgnn_merge_min_step(flat, n_models, n_steps))


def hopgnn_merge_apply(counts, ts: int):
    """-> the merged matrix (list of rows, one step fewer)."""
    n_models, n_steps = len(counts), len(counts[0])
    flat = (ctypes.c_int64 * (n_models * n_steps))(*[int(x) for r in counts for x in r])
    n = int(load_library().hopgnn_merge_apply(flat, n_models, n_steps, ts))
    if n < 0:
        raise HopgnnError("hopgnn_merge_apply: invalid argument")
    return [[int(flat[m * n + t]) for t in range(n)] for m in range(n_models)]


def hopgnn_sage_bwd_ws_bytes(dtype: torch.dtype, n_dst: int, d_in: int, d_out: int, want_dh: bool) -> int:
    return int(load_library().hopgnn_sage_bwd_ws_bytes(DTYPE_OF[dtype], n_dst, d_in, d_out, 1 if want_dh else 0))


def hopgnn_sage_bwd(Hsrc: torch.Tensor, n_src: int, self_idx: Optional[torch.Tensor], indptr: torch.Tensor,
                    idx: torch.Tensor, n_dst: int, W_self: torch.Tensor, W_neigh: torch.Tensor,
                    out_fwd: Optional[torch.Tensor], relu: bool, dOut: torch.Tensor, gW_self: torch.Tensor,
                    gW_neigh: torch.Tensor, gbias: Optional[torch.Tensor], dHsrc: Optional[torch.Tensor],
                    ws: torch.Tensor) -> None:
    d_in, d_out = W_self.shape
    rc = load_library().hopgnn_sage_bwd(_ptr(Hsrc), DTYPE_OF[Hsrc.dtype], n_src, d_in, _ptr(self_idx), _ptr(indptr),
                                        _ptr(idx), n_dst, _ptr(W_self), _ptr(W_neigh), _ptr(out_fwd),
                                        1 if relu else 0, _ptr(dOut), d_out, _ptr(gW_self), _ptr(gW_neigh),
                                        _ptr(gbias), _ptr(dHsrc), _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check(rc, "hopgnn_sage_bwd")


def hopgnn_sage_bwd_agg(Hsrc: torch.Tensor, n_src: int, self_idx: Optional[torch.Tensor], indptr: torch.Tensor,
                        idx: torch.Tensor, n_dst: int, W_self: torch.Tensor, W_neigh: torch.Tensor,
                        out_fwd: Optional[torch.Tensor], agg: int, relu: bool, dOut: torch.Tensor,
                        gW_self: torch.Tensor, gW_neigh: torch.Tensor, gbias: Optional[torch.Tensor],
                        dHsrc: Optional[torch.Tensor], ws: torch.Tensor) -> None:
    d_in, d_out = W_self.shape
    rc = load_library().hopgnn_sage_bwd_agg(_ptr(Hsrc), DTYPE_OF[Hsrc.dtype], n_src, d_in, _ptr(self_idx), _ptr(indptr),
                                            _ptr(idx), n_dst, _ptr(W_self), _ptr(W_neigh), _ptr(out_fwd), int(agg),
                                            1 if relu else 0, _ptr(dOut), d_out, _ptr(gW_self), _ptr(gW_neigh),
                                            _ptr(gbias), _ptr(dHsrc), _ptr(ws), ws.numel() * ws.element_size(),
                                            _stream())
    _check(rc, "hopgnn_sage_bwd_agg")


def hopgnn_gcn_bwd(Hsrc: torch.Tensor, n_src: int, self_idx: Optional[torch.Tensor], indptr: torch.Tensor,
                   idx: torch.Tensor, n_dst: int, W: torch.Tensor, out_fwd: Optional[torch.Tensor], norm: int,
                   relu: bool, dOut: torch.Tensor, gW: torch.Tensor, gbias: Optional[torch.Tensor],
                   dHsrc: Optional[torch.Tensor], ws: torch.Tensor, stream=None) -> None:
    d_in, d_out = W.shape
    rc = load_library().hopgnn_gcn_bwd(_ptr(Hsrc), DTYPE_OF[Hsrc.dtype], n_src, d_in, _ptr(self_idx), _ptr(indptr),
                                       _ptr(idx), n_dst, _ptr(W), _ptr(out_fwd), int(norm), 1 if relu else 0, _ptr(dOut),
                                       d_out, _ptr(gW), _ptr(gbias), _ptr(dHsrc), _ptr(ws),
                                       ws.numel() * ws.element_size(), _stream() if stream is None else stream)
    _check(rc, "hopgnn_gcn_bwd")


def hopgnn_gat_bwd_ws_bytes(dtype: torch.dtype, n_src: int, n_dst: int, d_in: int, d_out: int, n_heads: int) -> int:
    return int(load_library().hopgnn_gat_bwd_ws_bytes(DTYPE_OF[dtype], n_src, n_dst, d_in, d_out, n_heads))


def hopgnn_gat_bwd(Hsrc: torch.Tensor, n_src: int, self_idx: Optional[torch.Tensor], indptr: torch.Tensor,
                   idx: torch.Tensor, n_dst: int, W: torch.Tensor, a_src: torch.Tensor, a_dst: torch.Tensor,
                   out_fwd: Optional[torch.Tensor], fwd_ws: torch.Tensor, relu: bool, dOut: torch.Tensor, n_heads: int,
                   gW: torch.Tensor, ga_src: torch.Tensor, ga_dst: torch.Tensor, gbias: Optional[torch.Tensor],
                   dHsrc: Optional[torch.Tensor], ws: torch.Tensor, stream=None,
                   n_src_dev: Optional[torch.Tensor] = None) -> None:
    d_in, d_out = W.shape
    rc = load_library().hopgnn_gat_bwd(_ptr(Hsrc), DTYPE_OF[Hsrc.dtype], n_src, _ptr(n_src_dev), d_in, _ptr(self_idx), _ptr(indptr),
                                       _ptr(idx), n_dst, _ptr(W), _ptr(a_src), _ptr(a_dst), _ptr(out_fwd), _ptr(fwd_ws),
                                       1 if relu else 0, _ptr(dOut), d_out, int(n_heads), _ptr(gW), _ptr(ga_src),
                                       _ptr(ga_dst), _ptr(gbias), _ptr(dHsrc), _ptr(ws),
                                       ws.numel() * ws.element_size(), _stream() if stream is None else stream)
    _check(rc, "hopgnn_gat_bwd")


def hopgnn_sage_bwd_slots(Hsrc: torch.Tensor, n_src: int, indptr: torch.Tensor, idx: torch.Tensor, n_dst: int,
                          first_child_row: int, W_self: torch.Tensor, W_neigh: torch.Tensor,
                          out_fwd: Optional[torch.Tensor], relu: bool, dOut: torch.Tensor, gW_self: torch.Tensor,
                          gW_neigh: torch.Tensor, gbias: Optional[torch.Tensor], dHsrc: Optional[torch.Tensor],
                          ws: torch.Tensor, mean_fwd: Optional[torch.Tensor] = None) -> None:
    d_in, d_out = W_self.shape
    rc = load_library().hopgnn_sage_bwd_slots(_ptr(Hsrc), DTYPE_OF[Hsrc.dtype], n_src, d_in, _ptr(indptr), _ptr(idx),
                                              n_dst, first_child_row, _ptr(W_self), _ptr(W_neigh), _ptr(out_fwd),
                                              _ptr(mean_fwd), 1 if relu else 0, _ptr(dOut), d_out, _ptr(gW_self), _ptr(gW_neigh),
                                              _ptr(gbias), _ptr(dHsrc), _ptr(ws), ws.numel() * ws.element_size(),
                                              _stream())
    _check(rc, "hopgnn_sage_bwd_slots")


def hopgnn_sage_bwd_dev(Hsrc: torch.Tensor, n_src: int, n_src_dev: Optional[torch.Tensor],
                        self_idx: Optional[torch.Tensor], indptr: torch.Tensor, idx: torch.Tensor, n_dst: int,
                        n_dst_dev: Optional[torch.Tensor], W_self: torch.Tensor, W_neigh: torch.Tensor,
                        out_fwd: Optional[torch.Tensor], relu: bool, dOut: torch.Tensor, gW_self: torch.Tensor,
                        gW_neigh: torch.Tensor, gbias: Optional[torch.Tensor], dHsrc: Optional[torch.Tensor],
                        ws: torch.Tensor, mean_fwd: Optional[torch.Tensor] = None) -> None:
    d_in, d_out = W_self.shape
    rc = load_library().hopgnn_sage_bwd_dev(_ptr(Hsrc), DTYPE_OF[Hsrc.dtype], n_src, _ptr(n_src_dev), d_in,
                                            _ptr(self_idx), _ptr(indptr), _ptr(idx), n_dst, _ptr(n_dst_dev),
                                            _ptr(W_self), _ptr(W_neigh), _ptr(out_fwd), _ptr(mean_fwd),
                                            1 if relu else 0, _ptr(dOut),
                                            d_out, _ptr(gW_self), _ptr(gW_neigh), _ptr(gbias), _ptr(dHsrc), _ptr(ws),
                                            ws.numel() * ws.element_size(), _stream())
    _check(rc, "hopgnn_sage_bwd_dev")


def hopgnn_batch_fwd(plan: BatchPlan, seeds: torch.Tensor, keys, out: torch.Tensor, stream=None) -> None:
    """hopgnn_batch_fwd: len(keys) batches of plan.n_seeds seeds each; `out` receives the last
    layer's rows of every batch."""
    n = len(keys)
    if seeds.dtype != torch.int32 or not seeds.is_cuda or seeds.numel() != n * plan.n_seeds:
        raise HopgnnError("seeds must be %d int32 values on the device" % (n * plan.n_seeds))
    if not out.is_cuda or not out.is_contiguous() or DTYPE_OF.get(out.dtype) != plan.dt \
            or out.numel() != n * plan.n_seeds * plan.d_out[plan.n_layers - 1]:
        raise HopgnnError("out must be a contiguous device tensor [n_batches*n_seeds, d_out] of X's type")
    karr = (ctypes.c_uint64 * n)(*[k & 0xFFFFFFFFFFFFFFFF for k in keys])
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    _check(load_library().hopgnn_batch_fwd(ctypes.byref(plan), seeds.data_ptr(), karr, n, out.data_ptr(), st),
           "hopgnn_batch_fwd")


def hopgnn_gcn_fwd_ws_bytes(dtype: torch.dtype, n_dst: int, d_in: int, d_out: int) -> int:
    return int(load_library().hopgnn_gcn_fwd_ws_bytes(DTYPE_OF[dtype], n_dst, d_in, d_out))


def hopgnn_gcn_fwd(Hsrc: torch.Tensor, n_src: int, self_idx: Optional[torch.Tensor], indptr: torch.Tensor,
                   idx: torch.Tensor, n_dst: int, W: torch.Tensor, bias: Optional[torch.Tensor], norm: int, relu: bool,
                   out: torch.Tensor, ws: torch.Tensor) -> None:
    d_in, d_out = W.shape
    rc = load_library().hopgnn_gcn_fwd(_ptr(Hsrc), DTYPE_OF[Hsrc.dtype], n_src, d_in, _ptr(self_idx), _ptr(indptr),
                                       _ptr(idx), n_dst, _ptr(W), _ptr(bias), d_out, norm, 1 if relu else 0, _ptr(out),
                                       _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check(rc, "hopgnn_gcn_fwd")


def hopgnn_gat_fwd_ws_bytes(dtype: torch.dtype, n_src: int, d_in: int, d_out: int, n_heads: int) -> int:
    return int(load_library().hopgnn_gat_fwd_ws_bytes(DTYPE_OF[dtype], n_src, d_in, d_out, n_heads))


def hopgnn_gat_fwd(Hsrc: torch.Tensor, n_src: int, self_idx: Optional[torch.Tensor], indptr: torch.Tensor,
                   idx: torch.Tensor, n_dst: int, W: torch.Tensor, a_src: torch.Tensor, a_dst: torch.Tensor,
                   bias: Optional[torch.Tensor], n_heads: int, relu: bool, out: torch.Tensor, ws: torch.Tensor,
                   n_src_dev: Optional[torch.Tensor] = None) -> None:
    d_in, d_out = W.shape
    rc = load_library().hopgnn_gat_fwd(_ptr(Hsrc), DTYPE_OF[Hsrc.dtype], n_src, _ptr(n_src_dev), d_in, _ptr(self_idx),
                                       _ptr(indptr),
                                       _ptr(idx), n_dst, _ptr(W), _ptr(a_src), _ptr(a_dst), _ptr(bias), d_out, n_heads,
                                       1 if relu else 0, _ptr(out), _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check(rc, "hopgnn_gat_fwd")


def hopgnn_gcn_fwd_dev(Hsrc: torch.Tensor, n_src: int, self_idx: Optional[torch.Tensor], indptr: torch.Tensor,
                       idx: torch.Tensor, n_dst: int, n_dst_dev: Optional[torch.Tensor], W: torch.Tensor,
                       bias: Optional[torch.Tensor], norm: int, relu: bool, out: torch.Tensor, ws: torch.Tensor) -> None:
    d_in, d_out = W.shape
    rc = load_library().hopgnn_gcn_fwd_dev(_ptr(Hsrc), DTYPE_OF[Hsrc.dtype], n_src, d_in, _ptr(self_idx), _ptr(indptr),
                                           _ptr(idx), n_dst, _ptr(n_dst_dev), _ptr(W), _ptr(bias), d_out, norm,
                                           1 if relu else 0, _ptr(out), _ptr(ws), ws.numel() * ws.element_size(),
                                           _stream())
    _check(rc, "hopgnn_gcn_fwd_dev")


def hopgnn_gat_fwd_dev(Hsrc: torch.Tensor, n_src: int, n_src_dev: Optional[torch.Tensor],
                       self_idx: Optional[torch.Tensor], indptr: torch.Tensor, idx: torch.Tensor, n_dst: int,
                       n_dst_dev: Optional[torch.Tensor], W: torch.Tensor, a_src: torch.Tensor, a_dst: torch.Tensor,
                       bias: Optional[torch.Tensor], n_heads: int, relu: bool, out: torch.Tensor,
                       ws: torch.Tensor) -> None:
    d_in, d_out = W.shape
    rc = load_library().hopgnn_gat_fwd_dev(_ptr(Hsrc), DTYPE_OF[Hsrc.dtype], n_src, _ptr(n_src_dev), d_in,
                                           _ptr(self_idx), _ptr(indptr), _ptr(idx), n_dst, _ptr(n_dst_dev), _ptr(W),
                                           _ptr(a_src), _ptr(a_dst), _ptr(bias), d_out, n_heads, 1 if relu else 0,
                                           _ptr(out), _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check(rc, "hopgnn_gat_fwd_dev")


AGG_MEAN, AGG_SUM, AGG_MAX = 0, 1, 2


def hopgnn_sage_fwd_agg(Hsrc: torch.Tensor, n_src: int, self_idx: Optional[torch.Tensor], indptr: torch.Tensor,
                        idx: torch.Tensor, n_dst: int, W_self: torch.Tensor, W_neigh: torch.Tensor,
                        bias: Optional[torch.Tensor], agg: int, relu: bool, out: torch.Tensor, ws: torch.Tensor) -> None:
    d_in, d_out = W_self.shape
    rc = load_library().hopgnn_sage_fwd_agg(_ptr(Hsrc), DTYPE_OF[Hsrc.dtype], n_src, d_in, _ptr(self_idx), _ptr(indptr),
                                            _ptr(idx), n_dst, _ptr(W_self), _ptr(W_neigh), _ptr(bias), d_out, agg,
                                            1 if relu else 0, _ptr(out), _ptr(ws), ws.numel() * ws.element_size(),
                                            _stream())
    _check(rc, "hopgnn_sage_fwd_agg")


def hopgnn_sgd_update(W: torch.Tensor, grad: torch.Tensor, lr: float, zero_grad: bool = True, stream=None) -> None:
    if grad.dtype != torch.float32 or grad.numel() != W.numel():
        raise HopgnnError("grad must be fp32 with as many elements as W")
    st = _stream() if stream is None else stream
    _check(load_library().hopgnn_sgd_update(_ptr(W), DTYPE_OF[W.dtype], _ptr(grad), W.numel(), lr,
                                            1 if zero_grad else 0, st), "hopgnn_sgd_update")


class SgdTensors:
    """The parameter arrays of a model and their gradient accumulators, marshalled once for
    hopgnn_sgd_update_multi."""

    def __init__(self, pairs):
        pairs = [(W, g) for W, g in pairs if W is not None]
        if not pairs:
            raise HopgnnError("no tensors")
        dts = {W.dtype for W, _ in pairs}
        if len(dts) != 1 or any(g.dtype != torch.float32 or g.numel() != W.numel() for W, g in pairs):
            raise HopgnnError("one parameter type; gradients fp32 with as many elements as their parameters")
        self.dt = DTYPE_OF[pairs[0][0].dtype]
        self.n_tensors = len(pairs)
        self.W = (ctypes.c_void_p * self.n_tensors)(*[W.data_ptr() for W, _ in pairs])
        self.grad = (ctypes.c_void_p * self.n_tensors)(*[g.data_ptr() for _, g in pairs])
        self.n = (ctypes.c_int64 * self.n_tensors)(*[W.numel() for W, _ in pairs])
        self._keep = pairs

    def update(self, lr: float, zero_grad: bool = True, stream=None) -> None:
        st = _stream() if stream is None else stream
        rc = load_library().hopgnn_sgd_update_multi(self.W, self.dt, self.grad, self.n, self.n_tensors, lr,
                                                    1 if zero_grad else 0, st)
        if rc:
            _check(rc, "hopgnn_sgd_update_multi")


def hopgnn_sample_dedup_ws_bytes(n_seeds: int, fanouts: Sequence[int]) -> int:
    return int(load_library().hopgnn_sample_dedup_ws_bytes(n_seeds, _fan(fanouts), len(fanouts)))


def hopgnn_sample_dedup(offsets: torch.Tensor, indices: torch.Tensor, seeds: torch.Tensor, fanouts: Sequence[int],
                        key, node_vertex: torch.Tensor, level_start: torch.Tensor, indptr: torch.Tensor,
                        idx: torch.Tensor, ws: torch.Tensor, seeds_per_key: int = 0) -> None:
    """`key`: one key for the whole batch, or a list with one key per block of seeds_per_key seeds."""
    keys = list(key) if isinstance(key, (list, tuple)) else [key]
    spk = seeds_per_key if seeds_per_key > 0 else max(seeds.numel(), 1)
    if len(keys) != -(-seeds.numel() // spk) and seeds.numel() > 0:
        raise HopgnnError("one key per block of seeds_per_key seeds")
    karr = (ctypes.c_uint64 * max(len(keys), 1))(*[k & 0xFFFFFFFFFFFFFFFF for k in keys])
    g = _Csr(offsets.numel() - 1, indices.numel(), offsets.data_ptr(),
             1 if offsets.dtype == torch.int64 else 0, indices.data_ptr())
    if offsets.dtype not in (torch.int32, torch.int64) or indices.dtype != torch.int32:
        raise HopgnnError("offsets must be int32/int64 and indices int32")
    if level_start.dtype != torch.int64 or level_start.numel() < len(fanouts) + 2:
        raise HopgnnError("level_start must hold n_layers + 2 int64 values")
    rc = load_library().hopgnn_sample_dedup(ctypes.byref(g), _ptr(seeds), seeds.numel(), spk, _fan(fanouts), len(fanouts),
                                            karr, _ptr(node_vertex),
                                            _ptr(level_start), _ptr(indptr), _ptr(idx), _ptr(ws),
                                            ws.numel() * ws.element_size(), _stream())
    _check(rc, "hopgnn_sample_dedup")


def hopgnn_frontier_locality(node_vertex: torch.Tensor, level_start: torch.Tensor, indptr: torch.Tensor,
                             idx: torch.Tensor, n_seeds: int, n_layers: int, nodes_per_seed: int, owner: torch.Tensor,
                             n_total: torch.Tensor, n_coloc: torch.Tensor) -> None:
    if owner.dtype != torch.int32 or n_total.dtype != torch.int32 or n_coloc.dtype != torch.int32 \
            or level_start.dtype != torch.int64:
        raise HopgnnError("owner, n_total, n_coloc must be int32 and level_start int64")
    if n_total.numel() < n_seeds or n_coloc.numel() < n_seeds:
        raise HopgnnError("n_total and n_coloc must hold one value per seed")
    rc = load_library().hopgnn_frontier_locality(_ptr(node_vertex), _ptr(level_start), _ptr(indptr), _ptr(idx), n_seeds,
                                                 n_layers, nodes_per_seed, _ptr(owner), _ptr(n_total), _ptr(n_coloc),
                                                 _stream())
    _check(rc, "hopgnn_frontier_locality")


def hopgnn_layerwise_caps(budgets: Sequence[int]):
    """(nodes, non-leaf nodes, entries) one seed may need."""
    caps = (ctypes.c_int64 * 3)()
    _check(load_library().hopgnn_layerwise_caps(_fan(budgets), len(budgets), caps), "hopgnn_layerwise_caps")
    return int(caps[0]), int(caps[1]), int(caps[2])


def hopgnn_sample_layerwise_ws_bytes(n_seeds: int, budgets: Sequence[int]) -> int:
    return int(load_library().hopgnn_sample_layerwise_ws_bytes(n_seeds, _fan(budgets), len(budgets)))


def hopgnn_sample_layerwise(offsets: torch.Tensor, indices: torch.Tensor, seeds: torch.Tensor, budgets: Sequence[int],
                            key, node_vertex: torch.Tensor, level_start: torch.Tensor, indptr: torch.Tensor,
                            idx: torch.Tensor, ws: torch.Tensor, seeds_per_key: int = 0) -> None:
    """`key`: one key for the whole batch, or a list with one key per block of seeds_per_key seeds."""
    keys = list(key) if isinstance(key, (list, tuple)) else [key]
    spk = seeds_per_key if seeds_per_key > 0 else max(seeds.numel(), 1)
    if len(keys) != -(-seeds.numel() // spk) and seeds.numel() > 0:
        raise HopgnnError("one key per block of seeds_per_key seeds")
    karr = (ctypes.c_uint64 * max(len(keys), 1))(*[k & 0xFFFFFFFFFFFFFFFF for k in keys])
    if offsets.dtype not in (torch.int32, torch.int64) or indices.dtype != torch.int32:
        raise HopgnnError("offsets must be int32/int64 and indices int32")
    if level_start.dtype != torch.int64 or level_start.numel() < len(budgets) + 2:
        raise HopgnnError("level_start must hold n_layers + 2 int64 values")
    g = _Csr(offsets.numel() - 1, indices.numel(), offsets.data_ptr(),
             1 if offsets.dtype == torch.int64 else 0, indices.data_ptr())
    rc = load_library().hopgnn_sample_layerwise(ctypes.byref(g), _ptr(seeds), seeds.numel(), spk, _fan(budgets),
                                                len(budgets), karr, _ptr(node_vertex), _ptr(level_start), _ptr(indptr),
                                                _ptr(idx), _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check(rc, "hopgnn_sample_layerwise")


def hopgnn_compose_idx(idx: torch.Tensor, map_: torch.Tensor, out: torch.Tensor) -> None:
    _check(load_library().hopgnn_compose_idx(_ptr(idx), idx.numel(), _ptr(map_), _ptr(out), _stream()),
           "hopgnn_compose_idx")


def hopgnn_sage_fwd_dev(Hsrc: torch.Tensor, n_src: int, self_idx: Optional[torch.Tensor], indptr: torch.Tensor,
                        idx: torch.Tensor, n_dst: int, n_dst_dev: Optional[torch.Tensor], W_self: torch.Tensor,
                        W_neigh: torch.Tensor, bias: Optional[torch.Tensor], agg: int, relu: bool, out: torch.Tensor,
                        ws: torch.Tensor) -> None:
    d_in, d_out = W_self.shape
    rc = load_library().hopgnn_sage_fwd_dev(_ptr(Hsrc), DTYPE_OF[Hsrc.dtype], n_src, d_in, _ptr(self_idx), _ptr(indptr),
                                            _ptr(idx), n_dst, _ptr(n_dst_dev), _ptr(W_self), _ptr(W_neigh), _ptr(bias),
                                            d_out, agg, 1 if relu else 0, _ptr(out), _ptr(ws),
                                            ws.numel() * ws.element_size(), _stream())
    _check(rc, "hopgnn_sage_fwd_dev")
