"""ctypes front end of the CPU oracle (``hopgnn_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``.  The GPU package never imports
this module and this module never imports the GPU package.

Arrays are numpy, host memory.  2-byte float types (bf16 / fp16) travel as
``uint16`` bit patterns together with a dtype code, because numpy has no bf16.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

F32, BF16, F16, F64 = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hopgnn_oracle.c")
_LIB = os.path.join(_HERE, "libhopgnn_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C99, -O2) into a shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-std=c99", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        c = ctypes
        L.orc_mix.restype = c.c_uint64
        L.orc_mix.argtypes = [c.c_uint64]
        L.orc_hash64.restype = c.c_uint64
        L.orc_hash64.argtypes = [c.c_uint64, c.c_uint32, c.c_uint32, c.c_uint32, c.c_uint32]
        L.orc_slots_per_seed.restype = c.c_int64
        L.orc_slots_per_seed.argtypes = [c.c_void_p, c.c_int32]
        L.orc_sample.restype = c.c_int
        L.orc_sample.argtypes = [c.c_void_p, c.c_int, c.c_void_p, c.c_int64, c.c_void_p,
                                 c.c_int32, c.c_void_p, c.c_int32, c.c_uint64,
                                 c.c_void_p, c.c_void_p]
        L.orc_pregather.restype = c.c_int64
        L.orc_pregather.argtypes = [c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p]
        L.orc_gather.restype = c.c_int
        L.orc_gather.argtypes = [c.c_void_p, c.c_int64, c.c_int64, c.c_int64, c.c_void_p,
                                 c.c_int64, c.c_void_p]
        L.orc_micrograph_locality.restype = c.c_int
        L.orc_micrograph_locality.argtypes = [c.c_void_p, c.c_int32, c.c_void_p, c.c_int32, c.c_void_p,
                                              c.c_void_p, c.c_void_p]
        L.orc_split_by_owner.restype = c.c_int64
        L.orc_split_by_owner.argtypes = [c.c_void_p, c.c_int64, c.c_void_p, c.c_int32, c.c_void_p]
        L.orc_round_store.restype = None
        L.orc_round_store.argtypes = [c.c_void_p, c.c_int64, c.c_int, c.c_void_p]
        L.orc_load_f64.restype = None
        L.orc_load_f64.argtypes = [c.c_void_p, c.c_int64, c.c_int, c.c_void_p]
        L.orc_sage_fwd.restype = c.c_int
        L.orc_sage_fwd.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p,
                                   c.c_void_p, c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p,
                                   c.c_void_p, c.c_int32, c.c_int32, c.c_void_p]
        L.orc_sage_bwd.restype = c.c_int
        L.orc_sage_bwd.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                   c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_void_p,
                                   c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
        L.orc_sage_agg_fwd.restype = c.c_int
        L.orc_sage_agg_fwd.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                       c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, c.c_int32,
                                       c.c_void_p]
        L.orc_gcn_fwd.restype = c.c_int
        L.orc_gcn_fwd.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                  c.c_int64, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, c.c_int32, c.c_void_p]
        L.orc_gat_fwd.restype = c.c_int
        L.orc_gat_fwd.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                  c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32,
                                  c.c_int32, c.c_void_p]
        L.orc_sage_agg_bwd.restype = c.c_int
        L.orc_sage_agg_bwd.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                       c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, c.c_void_p,
                                       c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
        L.orc_gcn_bwd.restype = c.c_int
        L.orc_gcn_bwd.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                  c.c_int64, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, c.c_void_p, c.c_int32,
                                  c.c_void_p, c.c_void_p, c.c_void_p]
        L.orc_gat_bwd.restype = c.c_int
        L.orc_gat_bwd.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
                                  c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_void_p,
                                  c.c_int32, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
        _lib = L
    return _lib


_NP_OF = {F32: np.float32, BF16: np.uint16, F16: np.uint16, F64: np.float64}


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _arr(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def mix(z: int) -> int:
    return int(lib().orc_mix(z & 0xFFFFFFFFFFFFFFFF))


def hash64(key: int, root: int, v: int, h: int, j: int) -> int:
    return int(lib().orc_hash64(key & 0xFFFFFFFFFFFFFFFF, root & 0xFFFFFFFF, v & 0xFFFFFFFF,
                                h & 0xFFFFFFFF, j & 0xFFFFFFFF))


def slots_per_seed(fanouts) -> int:
    f = _arr(fanouts, np.int32)
    return int(lib().orc_slots_per_seed(_p(f), len(f)))


def level_sizes(n_seeds: int, fanouts):
    """[B*P_0, B*P_1, ..., B*P_L] (bookkeeping only, no method arithmetic)."""
    out, p = [n_seeds], 1
    for f in fanouts:
        p *= int(f)
        out.append(n_seeds * p)
    return out


def sample(offsets, indices, seeds, fanouts, key: int = 0):
    """-> (ids[T] int32 level-major, indptr[S_{L-1}+1] int32)."""
    offsets = np.ascontiguousarray(offsets)
    assert offsets.dtype in (np.int32, np.int64)
    indices = _arr(indices, np.int32)
    seeds = _arr(seeds, np.int32)
    f = _arr(fanouts, np.int32)
    B = len(seeds)
    lv = level_sizes(B, f)
    T = sum(lv)
    ids = np.empty(T, np.int32)
    indptr = np.empty(T - lv[-1] + 1, np.int32)
    rc = lib().orc_sample(_p(offsets), int(offsets.dtype == np.int64), _p(indices),
                          len(offsets) - 1, _p(seeds), B, _p(f), len(f),
                          key & 0xFFFFFFFFFFFFFFFF, _p(ids), _p(indptr))
    if rc:
        raise ValueError("orc_sample failed: %d" % rc)
    return ids, indptr


def pregather(ids):
    """-> (uniq[U] ascending int32, remap[len(ids)] int32)."""
    ids = _arr(ids, np.int32)
    uniq = np.empty(max(len(ids), 1), np.int32)
    remap = np.empty(len(ids), np.int32)
    U = lib().orc_pregather(_p(ids), len(ids), _p(uniq), _p(remap))
    if U < 0:
        raise MemoryError
    return uniq[:U].copy(), remap


def gather(X, uniq):
    """X: 2-D numpy array of any fixed-size dtype; rows copied byte for byte."""
    assert X.ndim == 2 and X.strides[1] == X.itemsize
    uniq = _arr(uniq, np.int32)
    out = np.empty((len(uniq), X.shape[1]), X.dtype)
    rc = lib().orc_gather(_p(X), X.shape[0], X.shape[1] * X.itemsize, X.strides[0],
                          _p(uniq), len(uniq), _p(out))
    if rc:
        raise ValueError("orc_gather failed: %d" % rc)
    return out


def micrograph_locality(ids, n_seeds: int, fanouts, owner):
    """-> (n_total[n_seeds], n_colocated[n_seeds]) int32: distinct vertices per micrograph and
    distinct non-root vertices that share the root's home server."""
    ids = _arr(ids, np.int32)
    f = _arr(fanouts, np.int32)
    owner = _arr(owner, np.int32)
    n_total = np.empty(n_seeds, np.int32)
    n_coloc = np.empty(n_seeds, np.int32)
    rc = lib().orc_micrograph_locality(_p(ids), n_seeds, _p(f), len(f), _p(owner), _p(n_total), _p(n_coloc))
    if rc:
        raise ValueError("orc_micrograph_locality failed: %d" % rc)
    return n_total, n_coloc


def split_by_owner(uniq, owner, server: int):
    """-> the entries of uniq that are not stored on `server` (in order)."""
    uniq = _arr(uniq, np.int32)
    owner = _arr(owner, np.int32)
    remote = np.empty(max(len(uniq), 1), np.int32)
    n = lib().orc_split_by_owner(_p(uniq), len(uniq), _p(owner), server, _p(remote))
    return remote[:n].copy()


def round_store(x64, dtype: int):
    """Round a float64 array once (nearest-even) to the storage dtype."""
    x64 = _arr(x64, np.float64)
    out = np.empty(x64.shape, _NP_OF[dtype])
    lib().orc_round_store(_p(x64), x64.size, dtype, _p(out))
    return out


def load_f64(a, dtype: int):
    a = _arr(a, _NP_OF[dtype])
    out = np.empty(a.shape, np.float64)
    lib().orc_load_f64(_p(a), a.size, dtype, _p(out))
    return out


def sage_fwd(Hsrc, dtype, self_idx, indptr, idx, W_self, W_neigh, bias, relu):
    """One GraphSAGE-mean layer in float64 -> out[n_dst, d_out] float64 (unrounded)."""
    npdt = _NP_OF[dtype]
    Hsrc = _arr(Hsrc, npdt)
    W_self = _arr(W_self, npdt)
    W_neigh = _arr(W_neigh, npdt)
    bias = None if bias is None else _arr(bias, npdt)
    n_src, d_in = Hsrc.shape
    d_out = W_self.shape[1]
    assert W_self.shape == (d_in, d_out) and W_neigh.shape == (d_in, d_out)
    indptr = _arr(indptr, np.int32)
    idx = _arr(idx, np.int32)
    n_dst = len(indptr) - 1
    self_idx = None if self_idx is None else _arr(self_idx, np.int32)
    out = np.empty((n_dst, d_out), np.float64)
    rc = lib().orc_sage_fwd(_p(Hsrc), dtype, n_src, d_in, _p(self_idx), _p(indptr), _p(idx),
                            n_dst, _p(W_self), _p(W_neigh), _p(bias), d_out, int(bool(relu)),
                            _p(out))
    if rc:
        raise ValueError("orc_sage_fwd failed: %d" % rc)
    return out


def sage_agg_fwd(Hsrc, dtype, self_idx, indptr, idx, W_self, W_neigh, bias, agg, relu):
    """GraphSAGE layer with neighbour aggregator agg (0 mean, 1 sum, 2 max) in float64."""
    npdt = _NP_OF[dtype]
    Hsrc = _arr(Hsrc, npdt)
    W_self = _arr(W_self, npdt)
    W_neigh = _arr(W_neigh, npdt)
    bias = None if bias is None else _arr(bias, npdt)
    n_src, d_in = Hsrc.shape
    d_out = W_self.shape[1]
    assert W_self.shape == (d_in, d_out) and W_neigh.shape == (d_in, d_out)
    indptr = _arr(indptr, np.int32)
    idx = _arr(idx, np.int32)
    n_dst = len(indptr) - 1
    self_idx = None if self_idx is None else _arr(self_idx, np.int32)
    out = np.empty((n_dst, d_out), np.float64)
    rc = lib().orc_sage_agg_fwd(_p(Hsrc), dtype, n_src, d_in, _p(self_idx), _p(indptr), _p(idx), n_dst, _p(W_self),
                                _p(W_neigh), _p(bias), d_out, int(agg), int(bool(relu)), _p(out))
    if rc:
        raise ValueError("orc_sage_agg_fwd failed: %d" % rc)
    return out


def gcn_fwd(Hsrc, dtype, self_idx, indptr, idx, W, bias, norm, relu):
    """One GCN-style layer (norm 0: sum, 1: mean over the vertex and its neighbours) in float64."""
    npdt = _NP_OF[dtype]
    Hsrc = _arr(Hsrc, npdt)
    W = _arr(W, npdt)
    bias = None if bias is None else _arr(bias, npdt)
    n_src, d_in = Hsrc.shape
    d_out = W.shape[1]
    assert W.shape == (d_in, d_out)
    indptr = _arr(indptr, np.int32)
    idx = _arr(idx, np.int32)
    n_dst = len(indptr) - 1
    self_idx = None if self_idx is None else _arr(self_idx, np.int32)
    out = np.empty((n_dst, d_out), np.float64)
    rc = lib().orc_gcn_fwd(_p(Hsrc), dtype, n_src, d_in, _p(self_idx), _p(indptr), _p(idx), n_dst, _p(W),
                           _p(bias), d_out, int(norm), int(bool(relu)), _p(out))
    if rc:
        raise ValueError("orc_gcn_fwd failed: %d" % rc)
    return out


def gat_fwd(Hsrc, dtype, self_idx, indptr, idx, W, a_src, a_dst, bias, n_heads, relu):
    """One graph-attention layer (heads concatenated) in float64 -> out[n_dst, d_out]."""
    npdt = _NP_OF[dtype]
    Hsrc = _arr(Hsrc, npdt)
    W = _arr(W, npdt)
    a_src = _arr(a_src, npdt)
    a_dst = _arr(a_dst, npdt)
    bias = None if bias is None else _arr(bias, npdt)
    n_src, d_in = Hsrc.shape
    d_out = W.shape[1]
    assert W.shape == (d_in, d_out) and a_src.size == d_out and a_dst.size == d_out
    indptr = _arr(indptr, np.int32)
    idx = _arr(idx, np.int32)
    n_dst = len(indptr) - 1
    self_idx = None if self_idx is None else _arr(self_idx, np.int32)
    out = np.empty((n_dst, d_out), np.float64)
    rc = lib().orc_gat_fwd(_p(Hsrc), dtype, n_src, d_in, _p(self_idx), _p(indptr), _p(idx), n_dst, _p(W),
                           _p(a_src), _p(a_dst), _p(bias), d_out, int(n_heads), int(bool(relu)), _p(out))
    if rc:
        raise ValueError("orc_gat_fwd failed: %d" % rc)
    return out


def sage_bwd(Hsrc, dtype, self_idx, indptr, idx, W_self, W_neigh, out_fwd, relu, dOut, want_dH=True):
    """Backward of one layer in float64 -> (gW_self, gW_neigh, gbias, dHsrc-or-None), fresh arrays."""
    npdt = _NP_OF[dtype]
    Hsrc = _arr(Hsrc, npdt)
    W_self = _arr(W_self, npdt)
    W_neigh = _arr(W_neigh, npdt)
    n_src, d_in = Hsrc.shape
    d_out = W_self.shape[1]
    indptr = _arr(indptr, np.int32)
    idx = _arr(idx, np.int32)
    n_dst = len(indptr) - 1
    self_idx = None if self_idx is None else _arr(self_idx, np.int32)
    out_fwd = None if out_fwd is None else _arr(out_fwd, npdt)
    dOut = _arr(dOut, np.float64)
    assert dOut.shape == (n_dst, d_out)
    gWs = np.zeros((d_in, d_out), np.float64)
    gWn = np.zeros((d_in, d_out), np.float64)
    gb = np.zeros(d_out, np.float64)
    dH = np.zeros((n_src, d_in), np.float64) if want_dH else None
    rc = lib().orc_sage_bwd(_p(Hsrc), dtype, n_src, d_in, _p(self_idx), _p(indptr), _p(idx), n_dst, _p(W_self),
                            _p(W_neigh), _p(out_fwd), int(bool(relu)), _p(dOut), d_out, _p(gWs), _p(gWn), _p(gb),
                            _p(dH))
    if rc:
        raise ValueError("orc_sage_bwd failed: %d" % rc)
    return gWs, gWn, gb, dH


def _bwd_common(Hsrc, dtype, self_idx, indptr, idx, out_fwd, dOut, d_out):
    npdt = _NP_OF[dtype]
    Hsrc = _arr(Hsrc, npdt)
    indptr = _arr(indptr, np.int32)
    idx = _arr(idx, np.int32)
    n_dst = len(indptr) - 1
    self_idx = None if self_idx is None else _arr(self_idx, np.int32)
    out_fwd = None if out_fwd is None else _arr(out_fwd, npdt)
    dOut = _arr(dOut, np.float64)
    assert dOut.shape == (n_dst, d_out)
    return npdt, Hsrc, self_idx, indptr, idx, n_dst, out_fwd, dOut


def sage_agg_bwd(Hsrc, dtype, self_idx, indptr, idx, W_self, W_neigh, out_fwd, agg, relu, dOut, want_dH=True):
    """Backward of the GraphSAGE layer with aggregator agg (0 mean, 1 sum, 2 max) in float64
    -> (gW_self, gW_neigh, gbias, dHsrc-or-None), fresh arrays."""
    d_in, d_out = np.shape(W_self)
    npdt, Hsrc, self_idx, indptr, idx, n_dst, out_fwd, dOut = _bwd_common(Hsrc, dtype, self_idx, indptr, idx, out_fwd,
                                                                         dOut, d_out)
    W_self = _arr(W_self, npdt)
    W_neigh = _arr(W_neigh, npdt)
    n_src = Hsrc.shape[0]
    gWs = np.zeros((d_in, d_out), np.float64)
    gWn = np.zeros((d_in, d_out), np.float64)
    gb = np.zeros(d_out, np.float64)
    dH = np.zeros((n_src, d_in), np.float64) if want_dH else None
    rc = lib().orc_sage_agg_bwd(_p(Hsrc), dtype, n_src, d_in, _p(self_idx), _p(indptr), _p(idx), n_dst, _p(W_self),
                                _p(W_neigh), _p(out_fwd), int(agg), int(bool(relu)), _p(dOut), d_out, _p(gWs), _p(gWn),
                                _p(gb), _p(dH))
    if rc:
        raise ValueError("orc_sage_agg_bwd failed: %d" % rc)
    return gWs, gWn, gb, dH


def gcn_bwd(Hsrc, dtype, self_idx, indptr, idx, W, out_fwd, norm, relu, dOut, want_dH=True):
    """Backward of the GCN-style layer in float64 -> (gW, gbias, dHsrc-or-None), fresh arrays."""
    d_in, d_out = np.shape(W)
    npdt, Hsrc, self_idx, indptr, idx, n_dst, out_fwd, dOut = _bwd_common(Hsrc, dtype, self_idx, indptr, idx, out_fwd,
                                                                         dOut, d_out)
    W = _arr(W, npdt)
    n_src = Hsrc.shape[0]
    gW = np.zeros((d_in, d_out), np.float64)
    gb = np.zeros(d_out, np.float64)
    dH = np.zeros((n_src, d_in), np.float64) if want_dH else None
    rc = lib().orc_gcn_bwd(_p(Hsrc), dtype, n_src, d_in, _p(self_idx), _p(indptr), _p(idx), n_dst, _p(W), _p(out_fwd),
                           int(norm), int(bool(relu)), _p(dOut), d_out, _p(gW), _p(gb), _p(dH))
    if rc:
        raise ValueError("orc_gcn_bwd failed: %d" % rc)
    return gW, gb, dH


def gat_bwd(Hsrc, dtype, self_idx, indptr, idx, W, a_src, a_dst, out_fwd, n_heads, relu, dOut, want_dH=True):
    """Backward of the graph-attention layer in float64 -> (gW, ga_src, ga_dst, gbias, dHsrc-or-None)."""
    d_in, d_out = np.shape(W)
    npdt, Hsrc, self_idx, indptr, idx, n_dst, out_fwd, dOut = _bwd_common(Hsrc, dtype, self_idx, indptr, idx, out_fwd,
                                                                         dOut, d_out)
    W = _arr(W, npdt)
    a_src = _arr(a_src, npdt)
    a_dst = _arr(a_dst, npdt)
    n_src = Hsrc.shape[0]
    gW = np.zeros((d_in, d_out), np.float64)
    gas = np.zeros(d_out, np.float64)
    gad = np.zeros(d_out, np.float64)
    gb = np.zeros(d_out, np.float64)
    dH = np.zeros((n_src, d_in), np.float64) if want_dH else None
    rc = lib().orc_gat_bwd(_p(Hsrc), dtype, n_src, d_in, _p(self_idx), _p(indptr), _p(idx), n_dst, _p(W), _p(a_src),
                           _p(a_dst), _p(out_fwd), int(bool(relu)), _p(dOut), d_out, int(n_heads), _p(gW), _p(gas),
                           _p(gad), _p(gb), _p(dH))
    if rc:
        raise ValueError("orc_gat_bwd failed: %d" % rc)
    return gW, gas, gad, gb, dH


def sgd_update(W, dtype, grad, lr):
    """End of an iteration (paper section 5.1, step 5: the model parameters are updated from the
    accumulated, synchronised gradients; the optimiser is not named - reading: plain SGD):
    W <- W - lr * grad in float64, rounded once to W's storage dtype.  Returns the new W bits."""
    w = load_f64(W, dtype)
    return round_store(w - float(lr) * np.asarray(grad, np.float64).reshape(w.shape), dtype)


def forward(X_rows, dtype, ids, indptr, remap, n_seeds, fanouts, weights):
    """All L layers of one batch on top of its gathered rows.

    X_rows : Xu [U, D] in the storage dtype (uint16 bit patterns for 2-byte types)
    ids, remap : this batch's level-major slot arrays (length T)
    indptr : as returned by ``sample`` (children of slot r are ids[B+indptr[r] : B+indptr[r+1]])
    weights : list of (W_self, W_neigh, bias-or-None) per layer, storage dtype
    Returns the list of per-layer outputs, each (out64, out_stored).
    Layer k (1-based) produces rows for the slots of levels 0..L-k; its input is
    the previous layer's *stored* (rounded) output; ReLU on all but the last.
    Layer 1 reads the gathered rows through remap; later layers read the
    previous output, whose row of a slot is the slot number itself.
    """
    L = len(fanouts)
    lv = level_sizes(n_seeds, fanouts)
    B = n_seeds
    outs = []
    H = X_rows
    for k in range(1, L + 1):
        n_dst = sum(lv[:L - k + 1])
        ip = np.asarray(indptr[:n_dst + 1], np.int32)
        nnz = int(ip[n_dst])
        if k == 1:
            self_idx = remap[:n_dst]
            idx = remap[B:B + nnz]
        else:
            self_idx = None
            e = np.arange(nnz, dtype=np.int32)
            idx = np.where(ids[B:B + nnz] >= 0, B + e, -1).astype(np.int32)
        Ws, Wn, b = weights[k - 1]
        o64 = sage_fwd(H, dtype, self_idx, ip, idx, Ws, Wn, b, relu=(k < L))
        st = round_store(o64, dtype)
        outs.append((o64, st))
        H = st
    return outs
