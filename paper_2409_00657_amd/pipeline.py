"""Host-side sequencing of the hot path: buffers + the order of the C-ABI calls.

One *batch* is  sample -> pregather -> gather -> L x sage_fwd  for B root
vertices (paper sections 2 and 4); a *group* pre-gathers G batches' micrographs
in one merged fetch (paper section 5.2) and then runs each batch's layers.
Nothing here computes anything: every step is one call into libhopgnn.so, all
on torch's current stream, with no host synchronisation inside a batch.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

from . import binding as hb
from . import synth


@dataclass
class BatchShape:
    """Sizes of the level-major slot layout for B seeds and the given fanouts."""
    n_seeds: int
    fanouts: List[int]

    def __post_init__(self):
        self.n_layers = len(self.fanouts)
        self.levels = [self.n_seeds]
        p = 1
        for f in self.fanouts:
            p *= int(f)
            self.levels.append(self.n_seeds * p)
        self.n_slots = sum(self.levels)                 # T
        self.n_nonleaf = self.n_slots - self.levels[-1]  # S_{L-1}

    def n_dst(self, layer: int) -> int:
        """Destination rows of layer k (1-based): the slots of levels 0..L-k."""
        return sum(self.levels[: self.n_layers - layer + 1])

    def nnz(self, layer: int) -> int:
        return sum(self.levels[1: self.n_layers - layer + 2])

    @property
    def n_entries(self) -> int:
        """Entries of the whole tree's neighbour lists: one per slot below the roots."""
        return self.n_slots - self.n_seeds


@dataclass
class LayerwiseShape:
    """Capacities of layer-wise sampled micrographs for B seeds: `fanouts` holds the budget of
    draws per level, so level h has at most fanouts[h-1] nodes per micrograph."""
    n_seeds: int
    fanouts: List[int]

    def __post_init__(self):
        self.n_layers = len(self.fanouts)
        per = [1] + [int(s) for s in self.fanouts]
        self.levels = [self.n_seeds * s for s in per]
        self.n_slots = sum(self.levels)
        self.n_nonleaf = self.n_slots - self.levels[-1]
        self.n_entries = self.n_seeds * sum(a * b for a, b in zip(per[:-1], per[1:]))

    def n_dst(self, layer: int) -> int:
        return sum(self.levels[: self.n_layers - layer + 1])


class HotPath:
    """Pre-allocated device buffers for groups of `group` batches of one shape."""

    def __init__(self, offsets: torch.Tensor, indices: torch.Tensor, X: torch.Tensor,
                 weights, n_seeds: int, fanouts: Sequence[int], group: int = 1,
                 pg_algo: int = hb.PG_AUTO, model: str = "sage", gat_heads: int = 4, merge: bool = False,
                 fuse_tree: bool = True):
        """`weights`: per layer (W_self, W_neigh, bias-or-None).  model "sage" uses all three;
        "gcn" (mean over the vertex and its neighbours) and "gat" use W_self as the layer's one
        weight matrix, "gat" with seeded attention vectors and `gat_heads` heads.
        merge: the group's micrographs form ONE level-major batch of group * n_seeds micrographs
        (block b of n_seeds seeds keeps its own key), so every layer is one launch over the group;
        `shape`, `ids`, `remap`, `H` then describe that merged batch and `layer_batches` is 1.
        fuse_tree: the single-call path (`forward`) lets every projection but the last also form the
        next layer's neighbour means from the slot tree's shape (plan.fuse_tree; same last-layer bits);
        after it H[k] holds only the rows of the next layer's destinations.  The step-by-step calls
        (`layer`, `layers`, `run_batch`, `run_group`) always run the two-kernel layers."""
        if model not in ("sage", "gcn", "gat"):
            raise hb.HopgnnError("model must be sage, gcn or gat")
        self.model, self.gat_heads = model, gat_heads
        self.fuse_tree = bool(fuse_tree)
        dev = X.device
        self.offsets, self.indices, self.X, self.weights = offsets, indices, X, weights
        self.n_vertices = offsets.numel() - 1
        self.merge = bool(merge) and group > 1
        self.n_keys, self.seeds_per_key = group, n_seeds       # one key per block of n_seeds seeds
        if self.merge:
            n_seeds, group = n_seeds * group, 1
        self.layer_batches = group
        self.shape = sh = BatchShape(n_seeds, list(fanouts))
        self.group = group
        self.pg_algo = pg_algo
        T, S, B = sh.n_slots, sh.n_nonleaf, n_seeds
        i32 = dict(dtype=torch.int32, device=dev)
        self.ids = torch.empty(group * T, **i32)
        self.indptr = torch.empty(S + 1, **i32)          # the same for every batch of this shape
        self._slot_idx_all = torch.empty(group * max(S - B, 1), **i32)
        self.slot_idx = list(self._slot_idx_all.view(group, -1))
        self.remap = torch.empty(group * T, **i32)
        self.cap = min(group * T, self.n_vertices)
        self.uniq = torch.empty(self.cap, **i32)
        self.n_uniq = torch.zeros(1, dtype=torch.int64, device=dev)
        self.Xu = torch.empty((self.cap, X.shape[1]), dtype=X.dtype, device=dev)
        self.pg_ws = torch.empty(hb.hopgnn_pregather_ws_bytes(group * T, self.n_vertices, pg_algo),
                                 dtype=torch.uint8, device=dev)
        hidden = weights[0][0].shape[1]
        self.H = [torch.empty((sh.n_dst(k), hidden), dtype=X.dtype, device=dev)
                  for k in range(1, sh.n_layers + 1)]
        ws_bytes = max(hb.hopgnn_sage_fwd_ws_bytes(X.dtype, sh.n_dst(k), weights[k - 1][0].shape[0],
                                                   hidden) for k in range(1, sh.n_layers + 1))
        if model == "gcn":
            ws_bytes = max(ws_bytes, max(hb.hopgnn_gcn_fwd_ws_bytes(X.dtype, sh.n_dst(k), weights[k - 1][0].shape[0],
                                                                    hidden) for k in range(1, sh.n_layers + 1)))
        if model == "gat":
            self.attn = [(synth.weight(1, hidden, X.dtype, 200 + 2 * k, device=dev).view(-1),
                          synth.weight(1, hidden, X.dtype, 201 + 2 * k, device=dev).view(-1))
                         for k in range(sh.n_layers)]
            n_src = [self.cap] + [sh.n_dst(k) for k in range(1, sh.n_layers)]
            ws_bytes = max(ws_bytes, max(hb.hopgnn_gat_fwd_ws_bytes(X.dtype, n_src[k], weights[k][0].shape[0], hidden,
                                                                    gat_heads) for k in range(sh.n_layers)))
        self.sage_ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self._prepare_calls()

    def _prepare_calls(self) -> None:
        """Marshal every argument that never changes once: the buffers are fixed, so a batch only
        has to supply the seeds pointer, the key and the stream.  (At ~10 launches of a few
        microseconds each, per-call tensor slicing and pointer extraction in Python would cost
        more than the kernels.)"""
        lib = hb.load_library()
        sh = self.shape
        T, B, L, S = sh.n_slots, sh.n_seeds, sh.n_layers, sh.n_nonleaf
        self._csr = hb._Csr(self.n_vertices, self.indices.numel(), self.offsets.data_ptr(),
                            1 if self.offsets.dtype == torch.int64 else 0, self.indices.data_ptr())
        self._fan = (ctypes.c_int32 * L)(*sh.fanouts)
        ids, remap = self.ids.data_ptr(), self.remap.data_ptr()
        dt = hb.DTYPE_OF[self.X.dtype]
        self._lib = lib
        self._sample_args = [(ctypes.byref(self._csr), B, self._fan, L, ids + 4 * b * T,
                              self.indptr.data_ptr(),
                              self.slot_idx[b].data_ptr() if L > 1 else None) for b in range(self.group)]
        self._pregather_args = (ids, self.group * T, self.n_vertices, self.pg_algo, self.uniq.data_ptr(),
                                self.n_uniq.data_ptr(), remap, self.pg_ws.data_ptr(), self.pg_ws.numel())
        self._gather_args = (self.X.data_ptr(), dt, self.X.shape[0], self.X.shape[1], self.X.stride(0),
                             self.uniq.data_ptr(), self.cap, self.n_uniq.data_ptr(), self.Xu.data_ptr())
        self._layer_args = []
        for b in range(self.group):
            rb = remap + 4 * b * T
            src, n_src, per_batch = self.Xu.data_ptr(), self.cap, []
            for k in range(1, L + 1):
                n_dst, nnz = sh.n_dst(k), sh.nnz(k)
                Ws, Wn, bias = self.weights[k - 1]
                d_in, d_out = Ws.shape
                self_idx, idx = (rb, rb + 4 * B) if k == 1 else (None, self.slot_idx[b].data_ptr())
                bp = None if bias is None else bias.data_ptr()
                tail = (1 if k < L else 0, self.H[k - 1].data_ptr(), self.sage_ws.data_ptr(), self.sage_ws.numel())
                head = (src, dt, n_src, d_in, self_idx, self.indptr.data_ptr(), idx, n_dst, Ws.data_ptr())
                if self.model == "gat":     # layer 1 projects only the rows the pre-gather found
                    head = (src, dt, n_src, self.n_uniq.data_ptr() if k == 1 else None) + head[3:]
                if self.model == "sage":
                    per_batch.append(head + (Wn.data_ptr(), bp, d_out) + tail)
                elif self.model == "gcn":
                    per_batch.append(head + (bp, d_out, 1) + tail)
                else:
                    a_src, a_dst = self.attn[k - 1]
                    per_batch.append(head + (a_src.data_ptr(), a_dst.data_ptr(), bp, d_out, self.gat_heads) + tail)
                src, n_src = self.H[k - 1].data_ptr(), n_dst
            self._layer_args.append(per_batch)
        self._layer_fn = {"sage": lib.hopgnn_sage_fwd, "gcn": lib.hopgnn_gcn_fwd, "gat": lib.hopgnn_gat_fwd}[self.model]
        # the same buffers as one plan for hopgnn_batch_fwd (the launch sequence issued from C)
        pl = self.plan = hb.BatchPlan()
        pl.graph = self._csr
        pl.X, pl.dt, pl.dim, pl.ld_elems = self.X.data_ptr(), dt, self.X.shape[1], self.X.stride(0)
        pl.n_seeds, pl.n_layers = self.seeds_per_key, L
        for i, f in enumerate(sh.fanouts):
            pl.fanouts[i] = f
        for i, (Ws, Wn, bias) in enumerate(self.weights):
            pl.d_out[i] = Ws.shape[1]
            pl.W_self[i], pl.W_neigh[i] = Ws.data_ptr(), Wn.data_ptr()
            pl.bias[i] = None if bias is None else bias.data_ptr()
            pl.H[i] = self.H[i].data_ptr()
        pl.pg_algo, pl.group = self.pg_algo, self.n_keys
        pl.merge_layers = 1 if self.merge else 0
        pl.layer_kind = {"sage": 0, "gcn": 1, "gat": 2}[self.model]
        pl.gcn_norm, pl.gat_heads = 1, self.gat_heads
        if self.model == "gat":
            for i, (a_s, a_d) in enumerate(self.attn):
                pl.a_src[i], pl.a_dst[i] = a_s.data_ptr(), a_d.data_ptr()
        pl.ids, pl.indptr, pl.slot_idx = ids, self.indptr.data_ptr(), self._slot_idx_all.data_ptr()
        pl.uniq, pl.uniq_capacity, pl.n_uniq = self.uniq.data_ptr(), self.cap, self.n_uniq.data_ptr()
        pl.remap, pl.Xu = remap, self.Xu.data_ptr()
        pl.pg_ws, pl.pg_ws_bytes = self.pg_ws.data_ptr(), self.pg_ws.numel()
        pl.sage_ws, pl.sage_ws_bytes = self.sage_ws.data_ptr(), self.sage_ws.numel()
        pl.mark_begin = pl.mark_end = None
        # the fused slot-tree path: its scratch holds the transposed weights, so weights that change
        # (training) need prepare_weights() again; 0 bytes = the flag does not apply to this plan
        pl.fuse_tree = 1 if self.fuse_tree else 0
        pl.tree_ws, pl.tree_ws_bytes = None, 0
        n_tree = int(lib.hopgnn_batch_tree_ws_bytes(ctypes.byref(pl))) if self.fuse_tree else 0
        self.fused = n_tree > 0
        if self.fused:
            self.tree_ws = torch.empty(n_tree, dtype=torch.uint8, device=self.X.device)
            pl.tree_ws, pl.tree_ws_bytes = self.tree_ws.data_ptr(), n_tree
            self.prepare_weights()
        else:
            pl.fuse_tree = 0
        # every call of the library leaves the pre-gather workspace clean, so prepare it once
        hb.hopgnn_pregather_ws_init(self.pg_ws, self.group * T, self.n_vertices, self.pg_algo)
        pl.pg_ws_clean = 1
        self._keys = (ctypes.c_uint64 * self.n_keys)()

    def prepare_weights(self, stream=None) -> None:
        """(Re)build what the fused slot-tree path keeps of the weights (hopgnn_batch_prepare)."""
        if self.fused:
            rc = self._lib.hopgnn_batch_prepare(ctypes.byref(self.plan), self._stream(stream))
            if rc:
                hb._check(rc, "hopgnn_batch_prepare")

    # -- the four steps ------------------------------------------------------
    # `stream` is a raw hipStream_t (int); None = torch's current stream.

    @staticmethod
    def _stream(stream):
        return torch.cuda.current_stream().cuda_stream if stream is None else stream

    def sample(self, b: int, seeds: torch.Tensor, key: int, stream=None) -> None:
        if self.merge:
            raise hb.HopgnnError("a merged group is sampled with sample_group")
        g, B, fan, L, ids, indptr, slot_idx = self._sample_args[b]
        if seeds.numel() != B or seeds.dtype != torch.int32 or not seeds.is_cuda:
            raise hb.HopgnnError("seeds must be %d int32 values on the device" % B)
        rc = self._lib.hopgnn_sample(g, seeds.data_ptr(), B, fan, L, key & 0xFFFFFFFFFFFFFFFF, ids, indptr,
                                     slot_idx, self._stream(stream))
        if rc:
            hb._check(rc, "hopgnn_sample")

    def sample_group(self, seeds: torch.Tensor, keys: Sequence[int], stream=None) -> None:
        """All of the group's batches in one launch; `seeds` holds their seeds back to back."""
        n, B, L = len(keys), self.seeds_per_key, self.shape.n_layers
        if seeds.numel() != n * B or seeds.dtype != torch.int32 or not seeds.is_cuda or n > self.n_keys:
            raise hb.HopgnnError("seeds must be %d x %d int32 values on the device" % (n, B))
        for i, k in enumerate(keys):
            self._keys[i] = k & 0xFFFFFFFFFFFFFFFF
        if self.merge:
            if n != self.n_keys:
                raise hb.HopgnnError("a merged group is sampled whole: %d keys" % self.n_keys)
            rc = self._lib.hopgnn_sample_merged(ctypes.byref(self._csr), seeds.data_ptr(), n * B, B, self._fan, L,
                                                self._keys, self.ids.data_ptr(), self.indptr.data_ptr(),
                                                self._slot_idx_all.data_ptr() if L > 1 else None,
                                                self._stream(stream))
            if rc:
                hb._check(rc, "hopgnn_sample_merged")
            return
        rc = self._lib.hopgnn_sample_group(ctypes.byref(self._csr), seeds.data_ptr(), B, self._fan, L, self._keys, n,
                                           self.ids.data_ptr(), self.indptr.data_ptr(),
                                           self._slot_idx_all.data_ptr() if L > 1 else None,
                                           self._slot_idx_all.numel() // self.group, self._stream(stream))
        if rc:
            hb._check(rc, "hopgnn_sample_group")

    def pregather(self, stream=None) -> None:
        rc = self._lib.hopgnn_pregather(*self._pregather_args, self._stream(stream))
        if rc:
            hb._check(rc, "hopgnn_pregather")

    def gather(self, stream=None) -> None:
        rc = self._lib.hopgnn_gather(*self._gather_args, self._stream(stream))
        if rc:
            hb._check(rc, "hopgnn_gather")

    def layer(self, b: int, k: int, stream=None) -> torch.Tensor:
        """Layer k (1-based) of batch b; its input is Xu (k = 1) or H[k-2]."""
        rc = self._layer_fn(*self._layer_args[b][k - 1], self._stream(stream))
        if rc:
            hb._check(rc, "hopgnn_%s_fwd" % self.model)
        return self.H[k - 1]

    def layers(self, b: int, stream=None) -> torch.Tensor:
        st = self._stream(stream)
        for k in range(1, self.shape.n_layers + 1):
            self.layer(b, k, st)
        return self.H[-1]

    # -- backward (fp32 activations) ------------------------------------------

    def enable_backward(self) -> None:
        """Allocate gradient accumulators (one set per layer, fp32, zero) and the buffers of the
        backward pass.  Gradients are fp32 whatever the activation type.  The loss used by the
        harness is L = 1/2 |H_L|^2 for fp32 activations (dL/dH_L = H_L, read in place) and
        L = <G, H_L> with a fixed G for 2-byte activations (dL/dH_L = G, fp32).
        self.gW[k]: (gW_self, gW_neigh, gbias) for "sage"; (gW, None, gbias) for "gcn";
        (gW, None, gbias) plus self.g_attn[k] = (ga_src, ga_dst) for "gat"."""
        sh, dev, dt = self.shape, self.X.device, self.X.dtype
        L = sh.n_layers
        if dt == torch.float32:
            self.dHL = self.H[L - 1]
        else:
            self.dHL = synth.weight(self.H[L - 1].shape[0], self.H[L - 1].shape[1], torch.float32, stream=99,
                                    device=dev)
        z = lambda t: None if t is None else torch.zeros_like(t, dtype=torch.float32)
        if self.model == "sage":
            self.gW = [(z(Ws), z(Wn), z(b)) for Ws, Wn, b in self.weights]
        else:
            self.gW = [(z(Ws), None, z(b)) for Ws, Wn, b in self.weights]
        params = [(W, g) for layer, grads in zip(self.weights, self.gW) for W, g in zip(layer, grads) if g is not None]
        if self.model == "gat":
            self.g_attn = [(z(a_s), z(a_d)) for a_s, a_d in self.attn]
            params += [(a, g) for pair, grads in zip(self.attn, self.g_attn) for a, g in zip(pair, grads)]
        hidden = self.weights[0][0].shape[1]
        d_in_of = lambda k: self.weights[k - 1][0].shape[0]
        n_src_of = lambda k: self.cap if k == 1 else sh.n_dst(k - 1)
        # dH[k] = gradient of layer k's output rows (k = 1..L-1), produced by layer k+1's backward
        self.dH = [torch.empty((sh.n_dst(k), hidden), dtype=torch.float32, device=dev) for k in range(1, L)]
        if self.model == "gat":
            ws_bytes = max(hb.hopgnn_gat_bwd_ws_bytes(dt, n_src_of(k), sh.n_dst(k), d_in_of(k), hidden, self.gat_heads)
                           for k in range(1, L + 1))
            fwd_bytes = [hb.hopgnn_gat_fwd_ws_bytes(dt, n_src_of(k), d_in_of(k), hidden, self.gat_heads)
                         for k in range(1, L + 1)]
        else:
            ws_bytes = max(hb.hopgnn_sage_bwd_ws_bytes(dt, sh.n_dst(k), d_in_of(k), hidden, k > 1) for k in range(1, L + 1))
            fwd = hb.hopgnn_sage_fwd_ws_bytes if self.model == "sage" else hb.hopgnn_gcn_fwd_ws_bytes
            fwd_bytes = [fwd(dt, sh.n_dst(k), d_in_of(k), hidden) for k in range(1, L + 1)]
        self.bwd_ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self._sgd = hb.SgdTensors(params)
        # every layer gets a forward workspace of its own: what the forward call leaves there (the
        # neighbour means; z and the attention scores) is then still in place for the layer's backward call
        self._fwd_ws = [torch.empty(n, dtype=torch.uint8, device=dev) for n in fwd_bytes]
        for per_batch in self._layer_args:
            for k in range(L):
                per_batch[k] = per_batch[k][:-2] + (self._fwd_ws[k].data_ptr(), self._fwd_ws[k].numel())
        self._bwd_args = []
        hdt = hb.DTYPE_OF[dt]
        for b in range(self.group):
            rb = self.remap.data_ptr() + 4 * b * sh.n_slots
            per_batch = []
            for k in range(L, 0, -1):
                Ws, Wn, _bias = self.weights[k - 1]
                d_in, d_out = Ws.shape
                n_dst, n_src = sh.n_dst(k), n_src_of(k)
                src = self.Xu.data_ptr() if k == 1 else self.H[k - 2].data_ptr()
                self_idx, idx = (rb, rb + 4 * sh.n_seeds) if k == 1 else (None, self.slot_idx[b].data_ptr())
                indptr = self.indptr.data_ptr()
                out, relu = self.H[k - 1].data_ptr(), 1 if k < L else 0
                d_out_grad = self.dHL.data_ptr() if k == L else self.dH[k - 1].data_ptr()
                gWs, gWn, gb = self.gW[k - 1]
                gbp = None if gb is None else gb.data_ptr()
                dHsrc = self.dH[k - 2].data_ptr() if k > 1 else None
                ws = (self.bwd_ws.data_ptr(), self.bwd_ws.numel())
                if self.model == "sage":
                    tail = (Ws.data_ptr(), Wn.data_ptr(), out, self._fwd_ws[k - 1].data_ptr(), relu, d_out_grad, d_out,
                            gWs.data_ptr(), gWn.data_ptr(), gbp, dHsrc) + ws
                    if k > 1:   # neighbour lists in slot order: the input gradient is written without atomics
                        per_batch.append((self._lib.hopgnn_sage_bwd_slots,
                                          (src, hdt, n_src, d_in, indptr, idx, n_dst, sh.n_seeds) + tail))
                    else:
                        per_batch.append((self._lib.hopgnn_sage_bwd_dev,
                                          (src, hdt, n_src, None, d_in, self_idx, indptr, idx, n_dst, None) + tail))
                elif self.model == "gcn":
                    per_batch.append((self._lib.hopgnn_gcn_bwd,
                                      (src, hdt, n_src, d_in, self_idx, indptr, idx, n_dst, Ws.data_ptr(), out, 1, relu,
                                       d_out_grad, d_out, gWs.data_ptr(), gbp, dHsrc) + ws))
                else:
                    a_s, a_d = self.attn[k - 1]
                    ga_s, ga_d = self.g_attn[k - 1]
                    per_batch.append((self._lib.hopgnn_gat_bwd,
                                      (src, hdt, n_src, self.n_uniq.data_ptr() if k == 1 else None, d_in, self_idx, indptr,
                                       idx, n_dst, Ws.data_ptr(), a_s.data_ptr(), a_d.data_ptr(), out,
                                       self._fwd_ws[k - 1].data_ptr(), relu, d_out_grad, d_out, self.gat_heads,
                                       gWs.data_ptr(), ga_s.data_ptr(), ga_d.data_ptr(), gbp, dHsrc) + ws))
            self._bwd_args.append(per_batch)

    def backward(self, b: int, stream=None) -> None:
        """Backward of batch b's layers, last to first; weight gradients accumulate in self.gW."""
        st = self._stream(stream)
        for fn, a in self._bwd_args[b]:
            rc = fn(*a, st)
            if rc:
                hb._check(rc, fn.__name__)

    def apply_sgd(self, lr: float, stream=None) -> None:
        """End of an iteration: every weight matrix (and bias) takes its accumulated gradient,
        W <- W - lr * gW, and the accumulators are cleared."""
        self._sgd.update(lr, True, self._stream(stream))

    # -- whole steps ---------------------------------------------------------

    def run_batch(self, seeds: torch.Tensor, key: int, stream=None) -> torch.Tensor:
        """One batch (group size 1): returns the [B, hidden] output of the last layer."""
        st = self._stream(stream)
        self.sample(0, seeds, key, st)
        self.pregather(st)
        self.gather(st)
        return self.layers(0, st)

    def forward(self, seeds: torch.Tensor, keys: Sequence[int], out: torch.Tensor, stream=None,
                marks=None) -> None:
        """The whole group in ONE library call (hopgnn_batch_fwd): `seeds` holds the group's
        seeds back to back, `out` [group*B, hidden] receives every batch's last-layer rows.
        `marks` = (begin, end) raw hipEvent_t handles recorded around the gather launch, or
        (begin, end, stage) for another stage of the sequence (binding.MARK_*)."""
        n = len(keys)
        if seeds.numel() != n * self.seeds_per_key or seeds.dtype != torch.int32 or not seeds.is_cuda:
            raise hb.HopgnnError("seeds must be %d int32 values on the device" % (n * self.seeds_per_key))
        if out.numel() != n * self.seeds_per_key * self.H[-1].shape[1] or out.dtype != self.X.dtype \
                or not out.is_cuda or not out.is_contiguous():
            raise hb.HopgnnError("out must be a contiguous [n_batches*B, hidden] device tensor of X's type")
        for i, k in enumerate(keys):
            self._keys[i] = k & 0xFFFFFFFFFFFFFFFF
        pl = self.plan
        if marks is None:
            pl.mark_begin = pl.mark_end = None
        else:
            pl.mark_begin, pl.mark_end = marks[0], marks[1]
            pl.mark_stage = marks[2] if len(marks) > 2 else hb.MARK_GATHER
        rc = self._lib.hopgnn_batch_fwd(ctypes.byref(pl), seeds.data_ptr(), self._keys, n, out.data_ptr(),
                                        self._stream(stream))
        if rc:
            hb._check(rc, "hopgnn_batch_fwd")

    def run_group(self, seeds_list: Sequence[torch.Tensor], keys: Sequence[int],
                  outs: Optional[List[torch.Tensor]] = None, stream=None) -> None:
        """G batches share one pre-gather and one gather; `outs[b]` (if given)
        receives a copy of batch b's final rows."""
        assert len(seeds_list) == self.n_keys
        st = self._stream(stream)
        self.sample_group(torch.cat(list(seeds_list)) if len(seeds_list) > 1 else seeds_list[0], keys, st)
        self.pregather(st)
        self.gather(st)
        B = self.seeds_per_key
        for b in range(self.layer_batches):
            h = self.layers(b, st)
            if outs is not None:
                if self.merge:      # one launch per layer covered every batch of the group
                    for i in range(self.n_keys):
                        outs[i].copy_(h[i * B:(i + 1) * B])
                else:
                    outs[b].copy_(h)


class DedupPath:
    """The forward path over per-micrograph deduplicated frontiers (hopgnn_sample_dedup): the same
    rows for the seeds as HotPath, over fewer rows below them.  Node counts depend on the data, so
    every buffer has the slot tree's size and the layers take their row counts from the device."""

    def __init__(self, offsets: torch.Tensor, indices: torch.Tensor, X: torch.Tensor, weights, n_seeds: int,
                 fanouts: Sequence[int], pg_algo: int = hb.PG_AUTO, group: int = 1, sampler: str = "node",
                 model: str = "sage", gat_heads: int = 4):
        """`group` batches of n_seeds seeds form one merged batch (block b draws with key b).
        sampler "node": the node-wise draws of the slot tree, every (level, vertex) kept once;
        "layer": layer-wise sampling, `fanouts` then holds the budget of draws per level.
        model "sage" | "gcn" | "gat" as in HotPath (forward only for gcn and gat)."""
        if sampler not in ("node", "layer"):
            raise hb.HopgnnError("sampler must be node or layer")
        if model not in ("sage", "gcn", "gat"):
            raise hb.HopgnnError("model must be sage, gcn or gat")
        self.sampler, self.model, self.gat_heads = sampler, model, gat_heads
        dev = X.device
        self.offsets, self.indices, self.X, self.weights = offsets, indices, X, weights
        self.n_vertices = offsets.numel() - 1
        self.n_keys, self.seeds_per_key = group, n_seeds
        n_seeds = n_seeds * group
        self.shape = sh = (BatchShape if sampler == "node" else LayerwiseShape)(n_seeds, list(fanouts))
        T, S, B, L, E = sh.n_slots, sh.n_nonleaf, n_seeds, sh.n_layers, max(sh.n_entries, 1)
        self.capacity = T
        i32 = dict(dtype=torch.int32, device=dev)
        self.node_vertex = torch.empty(T, **i32)
        self.level_start = torch.zeros(L + 2, dtype=torch.int64, device=dev)
        self.indptr = torch.empty(S + 1, **i32)
        self.idx = torch.empty(E, **i32)
        self.idx_l1 = torch.empty(E, **i32)      # the first layer's list: positions in Xu
        self.remap = torch.empty(T, **i32)
        self.cap = min(T, self.n_vertices)
        self.uniq = torch.empty(self.cap, **i32)
        self.n_uniq = torch.zeros(1, dtype=torch.int64, device=dev)
        self.Xu = torch.empty((self.cap, X.shape[1]), dtype=X.dtype, device=dev)
        self.pg_algo = pg_algo
        self.pg_ws = torch.empty(hb.hopgnn_pregather_ws_bytes(T, self.n_vertices, pg_algo), dtype=torch.uint8, device=dev)
        ws_bytes = (hb.hopgnn_sample_dedup_ws_bytes if sampler == "node" else hb.hopgnn_sample_layerwise_ws_bytes)
        self.dd_ws = torch.empty(ws_bytes(B, list(fanouts)), dtype=torch.uint8, device=dev)
        hidden = weights[0][0].shape[1]
        self.H = [torch.empty((sh.n_dst(k), hidden), dtype=X.dtype, device=dev) for k in range(1, L + 1)]
        ws_layers = max(hb.hopgnn_sage_fwd_ws_bytes(X.dtype, sh.n_dst(k), weights[k - 1][0].shape[0], hidden)
                        for k in range(1, L + 1))
        if model == "gcn":
            ws_layers = max(ws_layers, max(hb.hopgnn_gcn_fwd_ws_bytes(X.dtype, sh.n_dst(k), weights[k - 1][0].shape[0],
                                                                      hidden) for k in range(1, L + 1)))
        if model == "gat":
            self.attn = [(synth.weight(1, hidden, X.dtype, 200 + 2 * k, device=dev).view(-1),
                          synth.weight(1, hidden, X.dtype, 201 + 2 * k, device=dev).view(-1)) for k in range(L)]
            n_src = [self.cap] + [sh.n_dst(k) for k in range(1, L)]
            ws_layers = max(ws_layers, max(hb.hopgnn_gat_fwd_ws_bytes(X.dtype, n_src[k], weights[k][0].shape[0], hidden,
                                                                      gat_heads) for k in range(L)))
        self.sage_ws = torch.empty(ws_layers, dtype=torch.uint8, device=dev)
        # row count of layer k = first node of level L-k+1: one-element views into level_start
        self._n_dst_dev = [self.level_start[L - k + 1:L - k + 2] for k in range(1, L + 1)]
        # the same buffers as a plan for hopgnn_batch_fwd (the sequence issued from C)
        pl = self.plan = hb.BatchPlan()
        pl.graph = hb._Csr(self.n_vertices, indices.numel(), offsets.data_ptr(),
                           1 if offsets.dtype == torch.int64 else 0, indices.data_ptr())
        pl.X, pl.dt, pl.dim, pl.ld_elems = X.data_ptr(), hb.DTYPE_OF[X.dtype], X.shape[1], X.stride(0)
        pl.n_seeds, pl.n_layers = self.seeds_per_key, L
        for i, f in enumerate(sh.fanouts):
            pl.fanouts[i] = f
        for i, (Ws, Wn, bias) in enumerate(weights):
            pl.d_out[i] = Ws.shape[1]
            pl.W_self[i], pl.W_neigh[i] = Ws.data_ptr(), Wn.data_ptr()
            pl.bias[i] = None if bias is None else bias.data_ptr()
            pl.H[i] = self.H[i].data_ptr()
        pl.pg_algo, pl.group, pl.dedup = pg_algo, self.n_keys, 1 if sampler == "node" else 2
        pl.layer_kind = {"sage": 0, "gcn": 1, "gat": 2}[model]
        pl.gcn_norm, pl.gat_heads = 1, gat_heads
        if model == "gat":
            for i, (a_s, a_d) in enumerate(self.attn):
                pl.a_src[i], pl.a_dst[i] = a_s.data_ptr(), a_d.data_ptr()
        pl.indptr, pl.uniq, pl.uniq_capacity, pl.n_uniq = self.indptr.data_ptr(), self.uniq.data_ptr(), self.cap, \
            self.n_uniq.data_ptr()
        pl.remap, pl.Xu = self.remap.data_ptr(), self.Xu.data_ptr()
        pl.pg_ws, pl.pg_ws_bytes = self.pg_ws.data_ptr(), self.pg_ws.numel()
        pl.sage_ws, pl.sage_ws_bytes = self.sage_ws.data_ptr(), self.sage_ws.numel()
        pl.node_vertex, pl.level_start = self.node_vertex.data_ptr(), self.level_start.data_ptr()
        pl.dd_idx, pl.dd_idx_l1 = self.idx.data_ptr(), self.idx_l1.data_ptr()
        pl.dd_ws, pl.dd_ws_bytes = self.dd_ws.data_ptr(), self.dd_ws.numel()
        # every call of the library leaves the pre-gather workspace clean, so prepare it once
        hb.hopgnn_pregather_ws_init(self.pg_ws, T, self.n_vertices, pg_algo)
        pl.pg_ws_clean = 1
        self._keys = (ctypes.c_uint64 * self.n_keys)()
        self._lib = hb.load_library()

    def _key_list(self, key):
        keys = list(key) if isinstance(key, (list, tuple)) else [key]
        if len(keys) != self.n_keys:
            raise hb.HopgnnError("one key per batch of the group: %d" % self.n_keys)
        return keys

    def forward(self, seeds: torch.Tensor, key, out: torch.Tensor, stream=None, marks=None) -> None:
        """The whole (merged) batch in ONE library call; `out` [group*B, hidden] receives the last
        layer's rows; `key`: one key per batch of the group; `marks` = (begin, end) raw hipEvent_t
        handles recorded around the gather launch."""
        n = self.shape.n_seeds
        if seeds.numel() != n or seeds.dtype != torch.int32 or not seeds.is_cuda:
            raise hb.HopgnnError("seeds must be %d int32 values on the device" % n)
        if out.numel() != n * self.H[-1].shape[1] or out.dtype != self.X.dtype or not out.is_cuda \
                or not out.is_contiguous():
            raise hb.HopgnnError("out must be a contiguous [group*B, hidden] device tensor of X's type")
        for i, k in enumerate(self._key_list(key)):
            self._keys[i] = k & 0xFFFFFFFFFFFFFFFF
        pl = self.plan
        pl.mark_begin, pl.mark_end = marks if marks is not None else (None, None)
        pl.mark_stage = hb.MARK_GATHER
        st = torch.cuda.current_stream().cuda_stream if stream is None else stream
        rc = self._lib.hopgnn_batch_fwd(ctypes.byref(pl), seeds.data_ptr(), self._keys, self.n_keys, out.data_ptr(), st)
        if rc:
            hb._check(rc, "hopgnn_batch_fwd")

    # the steps, all on torch's current stream
    def sample(self, seeds: torch.Tensor, key) -> None:
        fn = hb.hopgnn_sample_dedup if self.sampler == "node" else hb.hopgnn_sample_layerwise
        fn(self.offsets, self.indices, seeds, self.shape.fanouts, self._key_list(key), self.node_vertex,
           self.level_start, self.indptr, self.idx, self.dd_ws, seeds_per_key=self.seeds_per_key)

    def pregather(self) -> None:
        hb.hopgnn_pregather(self.node_vertex, self.n_vertices, self.uniq, self.n_uniq, self.remap, self.pg_ws,
                            self.pg_algo)

    def gather(self) -> None:
        hb.hopgnn_gather(self.X, self.uniq, self.cap, self.n_uniq, self.Xu)

    def compose(self) -> None:
        hb.hopgnn_compose_idx(self.idx, self.remap, self.idx_l1)

    def _layer_ws(self, k: int) -> torch.Tensor:
        """Layer k's forward workspace: its own once the backward pass is enabled, else the shared one."""
        return self._fwd_ws[k - 1] if hasattr(self, "_fwd_ws") else self.sage_ws

    def layer(self, k: int) -> torch.Tensor:
        sh = self.shape
        Ws, Wn, bias = self.weights[k - 1]
        n_dst = sh.n_dst(k)
        src, n_src = (self.Xu, self.cap) if k == 1 else (self.H[k - 2], sh.n_dst(k - 1))
        self_idx, idx = (self.remap[:n_dst], self.idx_l1) if k == 1 else (None, self.idx)
        n_dst_dev, relu = self._n_dst_dev[k - 1], k < sh.n_layers
        if self.model == "sage":
            hb.hopgnn_sage_fwd_dev(src, n_src, self_idx, self.indptr[:n_dst + 1], idx, n_dst, n_dst_dev, Ws, Wn, bias,
                                   hb.AGG_MEAN, relu, self.H[k - 1], self._layer_ws(k))
        elif self.model == "gcn":
            hb.hopgnn_gcn_fwd_dev(src, n_src, self_idx, self.indptr[:n_dst + 1], idx, n_dst, n_dst_dev, Ws, bias, 1, relu,
                                  self.H[k - 1], self.sage_ws)
        else:       # the source rows that exist: the pre-gathered rows, then the previous layer's rows
            a_src, a_dst = self.attn[k - 1]
            hb.hopgnn_gat_fwd_dev(src, n_src, self.n_uniq if k == 1 else self._n_dst_dev[k - 2], self_idx,
                                  self.indptr[:n_dst + 1], idx, n_dst, n_dst_dev, Ws, a_src, a_dst, bias, self.gat_heads,
                                  relu, self.H[k - 1], self.sage_ws)
        return self.H[k - 1]

    def enable_backward(self) -> None:
        """Gradient accumulators (fp32, zero) and the buffers of the backward pass over the frontier
        structure, as HotPath.enable_backward: the harness's loss is L = 1/2 |H_L|^2 for fp32
        activations (dL/dH_L = H_L, read in place) and L = <G, H_L> with a fixed G otherwise."""
        if self.model != "sage":
            raise hb.HopgnnError("backward is built for the GraphSAGE-mean layer")
        sh, dev = self.shape, self.X.device
        L = sh.n_layers
        hidden = self.weights[0][0].shape[1]
        if self.X.dtype == torch.float32:
            self.dHL = self.H[L - 1]
        else:
            self.dHL = synth.weight(sh.n_seeds, hidden, torch.float32, stream=99, device=dev)
        self.gW = [(torch.zeros_like(Ws, dtype=torch.float32), torch.zeros_like(Wn, dtype=torch.float32),
                    None if b is None else torch.zeros_like(b, dtype=torch.float32)) for Ws, Wn, b in self.weights]
        # dH[k-1] = gradient of layer k's output rows (k = 1..L-1), produced by layer k+1's backward
        self.dH = [torch.empty((sh.n_dst(k), hidden), dtype=torch.float32, device=dev) for k in range(1, L)]
        ws_bytes = max(hb.hopgnn_sage_bwd_ws_bytes(self.X.dtype, sh.n_dst(k), self.weights[k - 1][0].shape[0],
                                                   hidden, k > 1) for k in range(1, L + 1))
        self.bwd_ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self._sgd = hb.SgdTensors([(W, g) for layer, grads in zip(self.weights, self.gW) for W, g in zip(layer, grads)])
        # a forward workspace per layer: the means a layer leaves there serve its backward call
        self._fwd_ws = [torch.empty(hb.hopgnn_sage_fwd_ws_bytes(self.X.dtype, sh.n_dst(k), self.weights[k - 1][0].shape[0],
                                                                hidden), dtype=torch.uint8, device=dev)
                        for k in range(1, L + 1)]
        self._raw_calls()

    def _raw_calls(self):
        """The library calls of one step with every constant argument marshalled once (a step is a
        few dozen launches of microseconds each: per-call marshalling would dominate it)."""
        lib, sh, pl = self._lib, self.shape, self.plan
        L, dt = sh.n_layers, hb.DTYPE_OF[self.X.dtype]
        fan = (ctypes.c_int32 * L)(*sh.fanouts)
        self._fan = fan
        p = lambda t: None if t is None else t.data_ptr()
        sample = lib.hopgnn_sample_dedup if self.sampler == "node" else lib.hopgnn_sample_layerwise
        self._call_sample = (sample, (ctypes.byref(pl.graph),), (sh.n_seeds, self.seeds_per_key, fan, L, self._keys,
                             p(self.node_vertex), p(self.level_start), p(self.indptr), p(self.idx), p(self.dd_ws),
                             self.dd_ws.numel()))
        fwd = [(lib.hopgnn_pregather, (p(self.node_vertex), sh.n_slots, self.n_vertices, self.pg_algo, p(self.uniq),
                                       p(self.n_uniq), p(self.remap), p(self.pg_ws), self.pg_ws.numel())),
               (lib.hopgnn_gather, (p(self.X), dt, self.n_vertices, self.X.shape[1], self.X.stride(0), p(self.uniq),
                                    self.cap, p(self.n_uniq), p(self.Xu))),
               (lib.hopgnn_compose_idx, (p(self.idx), self.idx.numel(), p(self.remap), p(self.idx_l1)))]
        for k in range(1, L + 1):
            Ws, Wn, bias = self.weights[k - 1]
            n_dst = sh.n_dst(k)
            src, n_src = (self.Xu, self.cap) if k == 1 else (self.H[k - 2], sh.n_dst(k - 1))
            fwd.append((lib.hopgnn_sage_fwd_dev,
                        (p(src), dt, n_src, Ws.shape[0], p(self.remap) if k == 1 else None, p(self.indptr),
                         p(self.idx_l1 if k == 1 else self.idx), n_dst, p(self._n_dst_dev[k - 1]), p(Ws), p(Wn), p(bias),
                         Ws.shape[1], hb.AGG_MEAN, 1 if k < L else 0, p(self.H[k - 1]), p(self._layer_ws(k)),
                         self._layer_ws(k).numel())))
        self._calls_fwd = fwd
        bwd = []
        if hasattr(self, "gW"):
            for k in range(L, 0, -1):
                Ws, Wn, _bias = self.weights[k - 1]
                gWs, gWn, gb = self.gW[k - 1]
                n_dst = sh.n_dst(k)
                if k == 1:
                    src, n_src, n_src_dev = self.Xu, self.cap, None
                else:
                    src, n_src, n_src_dev = self.H[k - 2], sh.n_dst(k - 1), self._n_dst_dev[k - 2]
                bwd.append((lib.hopgnn_sage_bwd_dev,
                            (p(src), dt, n_src, p(n_src_dev), Ws.shape[0], p(self.remap) if k == 1 else None,
                             p(self.indptr), p(self.idx_l1 if k == 1 else self.idx), n_dst, p(self._n_dst_dev[k - 1]),
                             p(Ws), p(Wn), p(self.H[k - 1]), p(self._fwd_ws[k - 1]), 1 if k < L else 0,
                             p(self.dHL if k == L else self.dH[k - 1]),
                             Ws.shape[1], p(gWs), p(gWn), p(gb), p(self.dH[k - 2]) if k > 1 else None, p(self.bwd_ws),
                             self.bwd_ws.numel())))
        self._calls_bwd = bwd

    def train_step(self, seeds: torch.Tensor, key, lr: float, stream=None, marks=None) -> None:
        """One iteration on `stream` (a raw hipStream_t, default torch's current one): forward call
        by call, backward with in-place accumulation, update.  `marks` as in run_batch."""
        if not hasattr(self, "gW"):
            raise hb.HopgnnError("enable_backward first")
        st = torch.cuda.current_stream().cuda_stream if stream is None else stream
        for i, k in enumerate(self._key_list(key)):
            self._keys[i] = k & 0xFFFFFFFFFFFFFFFF
        fn, head, tail = self._call_sample
        rc = fn(*head, seeds.data_ptr(), *tail, st)
        if rc:
            hb._check(rc, "sampling")
        for n, (fn, args) in enumerate(self._calls_fwd):
            if marks is not None and n == 1:
                marks[0].record()
            rc = fn(*args, st)
            if rc:
                hb._check(rc, fn.__name__)
            if marks is not None and n == 1:
                marks[1].record()
        for fn, args in self._calls_bwd:
            rc = fn(*args, st)
            if rc:
                hb._check(rc, fn.__name__)
        self._sgd.update(lr, True, st)

    def backward(self) -> None:
        """Backward of the layers of the batch last run by run_batch, last layer first; weight
        gradients accumulate in self.gW.  Row counts come from level_start on the device."""
        sh = self.shape
        L = sh.n_layers
        for k in range(L, 0, -1):
            Ws, Wn, _bias = self.weights[k - 1]
            gWs, gWn, gb = self.gW[k - 1]
            n_dst = sh.n_dst(k)
            if k == 1:
                src, n_src, n_src_dev = self.Xu, self.cap, None
            else:
                src, n_src, n_src_dev = self.H[k - 2], sh.n_dst(k - 1), self._n_dst_dev[k - 2]
            hb.hopgnn_sage_bwd_dev(src, n_src, n_src_dev, self.remap[:n_dst] if k == 1 else None,
                                   self.indptr[:n_dst + 1], self.idx_l1 if k == 1 else self.idx, n_dst,
                                   self._n_dst_dev[k - 1], Ws, Wn, self.H[k - 1], k < L,
                                   self.dHL if k == L else self.dH[k - 1], gWs, gWn, gb,
                                   self.dH[k - 2] if k > 1 else None, self.bwd_ws, mean_fwd=self._fwd_ws[k - 1])

    def apply_sgd(self, lr: float) -> None:
        """W <- W - lr * gW for every weight matrix and bias; the accumulators are cleared."""
        self._sgd.update(lr, True)

    def run_batch(self, seeds: torch.Tensor, key, marks=None) -> torch.Tensor:
        """Returns the [group*B, hidden] rows of the last layer (level 0 always has every root).
        `marks` = (begin, end) torch events recorded around the gather launch."""
        self.sample(seeds, key)
        self.pregather()
        if marks is not None:
            marks[0].record()
        self.gather()
        if marks is not None:
            marks[1].record()
        self.compose()
        for k in range(1, self.shape.n_layers + 1):
            self.layer(k)
        return self.H[-1]
