"""Host-side sequencing of the hot path: buffers + the order of the C-ABI calls.

One *batch* is  sample -> pregather -> gather -> L x sage_fwd  for B root
vertices (paper sections 2 and 4); a *group* pre-gathers G batches' micrographs
in one merged fetch (paper section 5.2) and then runs each batch's layers.
Nothing here computes anything: every step is one call into libhopgnn.so, all
on torch's current stream, with no host synchronisation inside a batch.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

from . import binding as hb


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


class HotPath:
    """Pre-allocated device buffers for groups of `group` batches of one shape."""

    def __init__(self, offsets: torch.Tensor, indices: torch.Tensor, X: torch.Tensor,
                 weights, n_seeds: int, fanouts: Sequence[int], group: int = 1,
                 pg_algo: int = hb.PG_AUTO):
        dev = X.device
        self.offsets, self.indices, self.X, self.weights = offsets, indices, X, weights
        self.n_vertices = offsets.numel() - 1
        self.shape = sh = BatchShape(n_seeds, list(fanouts))
        self.group = group
        self.pg_algo = pg_algo
        T, S, B = sh.n_slots, sh.n_nonleaf, n_seeds
        i32 = dict(dtype=torch.int32, device=dev)
        self.ids = torch.empty(group * T, **i32)
        self.indptr = torch.empty(S + 1, **i32)          # the same for every batch of this shape
        self.slot_idx = [torch.empty(max(S - B, 1), **i32) for _ in range(group)]
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
        self.sage_ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    # -- the four steps ------------------------------------------------------

    def sample(self, b: int, seeds: torch.Tensor, key: int) -> None:
        T = self.shape.n_slots
        hb.hopgnn_sample(self.offsets, self.indices, seeds, self.shape.fanouts, key,
                         self.ids[b * T:(b + 1) * T], self.indptr,
                         self.slot_idx[b] if self.shape.n_layers > 1 else None)

    def pregather(self) -> None:
        hb.hopgnn_pregather(self.ids, self.n_vertices, self.uniq, self.n_uniq, self.remap,
                            self.pg_ws, self.pg_algo)

    def gather(self) -> None:
        hb.hopgnn_gather(self.X, self.uniq, self.cap, self.n_uniq, self.Xu)

    def layers(self, b: int) -> torch.Tensor:
        sh = self.shape
        T, B, L = sh.n_slots, sh.n_seeds, sh.n_layers
        remap = self.remap[b * T:(b + 1) * T]
        src, n_src = self.Xu, self.cap
        for k in range(1, L + 1):
            n_dst, nnz = sh.n_dst(k), sh.nnz(k)
            Ws, Wn, bias = self.weights[k - 1]
            if k == 1:
                self_idx, idx = remap[:n_dst], remap[B:B + nnz]
            else:
                self_idx, idx = None, self.slot_idx[b][:nnz]
            hb.hopgnn_sage_fwd(src, n_src, self_idx, self.indptr[:n_dst + 1], idx, n_dst, Ws, Wn,
                               bias, k < L, self.H[k - 1], self.sage_ws)
            src, n_src = self.H[k - 1], n_dst
        return self.H[L - 1]

    # -- whole steps ---------------------------------------------------------

    def run_batch(self, seeds: torch.Tensor, key: int) -> torch.Tensor:
        """One batch (group size 1): returns the [B, hidden] output of the last layer."""
        self.sample(0, seeds, key)
        self.pregather()
        self.gather()
        return self.layers(0)

    def run_group(self, seeds_list: Sequence[torch.Tensor], keys: Sequence[int],
                  outs: Optional[List[torch.Tensor]] = None) -> None:
        """G batches share one pre-gather and one gather; `outs[b]` (if given)
        receives a copy of batch b's final rows."""
        assert len(seeds_list) == self.group
        for b, (s, k) in enumerate(zip(seeds_list, keys)):
            self.sample(b, s, k)
        self.pregather()
        self.gather()
        for b in range(self.group):
            h = self.layers(b)
            if outs is not None:
                outs[b].copy_(h)
