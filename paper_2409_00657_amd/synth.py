"""Seeded synthetic inputs: graphs, feature tables, seed lists, weights.

This module serves both the CPU oracle's tests and the GPU path.  It holds
none of the method's arithmetic (no sampling hash, no dedup, no layer math):
it only produces *inputs*, from a counter-based generator of its own (the
64-bit finaliser of MurmurHash3, which the method does not use), so a table
can be produced in chunks, on the host or on the device, and always comes out
the same for a given seed on a given device type.

The graphs stand in for the datasets the paper trains on (OGB-Arxiv,
OGB-Products, UK, IN, IT, Papers100M), which are not available here; only
their shapes (vertex/edge counts, feature widths, skewed degrees) are kept.

All generators return torch tensors on ``device``.
"""
from __future__ import annotations

import math
import os
from dataclasses import dataclass, field
from typing import List, Optional

import torch

DEFAULT_SEED = 0x5EED
_M64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Python int (mod 2^64) -> the int64 two's-complement value torch can hold."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def fmix64(x: torch.Tensor) -> torch.Tensor:
    """MurmurHash3 64-bit finaliser on int64 tensors (wrap-around arithmetic)."""
    x = x ^ _lsr(x, 33)
    x = x * _s64(0xFF51AFD7ED558CCD)
    x = x ^ _lsr(x, 33)
    x = x * _s64(0xC4CEB9FE1A85EC53)
    x = x ^ _lsr(x, 33)
    return x


def counter_bits(seed: int, stream: int, n: int, device, start: int = 0) -> torch.Tensor:
    """n pseudo-random int64 words: word i depends only on (seed, stream, start+i)."""
    base = _s64(((seed * 0x9E3779B97F4A7C15) ^ (stream * 0xD1B54A32D192ED03)) & _M64)
    ctr = torch.arange(start, start + n, dtype=torch.int64, device=device)
    return fmix64(fmix64(ctr + base) ^ _s64(0xA0761D6478BD642F * (stream + 1)))


def uniform01(bits: torch.Tensor) -> torch.Tensor:
    """float64 in [0,1) from the top 53 bits."""
    return _lsr(bits, 11).to(torch.float64) * (1.0 / (1 << 53))


def _normalish(bits: torch.Tensor) -> torch.Tensor:
    """~N(0,1) fp32 without transcendentals: sum of the four 16-bit lanes of a
    word (Irwin-Hall, variance 4*(2^32-1)/12), centred and scaled."""
    s = (bits & 0xFFFF) + (_lsr(bits, 16) & 0xFFFF) + (_lsr(bits, 32) & 0xFFFF) + _lsr(bits, 48)
    scale = 1.0 / math.sqrt(4.0 * ((1 << 32) - 1) / 12.0)
    return ((s - 2 * 65535).to(torch.float32)) * scale


# ------------------------------------------------------------------ graphs --

@dataclass
class Graph:
    n_vertices: int
    offsets: torch.Tensor      # [N+1] int32 or int64
    indices: torch.Tensor      # [E] int32
    name: str = ""

    @property
    def n_edges(self) -> int:
        return int(self.indices.numel())


def _stochastic_round(w: torch.Tensor, seed: int, stream: int) -> torch.Tensor:
    u = uniform01(counter_bits(seed, stream, w.numel(), w.device))
    fl = torch.floor(w)
    return (fl + (u < (w - fl)).to(w.dtype)).to(torch.int64)


def _offsets_from_degrees(deg: torch.Tensor, i64: bool) -> torch.Tensor:
    off = torch.zeros(deg.numel() + 1, dtype=torch.int64, device=deg.device)
    torch.cumsum(deg, 0, out=off[1:])
    if not i64:
        assert int(off[-1]) < 2 ** 31
        off = off.to(torch.int32)
    return off


def _edge_sources(off: torch.Tensor, lo: int, hi: int) -> torch.Tensor:
    """Source vertex of edges lo..hi-1 (CSR row lookup)."""
    e = torch.arange(lo, hi, dtype=torch.int64, device=off.device)
    return torch.searchsorted(off.to(torch.int64), e, right=True) - 1


def uniform_graph(n: int, deg_lo: int, deg_hi: int, seed: int = DEFAULT_SEED,
                  device="cpu", offsets_i64: bool = False) -> Graph:
    """Out-degree uniform in [deg_lo, deg_hi], every target uniform in [0, n)."""
    span = deg_hi - deg_lo + 1
    deg = deg_lo + (_lsr(counter_bits(seed, 1, n, device), 1) % span)
    off = _offsets_from_degrees(deg, offsets_i64)
    E = int(off[-1])
    idx = (_lsr(counter_bits(seed, 2, E, device), 1) % n).to(torch.int32)
    return Graph(n, off, idx, "uniform")


def rmat_graph(scale: int, avg_degree: float, a=0.57, b=0.19, c=0.19, d=0.05,
               seed: int = DEFAULT_SEED, device="cpu", offsets_i64: bool = False,
               chunk: int = 1 << 25) -> Graph:
    """Row-conditional R-MAT: the out-degree of i is a stochastic rounding of
    E*(a+b)^zeros(i)*(c+d)^ones(i); each target bit is 0 with probability
    a/(a+b) where the source bit is 0, c/(c+d) where it is 1.  Same edge
    distribution as edge-list R-MAT (Poissonised), but yields CSR directly."""
    n = 1 << scale
    E_target = avg_degree * n
    v = torch.arange(n, dtype=torch.int64, device=device)
    ones = torch.zeros(n, dtype=torch.int64, device=device)
    for k in range(scale):
        ones += (v >> k) & 1
    w = E_target * torch.pow(torch.tensor(a + b, dtype=torch.float64, device=device),
                             (scale - ones).to(torch.float64)) \
        * torch.pow(torch.tensor(c + d, dtype=torch.float64, device=device),
                    ones.to(torch.float64))
    deg = _stochastic_round(w, seed, 11)
    off = _offsets_from_degrees(deg, offsets_i64)
    E = int(off[-1])
    idx = torch.empty(E, dtype=torch.int32, device=device)
    p0, p1 = a / (a + b), c / (c + d)
    for lo in range(0, E, chunk):
        hi = min(E, lo + chunk)
        src = _edge_sources(off, lo, hi)
        dst = torch.zeros(hi - lo, dtype=torch.int64, device=device)
        for k in range(scale):
            u = uniform01(counter_bits(seed, 100 + k, hi - lo, device, start=lo))
            sb = (src >> k) & 1
            thr = torch.where(sb == 0, p0, p1)
            dst |= (u >= thr).to(torch.int64) << k
        idx[lo:hi] = dst.to(torch.int32)
    return Graph(n, off, idx, "rmat")


def chung_lu_graph(n: int, avg_degree: float, gamma: float, seed: int = DEFAULT_SEED,
                   device="cpu", offsets_i64: bool = True, chunk: int = 1 << 25) -> Graph:
    """Expected-degree power-law graph: w_i ~ (i+i0)^(-1/(gamma-1)) scaled to the
    mean degree and capped at sqrt(sum w); out-degree = stochastic rounding of
    w_i; every target is drawn with probability proportional to w (inverse CDF).
    Multi-edges and self-loops are kept."""
    i = torch.arange(n, dtype=torch.float64, device=device)
    w = torch.pow(i + 10.0, -1.0 / (gamma - 1.0))
    w *= (avg_degree * n) / float(w.sum())
    for _ in range(4):   # cap hubs, then rescale the rest back to the mean
        cap = math.sqrt(float(w.sum()))
        w = torch.clamp(w, max=cap)
        w *= (avg_degree * n) / float(w.sum())
    w = torch.clamp(w, max=math.sqrt(float(w.sum())))
    deg = _stochastic_round(w, seed, 21)
    off = _offsets_from_degrees(deg, offsets_i64)
    E = int(off[-1])
    cdf = torch.cumsum(w, 0)
    total = float(cdf[-1])
    idx = torch.empty(E, dtype=torch.int32, device=device)
    for lo in range(0, E, chunk):
        hi = min(E, lo + chunk)
        u = uniform01(counter_bits(seed, 22, hi - lo, device, start=lo)) * total
        idx[lo:hi] = torch.clamp(torch.searchsorted(cdf, u, right=True), max=n - 1).to(torch.int32)
    return Graph(n, off, idx, "chung_lu")


# ---------------------------------------------------------------- features --

def features(n: int, d: int, dtype: torch.dtype, seed: int = DEFAULT_SEED, device="cpu",
             chunk_rows: Optional[int] = None) -> torch.Tensor:
    """[n, d] table, ~N(0,1), element (r, c) a function of (seed, r*d+c) only."""
    X = torch.empty((n, d), dtype=dtype, device=device)
    if chunk_rows is None:
        chunk_rows = max(1, (1 << 26) // d)
    for lo in range(0, n, chunk_rows):
        hi = min(n, lo + chunk_rows)
        bits = counter_bits(seed, 31, (hi - lo) * d, device, start=lo * d)
        X[lo:hi] = _normalish(bits).view(hi - lo, d).to(dtype)
    return X


def seeds(n_vertices: int, batch: int, iteration: int, seed: int = DEFAULT_SEED,
          device="cpu") -> torch.Tensor:
    """`batch` root vertices drawn uniformly (with replacement) for one iteration."""
    bits = counter_bits(seed, 41, batch, device, start=iteration * batch)
    return (_lsr(bits, 1) % n_vertices).to(torch.int32)


def weight(d_in: int, d_out: int, dtype: torch.dtype, stream: int, seed: int = DEFAULT_SEED,
           device="cpu") -> torch.Tensor:
    """[d_in, d_out] ~ N(0, 1/sqrt(d_in)) (standard deviation 1/sqrt(fan_in))."""
    bits = counter_bits(seed, 1000 + stream, d_in * d_out, device)
    return (_normalish(bits) * (1.0 / math.sqrt(d_in))).view(d_in, d_out).to(dtype)


def sage_weights(d_in: int, hidden: int, n_layers: int, dtype: torch.dtype,
                 seed: int = DEFAULT_SEED, device="cpu", bias: bool = False):
    """Per layer (W_self, W_neigh, bias-or-None); layer 1 maps d_in -> hidden."""
    out = []
    for k in range(n_layers):
        di = d_in if k == 0 else hidden
        Ws = weight(di, hidden, dtype, 3 * k, seed, device)
        Wn = weight(di, hidden, dtype, 3 * k + 1, seed, device)
        b = None
        if bias:
            b = (_normalish(counter_bits(seed, 1000 + 3 * k + 2, hidden, device)) * 0.1).to(dtype)
        out.append((Ws, Wn, b))
    return out


# ----------------------------------------------------------------- configs --

@dataclass
class Config:
    """One of the five workload shapes (graph recipe, feature table, batch)."""
    name: str
    graph: str                     # "uniform" | "rmat" | "chung_lu"
    n_vertices: int
    avg_degree: float
    offsets_i64: bool
    d: int
    dtype: torch.dtype
    batch: int
    fanouts: List[int]
    hidden: int
    gamma: float = 0.0
    scale: int = 0
    groups: List[int] = field(default_factory=lambda: [1])

    def _cache_file(self, what: str, seed: int, device) -> Optional[str]:
        """Where HOPGNN_SYNTH_CACHE=<dir> keeps a generated input (None: no cache).  The generators are
        deterministic, so a cached tensor is the generated one; the cache exists so that a run under a
        counter-collecting profiler need not execute the generators' kernels."""
        d = os.environ.get("HOPGNN_SYNTH_CACHE")
        if not d:
            return None
        os.makedirs(d, exist_ok=True)
        kind = torch.device(device).type
        return os.path.join(d, "%s-%s-%x-%s.pt" % (self.name, what, seed, kind))

    def make_graph(self, seed=DEFAULT_SEED, device="cpu") -> Graph:
        path = self._cache_file("graph", seed, device)
        if path and os.path.exists(path):
            t = torch.load(path, map_location="cpu", weights_only=True)
            return Graph(self.n_vertices, t["offsets"].to(device), t["indices"].to(device), self.graph)
        if self.graph == "uniform":
            g = uniform_graph(self.n_vertices, 8, 16, seed, device, self.offsets_i64)
        elif self.graph == "rmat":
            g = rmat_graph(self.scale, self.avg_degree, seed=seed, device=device, offsets_i64=self.offsets_i64)
        else:
            g = chung_lu_graph(self.n_vertices, self.avg_degree, self.gamma, seed, device, self.offsets_i64)
        if path:
            torch.save({"offsets": g.offsets.cpu(), "indices": g.indices.cpu()}, path)
        return g

    def make_features(self, seed=DEFAULT_SEED, device="cpu") -> torch.Tensor:
        path = self._cache_file("features", seed, device)
        if path and os.path.exists(path):
            return torch.load(path, map_location="cpu", weights_only=True).to(device)
        X = features(self.n_vertices, self.d, self.dtype, seed, device)
        if path:
            torch.save(X.cpu(), path)
        return X

    def make_weights(self, seed=DEFAULT_SEED, device="cpu"):
        return sage_weights(self.d, self.hidden, len(self.fanouts), self.dtype, seed, device)


CONFIGS = {
    1: Config("cfg1-uniform-20k", "uniform", 20_000, 12, False, 32, torch.float32, 64, [5, 5], 32),
    2: Config("cfg2-rmat-s20", "rmat", 1 << 20, 16, False, 128, torch.float32, 1024, [10, 10], 128,
              scale=20),
    3: Config("cfg3-chunglu-2.4M", "chung_lu", 2_400_000, 62e6 / 2.4e6, True, 100, torch.float32,
              1024, [15, 10, 5], 256, gamma=2.1),
    4: Config("cfg4-rmat-s24", "rmat", 1 << 24, 32, True, 256, torch.bfloat16, 4096, [25, 10], 256,
              scale=24),
    5: Config("cfg5-chunglu-100M", "chung_lu", 100_000_000, 12, True, 128, torch.float16, 512,
              [10, 10, 10], 512, gamma=2.0, groups=[8, 16, 32, 64]),
}
