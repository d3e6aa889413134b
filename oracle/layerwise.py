"""Oracle for layer-wise sampling of micrographs.  TEST INFRASTRUCTURE ONLY.

The paper's locality study (section 4, the table of micrograph locality) samples micrographs both
node-wise and layer-wise, naming FastGCN for the latter and giving no further detail.  The reading
taken here, per micrograph (one root) and hop h = 1..L with a budget of s_h draws for the WHOLE
layer instead of a fanout per vertex:

  candidates   the neighbour lists of the previous level's nodes, concatenated in node order
               (ascending vertex) and list order; D = their total length
  draws        s_h positions p_j = hash64(key, root, -1, h, j) mod D, with replacement; the drawn
               vertex is the candidate at that position, so a vertex is drawn with probability
               proportional to the number of edges from the previous level into it (the
               layer-dependent importance distribution; draws over the whole vertex set would leave
               a one-root micrograph disconnected on any large graph)
  nodes        the ascending distinct drawn vertices (at most s_h); none if D = 0
  edges        as in layer-wise sampling every edge between the two node sets is kept: a
               previous-level node u is joined to every level-h node adjacent to it, each pair once
               (the 0/1 adjacency restricted to the two sets); the layer averages over them

Output in the layout of the deduplicated frontiers (level-major global numbering, CSR of positions
in the next level), with variable segment lengths and no -1 entries.
"""
from __future__ import annotations

import numpy as np

from . import hash64

TAG = -1        # the "vertex" field of a whole-layer draw: no vertex has this id


def sample_layerwise(offsets, indices, seeds, budgets, key=0):
    """`key`: one integer, or one per micrograph.
    Returns (node_vertex [n_nodes], level_start [L+2], indptr [n_nonleaf+1], idx [nnz])."""
    offsets = np.asarray(offsets)
    indices = np.asarray(indices)
    B, L = len(seeds), len(budgets)
    keys = [int(key)] * B if np.isscalar(key) else [int(k) for k in key]
    assert len(keys) == B
    per_level = [[np.array([int(s)], np.int64) for s in seeds]]
    segs = []        # per hop: per micrograph: list over previous-level nodes of position arrays
    for h in range(1, L + 1):
        s_h = int(budgets[h - 1])
        nxt, seg_h = [], []
        for m in range(B):
            root, prev = int(seeds[m]), per_level[h - 1][m]
            lists = [indices[int(offsets[u]):int(offsets[u + 1])] for u in prev]
            cand = np.concatenate(lists) if lists else np.zeros(0, np.int64)
            D = len(cand)
            if D == 0:
                nodes = np.zeros(0, np.int64)
            else:
                drawn = [int(cand[hash64(keys[m], root, TAG, h, j) % D]) for j in range(s_h)]
                nodes = np.unique(np.asarray(drawn, np.int64))
            nxt.append(nodes)
            seg_h.append([np.searchsorted(nodes, np.intersect1d(lst, nodes)) for lst in lists])
        per_level.append(nxt)
        segs.append(seg_h)
    counts = [[len(a) for a in lvl] for lvl in per_level]
    level_start = np.zeros(L + 2, np.int64)
    for h in range(L + 1):
        level_start[h + 1] = level_start[h] + sum(counts[h])
    node_vertex = np.concatenate([a for lvl in per_level for a in lvl])
    indptr, idx = [0], []
    for h in range(L):
        mg_off_next = np.concatenate([[0], np.cumsum(counts[h + 1])])
        for m in range(B):
            for pos in segs[h][m]:
                idx.extend(int(level_start[h + 1] + mg_off_next[m] + p) for p in pos)
                indptr.append(len(idx))
    return (node_vertex.astype(np.int32), level_start, np.asarray(indptr, np.int32), np.asarray(idx, np.int32))


from .frontier import layer_chain  # noqa: E402,F401  (the layers over the structure)
