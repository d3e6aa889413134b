"""Oracle for GraphSAGE-mean layers over a level-major frontier structure (the output layout of
the deduplicated-frontier and the layer-wise samplers).  TEST INFRASTRUCTURE ONLY.

Nodes are numbered level by level; layer k (1-based) computes the rows of levels 0..L-k from those
of levels 0..L-k+1 (paper section 2, "computation": one layer per hop, from the outermost inwards);
the first layer reads the pre-gathered feature rows (section 5.2).  Every step is one of the
oracle package's pinned functions (pre-gather, gather, the layer and its backward)."""
from __future__ import annotations

import numpy as np


def layer_inputs(k, L, level_start, indptr, idx, remap):
    """(n_dst, self_idx, indptr, idx) of layer k (1-based) in the numbering of its source rows."""
    n_dst = int(level_start[L - k + 1])
    nnz = int(indptr[n_dst])
    if k == 1:
        self_idx = remap[:n_dst]
        ix = np.where(idx[:nnz] >= 0, remap[np.maximum(idx[:nnz], 0)], -1).astype(np.int32)
    else:
        self_idx, ix = None, idx[:nnz]
    return n_dst, self_idx, indptr[:n_dst + 1], ix


def layer_chain(orc, X, fmt, node_vertex, level_start, indptr, idx, weights, layer=None):
    """Layers over a level-major frontier structure: layer k computes the rows of levels 0..L-k
    from those of levels 0..L-k+1 (the first from the pre-gathered feature rows).  `orc` is the
    oracle package (pre-gather, gather and the pinned layers).  The layer is GraphSAGE-mean with
    weights[k-1] = (W_self, W_neigh, bias), or `layer(k, H, self_idx, indptr, idx, relu)` -> float64
    rows (one of the other pinned layer functions).  Returns the root rows."""
    L = len(weights)
    uniq, remap = orc.pregather(node_vertex)
    H = orc.gather(X, uniq)
    for k in range(1, L + 1):
        _, self_idx, ip, ix = layer_inputs(k, L, level_start, indptr, idx, remap)
        if layer is None:
            out = orc.sage_fwd(H, fmt, self_idx, ip, ix, *weights[k - 1], relu=(k < L))
        else:
            out = layer(k, H, self_idx, ip, ix, k < L)
        H = orc.round_store(out, fmt)       # the next layer reads the rows as stored
    return out


def layer_chain_grads(orc, X, fmt, node_vertex, level_start, indptr, idx, weights, dOut):
    """Forward as layer_chain, then the backward pass from dOut = dL/d(root rows) (paper section
    5.1, steps 3-4: forward and backward per micrograph batch).  Returns
    (root rows, [(gW_self, gW_neigh, gbias) per layer])."""
    L = len(weights)
    uniq, remap = orc.pregather(node_vertex)
    H = [orc.gather(X, uniq)]
    out = None
    for k in range(1, L + 1):
        _, self_idx, ip, ix = layer_inputs(k, L, level_start, indptr, idx, remap)
        out = orc.sage_fwd(H[-1], fmt, self_idx, ip, ix, *weights[k - 1], relu=(k < L))
        H.append(orc.round_store(out, fmt))
    grads = [None] * L
    d = np.asarray(dOut, np.float64)
    for k in range(L, 0, -1):
        _, self_idx, ip, ix = layer_inputs(k, L, level_start, indptr, idx, remap)
        Ws, Wn, _b = weights[k - 1]
        relu = k < L
        gWs, gWn, gb, dH = orc.sage_bwd(H[k - 1], fmt, self_idx, ip, ix, Ws, Wn, H[k] if relu else None, relu, d,
                                        want_dH=(k > 1))
        grads[k - 1] = (gWs, gWn, gb)
        if k > 1:
            d = dH[:int(level_start[L - k + 2])]
    return out, grads


def locality(node_vertex, level_start, indptr, idx, n_seeds, owner):
    """R_micro's two counts (paper section 4, "data locality in micrographs") for the micrographs of
    a frontier structure: the micrograph of root m is every node reachable from node m through the
    structure's entries; n_total[m] = its distinct vertices, n_coloc[m] = its distinct vertices
    other than the root whose home server owner[v] is the root's.  Plain sets."""
    node_vertex = np.asarray(node_vertex)
    n_nonleaf = len(indptr) - 1
    n_total = np.zeros(n_seeds, np.int32)
    n_coloc = np.zeros(n_seeds, np.int32)
    for m in range(n_seeds):
        seen, frontier_nodes = {m}, [m]
        while frontier_nodes:
            nxt = []
            for q in frontier_nodes:
                if q >= n_nonleaf:
                    continue
                for u in idx[indptr[q]:indptr[q + 1]]:
                    u = int(u)
                    if u >= 0 and u not in seen:
                        seen.add(u)
                        nxt.append(u)
            frontier_nodes = nxt
        root = int(node_vertex[m])
        verts = {int(node_vertex[q]) for q in seen if node_vertex[q] >= 0}
        n_total[m] = len(verts)
        n_coloc[m] = sum(1 for v in verts if v != root and owner[v] == owner[root]) if root >= 0 else 0
    return n_total, n_coloc
