"""Oracle for per-micrograph deduplicated frontiers.  TEST INFRASTRUCTURE ONLY.

A micrograph is defined as the set of vertices its k-hop sampling reaches (paper section 4,
"micrograph definition"; the section counts DISTINCT vertices per micrograph).  The children a
vertex draws depend only on (key, root, vertex, hop, j), so equal vertices at one level of one
micrograph carry identical subtrees in the slot tree; keeping each (level, vertex) pair once gives
the same rows for the root with fewer rows below it.  Plain definition, numpy only:

  nodes of micrograph m at level h  = ascending distinct valid vertices of the slot tree's level h
  entries of a level-h node v       = its f_{h+1} sampled children in draw order j = 0..f-1, as
                                      positions in the next level's node list (-1: v has no
                                      neighbours), parallel edges kept
  global numbering                  = level-major: level 0 of every micrograph (seed order), then
                                      level 1 of every micrograph, ...
"""
from __future__ import annotations

import numpy as np

from . import hash64, level_sizes   # noqa: F401  (hash64 is the pinned hash)


def sample_dedup(offsets, indices, seeds, fanouts, key=0):
    """Returns (node_vertex [n_nodes], level_start [L+2], indptr [n_nonleaf+1], idx [nnz])."""
    offsets = np.asarray(offsets)
    indices = np.asarray(indices)
    B, L = len(seeds), len(fanouts)
    per_level = []            # per level: list over micrographs of sorted distinct vertex arrays
    entries = []              # per level h < L: list over micrographs of [n_nodes_h(m), f] child vertices (-1 none)
    cur = [np.array([int(s)], np.int64) for s in seeds]
    per_level.append(cur)
    for h in range(1, L + 1):
        f = int(fanouts[h - 1])
        nxt, ent = [], []
        for m in range(B):
            root = int(seeds[m])
            ch = np.full((len(cur[m]), f), -1, np.int64)
            for q, v in enumerate(cur[m]):
                v = int(v)
                o0, o1 = int(offsets[v]), int(offsets[v + 1])
                deg = o1 - o0
                if deg <= 0:
                    continue
                for j in range(f):
                    ch[q, j] = int(indices[o0 + hash64(key, root, v, h, j) % deg])
            ent.append(ch)
            valid = ch[ch >= 0]
            nxt.append(np.unique(valid))
        entries.append(ent)
        per_level.append(nxt)
        cur = nxt
    counts = [[len(a) for a in lvl] for lvl in per_level]
    level_start = np.zeros(L + 2, np.int64)
    for h in range(L + 1):
        level_start[h + 1] = level_start[h] + sum(counts[h])
    node_vertex = np.concatenate([np.concatenate(lvl) if len(lvl) else np.zeros(0, np.int64) for lvl in per_level])
    indptr, idx = [0], []
    for h in range(L):
        mg_off_next = np.concatenate([[0], np.cumsum(counts[h + 1])])
        for m in range(B):
            ch = entries[h][m]
            for q in range(ch.shape[0]):
                row = ch[q]
                pos = np.where(row >= 0, level_start[h + 1] + mg_off_next[m] +
                               np.searchsorted(per_level[h + 1][m], np.maximum(row, 0)), -1)
                idx.extend(int(p) for p in pos)
                indptr.append(len(idx))
    return (node_vertex.astype(np.int32), level_start, np.asarray(indptr, np.int32), np.asarray(idx, np.int32))


def expand_to_tree(node_vertex, level_start, indptr, idx, n_seeds, fanouts):
    """The slot tree the deduplicated structure stands for (level-major ids, -1 for invalid slots):
    walk every root's entries hop by hop."""
    L = len(fanouts)
    lv = level_sizes(n_seeds, fanouts)
    ids = np.full(sum(lv), -1, np.int32)
    # node index held by every slot of the previous level (-1 invalid)
    prev_nodes = np.arange(n_seeds, dtype=np.int64)
    ids[:n_seeds] = node_vertex[:n_seeds]
    base = n_seeds
    for h in range(1, L + 1):
        f = int(fanouts[h - 1])
        cur_nodes = np.full(len(prev_nodes) * f, -1, np.int64)
        for q, nd in enumerate(prev_nodes):
            if nd < 0:
                continue
            seg = idx[indptr[nd]:indptr[nd + 1]]
            assert len(seg) == f
            cur_nodes[q * f:(q + 1) * f] = seg
        ids[base:base + len(cur_nodes)] = np.where(cur_nodes >= 0, node_vertex[np.maximum(cur_nodes, 0)], -1)
        base += len(cur_nodes)
        prev_nodes = cur_nodes
    return ids
