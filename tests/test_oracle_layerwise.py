"""Pins of the layer-wise sampling oracle (section 4's layer-wise sampled micrographs): the
restricted 0/1 adjacency of scipy, the dense formulation of the layer, the importance distribution
of the draws, and degenerate graphs whose result is known without any hash."""
import numpy as np
import pytest
import scipy.sparse as sp
from scipy import stats

from oracle import layerwise

F64 = 3


def _graph(rng, n, max_deg, p_isolated=0.1):
    deg = rng.integers(1, max_deg + 1, size=n)
    deg[rng.random(n) < p_isolated] = 0
    off = np.zeros(n + 1, np.int64)
    off[1:] = np.cumsum(deg)
    idx = rng.integers(0, n, size=int(off[-1])).astype(np.int32)      # parallel edges and loops occur
    return off, idx


def _split_levels(nv, ls, ip, ix, B):
    """Cut every level into its micrographs.  Level 0 has one node each; the nodes of level h+1
    that belong to micrograph m are those its level-h nodes point at - contiguous and, because
    every node of a level was drawn from the previous level's lists, covering the level unless a
    node is pointed at by nobody (impossible: a drawn vertex is adjacent to the node it was drawn from)."""
    L = len(ls) - 2
    cuts = [list(range(B + 1))]                      # positions inside level 0
    for h in range(L):
        nxt = [0]
        for m in range(B):
            lo, hi = int(ls[h]) + cuts[h][m], int(ls[h]) + cuts[h][m + 1]
            ent = ix[ip[lo]:ip[hi]] if hi > lo else np.zeros(0, np.int32)
            nxt.append(int(ent.max()) + 1 - int(ls[h + 1]) if len(ent) else nxt[-1])
        cuts.append(nxt)
    return cuts


@pytest.mark.parametrize("budgets", [[4], [3, 5], [6, 4, 5], [2, 2, 2, 2]])
def test_structure_is_the_restricted_adjacency(budgets):
    rng = np.random.default_rng(10 + len(budgets))
    n = 70
    off, idx = _graph(rng, n, 6)
    A = sp.csr_matrix((np.ones(len(idx)), idx.copy(), off.copy()), shape=(n, n))   # scipy edits its arrays in place
    A.sum_duplicates()
    A01 = (A > 0).astype(np.int8).tocsr()
    seeds = rng.integers(0, n, size=12).astype(np.int32)
    seeds[5] = seeds[1]
    B, L = len(seeds), len(budgets)
    for key in (0, 31):
        nv, ls, ip, ix = layerwise.sample_layerwise(off, idx, seeds, budgets, key)
        assert ls[0] == 0 and ls[1] == B and ls[-1] == len(nv)
        np.testing.assert_array_equal(nv[:B], seeds)
        assert len(ip) == ls[L] + 1 and ip[0] == 0 and ip[-1] == len(ix)
        assert (np.diff(ip) >= 0).all()
        cuts = _split_levels(nv, ls, ip, ix, B)
        for h in range(L):
            assert cuts[h + 1][-1] == ls[h + 2] - ls[h + 1]        # the micrographs cover the level
            for m in range(B):
                prev = nv[ls[h] + cuts[h][m]: ls[h] + cuts[h][m + 1]].astype(np.int64)
                cur = nv[ls[h + 1] + cuts[h + 1][m]: ls[h + 1] + cuts[h + 1][m + 1]].astype(np.int64)
                assert len(cur) <= budgets[h]
                assert (np.diff(cur) > 0).all()                      # ascending and distinct
                if len(prev) == 0 or off[prev + 1].sum() == off[prev].sum():
                    assert len(cur) == 0                             # no candidate: an empty level
                    continue
                assert len(cur) >= 1
                sub = A01[prev][:, cur].tocsr()                      # scipy's restricted adjacency
                sub.sort_indices()
                base = int(ls[h + 1]) + cuts[h + 1][m]
                for q in range(len(prev)):
                    g = int(ls[h]) + cuts[h][m] + q
                    np.testing.assert_array_equal(ix[ip[g]:ip[g + 1]] - base, sub.indices[sub.indptr[q]:sub.indptr[q + 1]])
                # every node of the level is adjacent to the previous level
                assert (np.asarray(sub.sum(axis=0)).ravel() > 0).all()


def test_draws_follow_the_importance_distribution():
    """One draw per key: level 1 is uniform over the root's list WITH multiplicity, level 2 is
    proportional to the number of edges from level 1 into a vertex."""
    # vertex 0: list [1,1,1,2]; 1: [3,4]; 2: [4,4,4,5,0,0]; others empty
    lists = {0: [1, 1, 1, 2], 1: [3, 4], 2: [4, 4, 4, 5, 0, 0]}
    n = 6
    off = np.zeros(n + 1, np.int64)
    idx = []
    for v in range(n):
        idx += lists.get(v, [])
        off[v + 1] = len(idx)
    idx = np.asarray(idx, np.int32)
    n_keys = 3000
    c1 = np.zeros(n)
    c2_given = {1: np.zeros(n), 2: np.zeros(n)}
    for key in range(n_keys):
        nv, ls, ip, ix = layerwise.sample_layerwise(off, idx, [0], [1, 1], key)
        v1 = int(nv[1])
        c1[v1] += 1
        assert ls[3] - ls[2] == 1
        c2_given[v1][int(nv[2])] += 1
    assert c1[[0, 3, 4, 5]].sum() == 0
    assert stats.chisquare(c1[[1, 2]], n_keys * np.array([0.75, 0.25])).pvalue > 1e-4
    assert stats.chisquare(c2_given[1][[3, 4]], c2_given[1].sum() * np.array([0.5, 0.5])).pvalue > 1e-4
    assert stats.chisquare(c2_given[2][[4, 5, 0]], c2_given[2].sum() * np.array([3, 1, 2]) / 6).pvalue > 1e-4
    # both level-1 nodes present: candidates [3,4 | 4,4,4,5,0,0] -> 3:1, 4:4, 5:1, 0:2 of 8
    c = np.zeros(n)
    n_both = 0
    for key in range(n_keys):
        nv, ls, ip, ix = layerwise.sample_layerwise(off, idx, [0], [8, 1], key)
        if ls[2] - ls[1] == 2:
            n_both += 1
            c[int(nv[ls[2]])] += 1
    assert n_both > n_keys // 2
    assert stats.chisquare(c[[3, 4, 5, 0]], n_both * np.array([1, 4, 1, 2]) / 8).pvalue > 1e-4


def test_large_budget_on_a_ring_gives_the_full_neighbourhood_layers():
    n = 12
    off = np.arange(n + 1, dtype=np.int64) * 2
    idx = np.stack([(np.arange(n) - 1) % n, (np.arange(n) + 1) % n], 1).ravel().astype(np.int32)
    nv, ls, ip, ix = layerwise.sample_layerwise(off, idx, [5, 0], [64, 64, 64], 3)
    # layer h of root r on a ring: r-h, r-h+2, ..., r+h  (64 draws miss one of <= 8 candidates with p < 1e-3)
    want = lambda r, h: np.unique([(r + t) % n for t in range(-h, h + 1, 2)])
    np.testing.assert_array_equal(nv[ls[1]:ls[2]], np.concatenate([want(5, 1), want(0, 1)]))
    np.testing.assert_array_equal(nv[ls[2]:ls[3]], np.concatenate([want(5, 2), want(0, 2)]))
    np.testing.assert_array_equal(nv[ls[3]:ls[4]], np.concatenate([want(5, 3), want(0, 3)]))
    # every ring vertex of a level has its two neighbours in the next level
    assert (np.diff(ip) == 2).all()


def test_budget_one_is_a_walk_and_dead_ends_empty_the_levels():
    # 0 -> 1 -> 2 -> (nothing); 3 isolated
    off = np.array([0, 1, 2, 2, 2], np.int64)
    idx = np.array([1, 2], np.int32)
    nv, ls, ip, ix = layerwise.sample_layerwise(off, idx, [0, 3, 1], [1, 1, 1], 8)
    np.testing.assert_array_equal(ls, [0, 3, 5, 6, 6])
    np.testing.assert_array_equal(nv, [0, 3, 1, 1, 2, 2])
    # entries: level 0 nodes (0 -> node 3, 3 -> none, 1 -> node 4), level 1 nodes (1 -> node 5, 2 -> none), level 2 (2 -> none)
    np.testing.assert_array_equal(ip, [0, 1, 1, 2, 3, 3, 3])
    np.testing.assert_array_equal(ix, [3, 4, 5])


def test_keys_per_micrograph_and_repeated_roots():
    rng = np.random.default_rng(3)
    off, idx = _graph(rng, 50, 5, 0.0)
    a = layerwise.sample_layerwise(off, idx, [7, 7], [3, 3], [5, 6])
    b = layerwise.sample_layerwise(off, idx, [7], [3, 3], 5)
    c = layerwise.sample_layerwise(off, idx, [7], [3, 3], 6)
    np.testing.assert_array_equal(a[0][a[1][1]:a[1][2]], np.concatenate([b[0][1:b[1][2]], c[0][1:c[1][2]]]))
    same = layerwise.sample_layerwise(off, idx, [7, 7], [3, 3], 5)
    n1 = (same[1][2] - same[1][1]) // 2
    np.testing.assert_array_equal(same[0][2:2 + n1], same[0][2 + n1:2 + 2 * n1])


def test_layer_chain_is_the_dense_formula(orc):
    """Two layers for one root against dense matrices: rows of the restricted 0/1 adjacency,
    normalised by their sums, times the next level's rows."""
    rng = np.random.default_rng(9)
    n, d, hid = 40, 5, 4
    off, idx = _graph(rng, n, 5, 0.0)
    A = np.zeros((n, n))
    for u in range(n):
        A[u, idx[off[u]:off[u + 1]]] = 1.0
    X = rng.standard_normal((n, d))
    Ws = [(rng.standard_normal((d, hid)), rng.standard_normal((d, hid)), rng.standard_normal(hid)),
          (rng.standard_normal((hid, hid)), rng.standard_normal((hid, hid)), rng.standard_normal(hid))]
    for root in (0, 17):
        nv, ls, ip, ix = layerwise.sample_layerwise(off, idx, [root], [4, 6], 21)
        S1, S2 = nv[ls[1]:ls[2]].astype(int), nv[ls[2]:ls[3]].astype(int)

        def mean_of(rows, cols, Hc):
            sub = A[np.ix_(rows, cols)]
            cnt = sub.sum(1, keepdims=True)
            return np.where(cnt > 0, sub @ Hc / np.maximum(cnt, 1), 0.0)
        # layer 1 on levels 0 and 1, layer 2 on the root
        h_root = np.maximum(X[[root]] @ Ws[0][0] + mean_of([root], S1, X[S1]) @ Ws[0][1] + Ws[0][2], 0)
        h_S1 = np.maximum(X[S1] @ Ws[0][0] + mean_of(S1, S2, X[S2]) @ Ws[0][1] + Ws[0][2], 0)
        out = h_root @ Ws[1][0] + mean_of([root], S1, h_S1) @ Ws[1][1] + Ws[1][2]
        got = layerwise.layer_chain(orc, X, F64, nv, ls, ip, ix, Ws)
        np.testing.assert_allclose(got, out, rtol=1e-11, atol=1e-12)
