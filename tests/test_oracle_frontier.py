"""Pins of the layer chain and its gradients over a frontier structure (oracle/frontier.py):
central differences of L = <G, root rows> in float64, and - for the deduplicated frontiers, which
compute the same function of the weights as the slot tree - the tree chain's gradients."""
import numpy as np
import pytest

from oracle import dedup, frontier, layerwise

F64 = 3


def _graph(rng, n, max_deg, p_isolated=0.1):
    deg = rng.integers(1, max_deg + 1, size=n)
    deg[rng.random(n) < p_isolated] = 0
    off = np.zeros(n + 1, np.int64)
    off[1:] = np.cumsum(deg)
    idx = rng.integers(0, n, size=int(off[-1])).astype(np.int32)
    return off, idx


def _weights(rng, d, hid, L):
    return [(rng.standard_normal((d if k == 0 else hid, hid)) / 3, rng.standard_normal((d if k == 0 else hid, hid)) / 3,
             rng.standard_normal(hid) / 3) for k in range(L)]


@pytest.mark.parametrize("sampler", ["dedup", "layerwise"])
def test_gradients_match_central_differences(orc, sampler):
    rng = np.random.default_rng(17)
    n, d, hid, L = 60, 4, 5, 3
    off, idx = _graph(rng, n, 5)
    seeds = rng.integers(0, n, size=5).astype(np.int32)
    X = rng.standard_normal((n, d))
    W = _weights(rng, d, hid, L)
    if sampler == "dedup":
        st = dedup.sample_dedup(off, idx, seeds, [3, 3, 2], 4)
    else:
        st = layerwise.sample_layerwise(off, idx, seeds, [3, 4, 4], 4)
    G = rng.standard_normal((len(seeds), hid))
    out, grads = frontier.layer_chain_grads(orc, X, F64, *st, W, G)
    np.testing.assert_allclose(out, frontier.layer_chain(orc, X, F64, *st, W), rtol=0, atol=0)
    loss = lambda Wp: float((G * frontier.layer_chain(orc, X, F64, *st, Wp)).sum())
    eps = 1e-6
    for k in range(L):
        for part in range(3):
            A = W[k][part]
            picks = [tuple(rng.integers(0, s) for s in A.shape) for _ in range(4)]
            for at in picks:
                Wp = [list(w) for w in W]
                Wm = [list(w) for w in W]
                Wp[k][part] = A.copy()
                Wm[k][part] = A.copy()
                Wp[k][part][at] += eps
                Wm[k][part][at] -= eps
                fd = (loss([tuple(w) for w in Wp]) - loss([tuple(w) for w in Wm])) / (2 * eps)
                assert abs(fd - grads[k][part][at]) <= 1e-6 * max(1.0, abs(fd)), (k, part, at)


def test_deduplicated_chain_has_the_tree_chains_gradients(orc):
    rng = np.random.default_rng(23)
    n, d, hid, fan = 80, 5, 6, [4, 3]
    off, idx = _graph(rng, n, 4)
    seeds = rng.integers(0, n, size=7).astype(np.int32)
    B, L = len(seeds), 2
    X = rng.standard_normal((n, d))
    W = _weights(rng, d, hid, L)
    G = rng.standard_normal((B, hid))
    _, grads = frontier.layer_chain_grads(orc, X, F64, *dedup.sample_dedup(off, idx, seeds, fan, 6), W, G)
    # the slot tree, layer by layer with the pinned single-layer functions
    ids, ip = orc.sample(off, idx, seeds, fan, 6)
    uniq, remap = orc.pregather(ids)
    Xu = orc.gather(X, uniq)
    lv = orc.level_sizes(B, fan)
    n1, nnz1 = lv[0] + lv[1], lv[1] + lv[2]
    H1 = orc.sage_fwd(Xu, F64, remap[:n1], ip[:n1 + 1], remap[B:B + nnz1], *W[0], relu=True)
    slot_idx = np.where(ids[B:B + lv[1]] >= 0, B + np.arange(lv[1]), -1).astype(np.int32)
    g2 = orc.sage_bwd(H1, F64, None, ip[:B + 1], slot_idx, W[1][0], W[1][1], None, False, G)
    g1 = orc.sage_bwd(Xu, F64, remap[:n1], ip[:n1 + 1], remap[B:B + nnz1], W[0][0], W[0][1], H1, True, g2[3],
                      want_dH=False)
    for part in range(3):
        np.testing.assert_allclose(grads[1][part], g2[part], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(grads[0][part], g1[part], rtol=1e-10, atol=1e-12)


def test_locality_of_deduplicated_micrographs_is_the_slot_trees(orc):
    rng = np.random.default_rng(31)
    n, fan = 90, [4, 3, 2]
    off, idx = _graph(rng, n, 5)
    seeds = rng.integers(0, n, size=11).astype(np.int32)
    owner = rng.integers(0, 3, size=n).astype(np.int32)
    ids, _ = orc.sample(off, idx, seeds, fan, 2)
    want = orc.micrograph_locality(ids, len(seeds), fan, owner)
    got = frontier.locality(*dedup.sample_dedup(off, idx, seeds, fan, 2), len(seeds), owner)
    np.testing.assert_array_equal(got[0], want[0])
    np.testing.assert_array_equal(got[1], want[1])


def test_locality_of_layerwise_micrographs_against_one_seed_at_a_time():
    """A micrograph's draws depend on (key, root) only, so sampling each seed alone gives its vertex
    set directly; the worked ring: level sets r±1, r±2 and r, with two servers of half a ring."""
    rng = np.random.default_rng(37)
    n, bud = 70, [3, 5, 4]
    off, idx = _graph(rng, n, 6)
    seeds = rng.integers(0, n, size=9).astype(np.int32)
    seeds[4] = seeds[2]
    keys = [int(k) for k in rng.integers(0, 1000, size=9)]
    owner = rng.integers(0, 4, size=n).astype(np.int32)
    got = frontier.locality(*layerwise.sample_layerwise(off, idx, seeds, bud, keys), len(seeds), owner)
    for m, (s, k) in enumerate(zip(seeds, keys)):
        nv = layerwise.sample_layerwise(off, idx, [s], bud, k)[0]
        verts = set(int(v) for v in nv)
        assert got[0][m] == len(verts)
        assert got[1][m] == sum(1 for v in verts if v != s and owner[v] == owner[s])
    # ring of 12, root 5, budgets large enough for the full layers: {4,6}, {3,5,7} -> 5 distinct
    # vertices; servers {0..5} and {6..11}: co-located non-root vertices are 3 and 4
    ring_off = np.arange(13, dtype=np.int64) * 2
    ring_idx = np.stack([(np.arange(12) - 1) % 12, (np.arange(12) + 1) % 12], 1).ravel().astype(np.int32)
    ring_owner = (np.arange(12) >= 6).astype(np.int32)
    t, c = frontier.locality(*layerwise.sample_layerwise(ring_off, ring_idx, [5], [64, 64], 3), 1, ring_owner)
    assert (t[0], c[0]) == (5, 2)


def test_planted_partition_locality_follows_the_papers_table():
    """The trend of the paper's locality table on a graph with planted locality: S servers, every
    edge stays on its server with probability p_in.  For both samplers R_micro of one-hop micrographs
    is about p_in, it decays with depth, and it stays above R_sub = 1/S of uniformly random vertices."""
    rng = np.random.default_rng(41)
    S, per, deg, p_in = 4, 150, 6, 0.8
    n = S * per
    owner = (np.arange(n) // per).astype(np.int32)
    off = np.arange(n + 1, dtype=np.int64) * deg
    stay = rng.random((n, deg)) < p_in
    inside = owner[:, None] * per + rng.integers(0, per, size=(n, deg))
    anywhere = rng.integers(0, n, size=(n, deg))
    idx = np.where(stay, inside, anywhere).astype(np.int32).ravel()
    seeds = rng.integers(0, n, size=120).astype(np.int32)
    p_same = p_in + (1 - p_in) / S                       # a random target lands at home with 1/S
    for name, sample, shapes in (("node", dedup.sample_dedup, ([6], [4, 4], [3, 3, 3, 3])),
                                 ("layer", layerwise.sample_layerwise, ([6], [6, 8], [6, 8, 8, 8]))):
        r = []
        for fan in shapes:
            t, c = frontier.locality(*sample(off, idx, seeds, fan, 5), len(seeds), owner)
            r.append(float(c.sum()) / float((t - 1).sum()))        # co-located share of the non-root vertices
        assert abs(r[0] - p_same) < 0.06, (name, r)
        assert r[0] > r[1] > r[2] > 1.0 / S + 0.05, (name, r)


@pytest.mark.parametrize("kind", ["gcn", "gat"])
def test_other_layers_over_deduplicated_frontiers_give_the_tree_rows(orc, kind):
    """GCN-style and attention layers over the deduplicated structure (parallel edges kept) against
    the same layers over the slot tree, layer by layer with the pinned single-layer functions."""
    rng = np.random.default_rng(29)
    n, d, hid, fan, heads = 70, 5, 6, [4, 3, 2], 2
    off, idx = _graph(rng, n, 4)
    seeds = rng.integers(0, n, size=6).astype(np.int32)
    B, L = len(seeds), 3
    X = rng.standard_normal((n, d))
    W = _weights(rng, d, hid, L)
    attn = [(rng.standard_normal(hid), rng.standard_normal(hid)) for _ in range(L)]

    def layer(k, H, self_idx, ip, ix, relu):
        if kind == "gcn":
            return orc.gcn_fwd(H, F64, self_idx, ip, ix, W[k - 1][0], W[k - 1][2], 1, relu)
        return orc.gat_fwd(H, F64, self_idx, ip, ix, W[k - 1][0], attn[k - 1][0], attn[k - 1][1], W[k - 1][2], heads, relu)
    got = frontier.layer_chain(orc, X, F64, *dedup.sample_dedup(off, idx, seeds, fan, 8), W, layer=layer)
    ids, ip = orc.sample(off, idx, seeds, fan, 8)
    uniq, remap = orc.pregather(ids)
    lv = orc.level_sizes(B, fan)
    H = orc.gather(X, uniq)
    for k in range(1, L + 1):
        n_dst = sum(lv[:L - k + 1])
        nnz = int(ip[n_dst])
        if k == 1:
            self_idx, ix = remap[:n_dst], remap[B:B + nnz]
        else:
            self_idx, ix = None, np.where(ids[B:B + nnz] >= 0, B + np.arange(nnz), -1).astype(np.int32)
        H = layer(k, H, self_idx, ip[:n_dst + 1], ix, k < L)
    np.testing.assert_allclose(got, H, rtol=1e-10, atol=1e-12)
