"""Pins of the deduplicated-frontier oracle: expanding it hop by hop reproduces the pinned slot-tree
sampler exactly; its node lists are the ascending distinct vertices of the tree's levels; a layer
chain over it gives the tree's root rows."""
import numpy as np
import pytest

from oracle import dedup

F64 = 3


def _graph(rng, n, max_deg, p_isolated=0.1):
    deg = rng.integers(1, max_deg + 1, size=n)
    deg[rng.random(n) < p_isolated] = 0
    off = np.zeros(n + 1, np.int64)
    off[1:] = np.cumsum(deg)
    idx = rng.integers(0, n, size=int(off[-1])).astype(np.int32)
    return off, idx


@pytest.mark.parametrize("fanouts", [[4], [3, 2], [5, 4, 3], [2, 2, 2, 2]])
def test_expansion_reproduces_the_slot_tree(orc, fanouts):
    rng = np.random.default_rng(len(fanouts))
    off, idx = _graph(rng, 60, 5)
    seeds = rng.integers(0, 60, size=9).astype(np.int32)
    seeds[3] = seeds[0]                       # the same root twice: two separate micrographs
    for key in (0, 77):
        nv, ls, ip, ix = dedup.sample_dedup(off, idx, seeds, fanouts, key)
        tree_ids, _ = orc.sample(off, idx, seeds, fanouts, key)
        np.testing.assert_array_equal(dedup.expand_to_tree(nv, ls, ip, ix, len(seeds), fanouts), tree_ids)
        # node lists: per micrograph and level the ascending distinct valid vertices of the tree
        lv = orc.level_sizes(len(seeds), fanouts)
        B = len(seeds)
        pos = int(ls[0])
        for h in range(len(fanouts) + 1):
            base, P = sum(lv[:h]), lv[h] // B
            assert pos == ls[h]
            for m in range(B):
                seg = tree_ids[base + m * P: base + (m + 1) * P]
                want = np.unique(seg[seg >= 0])
                np.testing.assert_array_equal(nv[pos:pos + len(want)], want)
                pos += len(want)
        assert pos == ls[-1] == len(nv)
        assert len(ip) == ls[len(fanouts)] + 1 and ip[-1] == len(ix)
        # fewer rows than slots as soon as a draw repeats
        assert len(nv) <= len(tree_ids)


def test_layers_over_the_deduplicated_structure_give_the_tree_rows(orc):
    rng = np.random.default_rng(5)
    off, idx = _graph(rng, 80, 4)
    seeds = rng.integers(0, 80, size=6).astype(np.int32)
    fan, d, hid = [4, 3, 3], 5, 6
    X = rng.standard_normal((80, d))
    Ws = [(rng.standard_normal((d if k == 0 else hid, hid)), rng.standard_normal((d if k == 0 else hid, hid)),
           rng.standard_normal(hid)) for k in range(3)]
    B, L = len(seeds), 3
    # the tree chain (the pinned whole-batch oracle)
    ids, ip = orc.sample(off, idx, seeds, fan, 9)
    uniq, remap = orc.pregather(ids)
    Xu = orc.gather(X, uniq)
    tree_out = orc.forward(Xu, F64, ids, ip, remap, B, fan, Ws)[-1][0]
    # the same layers over the deduplicated nodes
    nv, ls, dip, dix = dedup.sample_dedup(off, idx, seeds, fan, 9)
    u2, r2 = orc.pregather(nv)
    np.testing.assert_array_equal(u2, uniq)                 # the same vertex set is fetched
    H = orc.gather(X, u2)
    for k in range(1, L + 1):
        n_dst = int(ls[L - k + 1])
        nnz = int(dip[n_dst])
        if k == 1:
            self_idx = r2[:n_dst]
            ix = np.where(dix[:nnz] >= 0, r2[np.maximum(dix[:nnz], 0)], -1).astype(np.int32)
        else:
            self_idx, ix = None, dix[:nnz]
        H = orc.sage_fwd(H, F64, self_idx, dip[:n_dst + 1], ix, *Ws[k - 1], relu=(k < L))
    np.testing.assert_allclose(H, tree_out, rtol=1e-11, atol=1e-12)
