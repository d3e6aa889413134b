"""Pins for the oracle's micrograph sampler: closed-form graphs, brute-force
path walking on tiny graphs, invariants, and a hand-built 8-vertex example whose
vertex counts are the ones the paper states for its micrographs 6 and 3."""
import os
import re

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def csr_from_lists(rows, dtype=np.int32):
    off = np.zeros(len(rows) + 1, dtype)
    for i, r in enumerate(rows):
        off[i + 1] = off[i] + len(r)
    idx = np.array([x for r in rows for x in r], np.int32)
    return off, idx


def levels(orc, ids, B, fanouts):
    lv = orc.level_sizes(B, fanouts)
    out, p = [], 0
    for n in lv:
        out.append(ids[p:p + n])
        p += n
    assert p == len(ids)
    return out


def test_slots_per_seed_and_fanout_order(orc):
    assert orc.slots_per_seed([5, 5]) == 31
    assert orc.slots_per_seed([10, 10]) == 111
    # fanout[0] applies at the root: 1 + 15 + 150 + 750
    assert orc.slots_per_seed([15, 10, 5]) == 916
    assert orc.slots_per_seed([10, 10, 10]) == 1111
    assert orc.slots_per_seed([25, 10]) == 276
    assert orc.slots_per_seed([3, 0]) == -1
    assert orc.slots_per_seed([]) == -1


def test_directed_ring_closed_form(orc):
    # nbr(v) = {v+1 mod N}: every slot of level h of seed s holds s+h.
    N = 11
    off, idx = csr_from_lists([[(v + 1) % N] for v in range(N)])
    seeds = np.array([0, 9, 10, 4], np.int32)
    fan = [3, 2, 2]
    ids, indptr = orc.sample(off, idx, seeds, fan, key=7)
    P = 1
    for h, lvl in enumerate(levels(orc, ids, len(seeds), fan)):
        expect = np.repeat((seeds + h) % N, P)
        np.testing.assert_array_equal(lvl, expect)
        P *= fan[h] if h < len(fan) else 1
    uniq, _ = orc.pregather(ids)
    assert set(uniq.tolist()) == {(s + h) % N for s in seeds.tolist() for h in range(4)}


def test_complete_graph_identity_rows_gives_hash_mod_n(orc):
    # row v = [0, 1, ..., N-1]: the sampled child IS hash64 mod N, so this checks
    # which (root, vertex, hop, draw) each slot feeds to the hash and where the
    # result lands in the level-major array.
    N = 13
    off, idx = csr_from_lists([list(range(N)) for _ in range(N)])
    seeds = np.array([3, 12, 0], np.int32)
    fan = [4, 3]
    key = 0xABCDEF
    ids, _ = orc.sample(off, idx, seeds, fan, key=key)
    B = len(seeds)
    l0, l1, l2 = levels(orc, ids, B, fan)
    np.testing.assert_array_equal(l0, seeds)
    for m in range(B):
        for j in range(4):
            c = orc.hash64(key, int(seeds[m]), int(seeds[m]), 1, j) % N
            assert l1[m * 4 + j] == c
            for j2 in range(3):
                g = orc.hash64(key, int(seeds[m]), int(c), 2, j2) % N
                assert l2[(m * 4 + j) * 3 + j2] == g


def test_modulo_is_exact_u64_remainder_not_multiply_high(orc):
    # Degree 3 row holding [100, 101, 102]; x % 3 must be the true remainder of
    # the full 64-bit value (a multiply-high range reduction would differ).
    rows = [[0]] * 103
    rows[7] = [100, 101, 102]
    off, idx = csr_from_lists(rows)
    ids, _ = orc.sample(off, idx, np.array([7], np.int32), [16], key=5)
    exp = [100 + orc.hash64(5, 7, 7, 1, j) % 3 for j in range(16)]
    mulhi = [100 + ((orc.hash64(5, 7, 7, 1, j) * 3) >> 64) for j in range(16)]
    assert ids[1:].tolist() == exp
    assert exp != mulhi


def test_zero_degree_and_invalid_propagation(orc):
    # 0 -> [1, 2]; 1 -> []; 2 -> [0]
    off, idx = csr_from_lists([[1, 2], [], [0]])
    seeds = np.array([1, 0], np.int32)
    fan = [2, 2]
    ids, indptr = orc.sample(off, idx, seeds, fan, key=0)
    l0, l1, l2 = levels(orc, ids, 2, fan)
    assert l1[:2].tolist() == [-1, -1]           # seed 1 has no neighbours
    assert l2[:4].tolist() == [-1, -1, -1, -1]   # invalid parents stay invalid
    for j in range(2):
        c = l1[2 + j]
        assert c in (1, 2)
        kids = l2[(2 + j) * 2:(2 + j) * 2 + 2].tolist()
        assert kids == ([-1, -1] if c == 1 else [0, 0])


def _walk(orc, rows, key, root, fan):
    """Independent path-walking enumeration: {path tuple -> vertex}."""
    out = {(): root}

    def rec(path, v, h):
        if h > len(fan):
            return
        for j in range(fan[h - 1]):
            if v < 0 or len(rows[v]) == 0:
                c = -1
            else:
                c = rows[v][orc.hash64(key, root, v, h, j) % len(rows[v])]
            out[path + (j,)] = c
            rec(path + (j,), c, h + 1)

    rec((), root, 1)
    return out


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_brute_force_path_walk_on_tiny_graphs(orc, seed):
    rng = np.random.default_rng(seed)
    N = int(rng.integers(3, 17))
    rows = [rng.integers(0, N, size=int(rng.integers(0, 5))).tolist() for _ in range(N)]
    fan = [int(x) for x in rng.integers(1, 4, size=int(rng.integers(1, 4)))]
    B = int(rng.integers(1, 6))
    seeds = rng.integers(0, N, size=B).astype(np.int32)
    key = int(rng.integers(0, 2 ** 62))
    for dt in (np.int32, np.int64):
        off, idx = csr_from_lists(rows, dt)
        ids, indptr = orc.sample(off, idx, seeds, fan, key=key)
        lv = levels(orc, ids, B, fan)
        for m in range(B):
            paths = _walk(orc, rows, key, int(seeds[m]), fan)
            for path, v in paths.items():
                h = len(path)
                Ph = int(np.prod(fan[:h])) if h else 1
                p = 0
                for d, j in enumerate(path):      # mixed-radix path index
                    p = p * fan[d] + j
                assert lv[h][m * Ph + p] == v, (m, path)
            assert len(paths) == orc.slots_per_seed(fan)
        # indptr: children of non-leaf slot r are ids[B+indptr[r] : B+indptr[r+1]]
        n_nonleaf = len(ids) - len(lv[-1])
        assert len(indptr) == n_nonleaf + 1 and indptr[0] == 0
        assert indptr[-1] == len(ids) - B
        r = 0
        for h in range(len(fan)):
            for q in range(len(lv[h])):
                seg = ids[B + indptr[r]:B + indptr[r + 1]]
                np.testing.assert_array_equal(seg, lv[h + 1][q * fan[h]:(q + 1) * fan[h]])
                r += 1


def test_invariants_on_random_graph(orc):
    rng = np.random.default_rng(42)
    N = 500
    rows = [rng.integers(0, N, size=int(rng.integers(0, 12))).tolist() for _ in range(N)]
    off, idx = csr_from_lists(rows)
    seeds = rng.integers(0, N, size=40).astype(np.int32)
    fan = [4, 3, 2]
    ids, indptr = orc.sample(off, idx, seeds, fan, key=11)
    lv = levels(orc, ids, 40, fan)
    # (i) every valid child is a true CSR neighbour of its parent
    for h in range(3):
        par = np.repeat(lv[h], fan[h])
        ch = lv[h + 1]
        for p, c in zip(par.tolist(), ch.tolist()):
            if c >= 0:
                assert c in rows[p]
            else:
                assert p < 0 or len(rows[p]) == 0
    # (iv) equal vertices at one level of one micrograph have identical children
    P1, P2 = 4, 12
    for m in range(40):
        l1 = lv[1][m * P1:(m + 1) * P1]
        seen = {}
        for p, v in enumerate(l1.tolist()):
            kids = lv[2][(m * P1 + p) * 3:(m * P1 + p + 1) * 3].tolist()
            assert seen.setdefault(v, kids) == kids
    # (v) permuting the seeds permutes micrographs and leaves the union unchanged
    perm = rng.permutation(40)
    ids_p, _ = orc.sample(off, idx, seeds[perm], fan, key=11)
    lvp = levels(orc, ids_p, 40, fan)
    Ps = [1, 4, 12, 24]
    for h in range(4):
        a = lv[h].reshape(40, Ps[h])[perm]
        np.testing.assert_array_equal(a, lvp[h].reshape(40, Ps[h]))
    assert set(ids.tolist()) == set(ids_p.tolist())
    # changing the key changes the draws
    ids_k, _ = orc.sample(off, idx, seeds, fan, key=12)
    assert (ids_k != ids).any()
    # duplicate seeds give identical micrographs
    ids_d, _ = orc.sample(off, idx, np.array([seeds[0], seeds[0]], np.int32), fan, key=11)
    lvd = levels(orc, ids_d, 2, fan)
    for h in range(4):
        np.testing.assert_array_equal(lvd[h][:Ps[h]], lvd[h][Ps[h]:])


def test_draws_are_uniform_over_the_row(orc):
    # chi-square of the chosen position over many roots for one degree-7 vertex
    deg = 7
    rows = [[0]] * 4000
    rows[5] = list(range(100, 100 + deg))
    rows = rows + [[0]] * 200
    N = len(rows)
    # roots whose only neighbour is vertex 5, so hop 2 always draws from row 5
    for r in range(1000, 4000):
        rows[r] = [5]
    off, idx = csr_from_lists(rows)
    seeds = np.arange(1000, 4000, dtype=np.int32)
    ids, _ = orc.sample(off, idx, seeds, [1, 8], key=3)
    leaf = ids[2 * len(seeds):]
    counts = np.bincount(leaf - 100, minlength=deg)
    n = counts.sum()
    assert n == 8 * 3000
    chi2 = ((counts - n / deg) ** 2 / (n / deg)).sum()
    assert chi2 < 30.0       # 6 d.o.f.: P(chi2 > 30) < 5e-5


def _paper_counts():
    out = {}
    for line in open(os.path.join(HERE, "golden", "micrograph_locality_example.txt")):
        m = re.match(r"micrograph (\d+): distinct (\d+) local (\d+)", line)
        if m:
            out[int(m.group(1))] = (int(m.group(2)), int(m.group(3)))
    return out


def test_eight_vertex_example_matches_paper_counts(orc):
    # Edges invented (the paper's figure is not available) so that the counts the
    # paper states come out whenever both of a root's neighbours are drawn:
    #   6 -> {5,7}, 5 -> {1}, 7 -> {6};   3 -> {2,4}, 2 -> {1}, 4 -> {5}
    rows = [[1], [0], [1], [2, 4], [5], [1], [5, 7], [6]]
    home = {v: (0 if v >= 4 else 1) for v in range(8)}
    off, idx = csr_from_lists(rows)
    paper = _paper_counts()
    assert paper == {6: (4, 3), 3: (5, 3)}
    # smallest key for which both roots draw both of their neighbours
    key = next(k for k in range(64)
               if all(len({orc.hash64(k, r, r, 1, j) % 2 for j in range(2)}) == 2 for r in (6, 3)))
    ids, _ = orc.sample(off, idx, np.array([6, 3], np.int32), [2, 2], key=key)
    lv = levels(orc, ids, 2, [2, 2])
    for m, root in enumerate((6, 3)):
        verts = {int(lv[0][m])} | set(lv[1][2 * m:2 * m + 2].tolist()) | set(lv[2][4 * m:4 * m + 4].tolist())
        assert len(verts) == paper[root][0]
        assert sum(home[v] == home[root] for v in verts) == paper[root][1]
    assert set(lv[1][0:2].tolist()) == {5, 7} and set(lv[1][2:4].tolist()) == {2, 4}
