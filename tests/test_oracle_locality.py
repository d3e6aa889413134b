"""Pins for the oracle's locality statistics: the paper's two worked micrographs,
closed forms for a random partition, and brute force with python sets."""
import numpy as np

from test_oracle_sample import _paper_counts, csr_from_lists, levels


def test_paper_example_micrographs_6_and_3(orc):
    # same invented edges as in the sampling test; homes: server 0 = {4,5,6,7}, server 1 = {0,1,2,3}
    rows = [[1], [0], [1], [2, 4], [5], [1], [5, 7], [6]]
    owner = np.array([1, 1, 1, 1, 0, 0, 0, 0], np.int32)
    off, idx = csr_from_lists(rows)
    key = next(k for k in range(64)
               if all(len({orc.hash64(k, r, r, 1, j) % 2 for j in range(2)}) == 2 for r in (6, 3)))
    ids, _ = orc.sample(off, idx, np.array([6, 3], np.int32), [2, 2], key=key)
    n_total, n_coloc = orc.micrograph_locality(ids, 2, [2, 2], owner)
    paper = _paper_counts()          # {6: (4 distinct, 3 local incl. root), 3: (5, 3)}
    assert n_total.tolist() == [paper[6][0], paper[3][0]]
    # the example counts the root as local: colocated non-root + 1
    assert (n_coloc + 1).tolist() == [paper[6][1], paper[3][1]]
    # 75 % and 60 % as stated
    assert (n_coloc[0] + 1) / n_total[0] == 0.75 and (n_coloc[1] + 1) / n_total[1] == 0.60


def test_brute_force_with_sets(orc):
    rng = np.random.default_rng(4)
    N = 300
    rows = [rng.integers(0, N, size=int(rng.integers(0, 7))).tolist() for _ in range(N)]
    off, idx = csr_from_lists(rows)
    owner = rng.integers(0, 4, size=N).astype(np.int32)
    seeds = rng.integers(0, N, size=25).astype(np.int32)
    fan = [3, 2, 2]
    ids, _ = orc.sample(off, idx, seeds, fan, key=9)
    n_total, n_coloc = orc.micrograph_locality(ids, 25, fan, owner)
    lv = levels(orc, ids, 25, fan)
    P = [1, 3, 6, 12]
    for m in range(25):
        verts = set()
        for h in range(4):
            verts |= {int(v) for v in lv[h][m * P[h]:(m + 1) * P[h]] if v >= 0}
        root = int(seeds[m])
        assert n_total[m] == len(verts)
        assert n_coloc[m] == sum(1 for v in verts if v != root and owner[v] == owner[root])
    # a root with no neighbours is alone in its micrograph
    off2, idx2 = csr_from_lists([[], [0]])
    ids2, _ = orc.sample(off2, idx2, np.array([0], np.int32), [2], key=0)
    t, c = orc.micrograph_locality(ids2, 1, [2], np.array([0, 0], np.int32))
    assert t.tolist() == [1] and c.tolist() == [0]


def test_random_partition_closed_form(orc):
    # with homes drawn uniformly over S servers, a non-root vertex is co-located with
    # probability 1/S: R_micro -> (1/S)(1 - 1/N_total); the paper's R_sub column is 1/S
    rng = np.random.default_rng(8)
    N = 20000
    rows = [rng.integers(0, N, size=12).tolist() for _ in range(N)]
    off, idx = csr_from_lists(rows)
    seeds = rng.integers(0, N, size=400).astype(np.int32)
    ids, _ = orc.sample(off, idx, seeds, [5, 5], key=2)
    for S in (2, 4, 8, 16):
        owner = rng.integers(0, S, size=N).astype(np.int32)
        n_total, n_coloc = orc.micrograph_locality(ids, 400, [5, 5], owner)
        frac = n_coloc.sum() / (n_total.sum() - 400)          # over non-root vertices
        assert abs(frac - 1 / S) < 4 * np.sqrt((1 / S) * (1 - 1 / S) / (n_total.sum() - 400))


def test_split_by_owner(orc):
    rng = np.random.default_rng(1)
    owner = rng.integers(0, 3, size=1000).astype(np.int32)
    uniq = np.unique(rng.integers(0, 1000, size=400)).astype(np.int32)
    for server in range(3):
        remote = orc.split_by_owner(uniq, owner, server)
        want = [int(v) for v in uniq if owner[v] != server]
        assert remote.tolist() == want
    assert len(orc.split_by_owner(np.array([], np.int32), owner, 0)) == 0
    # everything local / everything remote
    assert len(orc.split_by_owner(uniq, np.zeros(1000, np.int32), 0)) == 0
    assert orc.split_by_owner(uniq, np.zeros(1000, np.int32), 1).tolist() == uniq.tolist()
