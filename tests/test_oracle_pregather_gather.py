"""Pins for the oracle's pre-gather (merged duplicate-free ID set + remap) and
row gather."""
import math
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def test_paper_worked_example_three_fetches_become_two(orc):
    steps, expect = [], {}
    for line in open(os.path.join(HERE, "golden", "pregather_worked_example.txt")):
        line = line.strip()
        if line.startswith("step"):
            steps.append([int(x) for x in line.split(":")[1].split()])
        elif line.startswith(("without", "with")):
            k, v = line.split(":")
            expect[k] = int(v)
    assert steps == [[1], [1, 0]]
    per_step = sum(len(orc.pregather(np.array(s, np.int32))[0]) for s in steps)
    merged_ids = np.array([x for s in steps for x in s], np.int32)
    uniq, remap = orc.pregather(merged_ids)
    assert per_step == expect["without"] == 3
    assert len(uniq) == expect["with"] == 2
    assert uniq.tolist() == [0, 1] and remap.tolist() == [1, 1, 0]


def test_set_union_ascending_and_remap_roundtrip(orc):
    rng = np.random.default_rng(0)
    for n, hi in [(1, 5), (17, 4), (1000, 300), (5000, 2 ** 31 - 1), (4096, 64)]:
        ids = rng.integers(0, hi, size=n).astype(np.int32)
        ids[rng.random(n) < 0.2] = -1
        uniq, remap = orc.pregather(ids)
        valid = ids >= 0
        want = set(ids[valid].tolist())              # hash set: a different algorithm
        assert set(uniq.tolist()) == want and len(uniq) == len(want)
        assert (np.diff(uniq.astype(np.int64)) > 0).all()
        assert (remap[~valid] == -1).all() and (remap[valid] >= 0).all()
        np.testing.assert_array_equal(uniq[remap[valid]], ids[valid])
        assert len(uniq) <= min(valid.sum(), hi)


def test_empty_and_all_invalid(orc):
    uniq, remap = orc.pregather(np.array([], np.int32))
    assert len(uniq) == 0 and len(remap) == 0
    uniq, remap = orc.pregather(np.array([-1, -1, -1], np.int32))
    assert len(uniq) == 0 and remap.tolist() == [-1, -1, -1]
    uniq, remap = orc.pregather(np.array([2 ** 31 - 1, 0, 2 ** 31 - 1], np.int32))
    assert uniq.tolist() == [0, 2 ** 31 - 1] and remap.tolist() == [1, 0, 1]


def test_group_is_union_of_batches(orc):
    rng = np.random.default_rng(3)
    batches = [rng.integers(0, 200, size=150).astype(np.int32) for _ in range(4)]
    u_all, _ = orc.pregather(np.concatenate(batches))
    per = [set(orc.pregather(b)[0].tolist()) for b in batches]
    assert set(u_all.tolist()) == set().union(*per)
    assert len(u_all) <= sum(len(p) for p in per)


def test_expected_unique_count_for_uniform_targets(orc):
    # T draws uniform over N vertices: E[U] = N (1 - (1 - 1/N)^T)
    rng = np.random.default_rng(5)
    N, T = 20000, 1984
    us = [len(orc.pregather(rng.integers(0, N, size=T).astype(np.int32))[0]) for _ in range(20)]
    mean = N * (1 - (1 - 1 / N) ** T)
    assert abs(np.mean(us) - mean) < 6.0       # sd of one draw ~ 9.5, of the mean ~ 2.1
    assert abs(mean - N * (1 - math.exp(-T / N))) < 1.0


def test_gather_rows_byte_for_byte(orc):
    rng = np.random.default_rng(1)
    for dt, d in [(np.float32, 32), (np.float32, 100), (np.uint16, 128), (np.uint8, 7)]:
        X = rng.integers(0, 256, size=(50, d * np.dtype(dt).itemsize), dtype=np.uint8).view(dt)
        uniq = np.unique(rng.integers(0, 50, size=30)).astype(np.int32)
        Xu = orc.gather(X, uniq)
        assert Xu.dtype == X.dtype and Xu.shape == (len(uniq), d)
        for i, u in enumerate(uniq.tolist()):
            assert Xu[i].tobytes() == X[u].tobytes()
        # identity index list reproduces the table
        assert orc.gather(X, np.arange(50, dtype=np.int32)).tobytes() == X.tobytes()
    # strided source rows (leading dimension larger than the row)
    big = rng.standard_normal((20, 48)).astype(np.float32)
    view = big[:, :40]
    Xu = orc.gather(view, np.array([3, 19], np.int32))
    np.testing.assert_array_equal(Xu, view[[3, 19]])
    assert len(orc.gather(big, np.array([], np.int32))) == 0
