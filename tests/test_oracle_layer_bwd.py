"""Pins for the oracle's backward of the other layer kinds (GraphSAGE with sum / max aggregator,
GCN-style, attention): central finite differences of the oracle's forward functions in float64 (which
are pinned on their own against dense formulas), dense-matrix closed forms written with numpy, and
special cases that reduce to one another."""
import numpy as np
import pytest

F64 = 3


def rand_csr(rng, n_dst, n_src, max_len, p_invalid=0.15):
    lens = rng.integers(0, max_len + 1, size=n_dst)
    indptr = np.zeros(n_dst + 1, np.int32)
    indptr[1:] = np.cumsum(lens)
    idx = rng.integers(0, n_src, size=int(indptr[-1])).astype(np.int32)
    idx[rng.random(len(idx)) < p_invalid] = -1
    return indptr, idx


def fd_grad(loss, arrs, pos, eps=1e-6):
    """Central differences of loss(*arrs) with respect to arrs[pos]."""
    g = np.zeros_like(arrs[pos])
    for i in np.ndindex(arrs[pos].shape):
        a = [x.copy() for x in arrs]
        a[pos][i] += eps
        fh = loss(*a)
        a[pos][i] -= 2 * eps
        fl = loss(*a)
        g[i] = (fh - fl) / (2 * eps)
    return g


def _case(seed, n_src=9, n_dst=6, d_in=4, d_out=6):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((n_src, d_in))
    indptr, idx = rand_csr(rng, n_dst, n_src, 4)
    self_idx = rng.integers(0, n_src, size=n_dst).astype(np.int32)
    self_idx[1] = -1
    G = rng.standard_normal((n_dst, d_out))
    return rng, H, indptr, idx, self_idx, G


@pytest.mark.parametrize("agg", [0, 1, 2])
@pytest.mark.parametrize("relu", [False, True])
def test_sage_aggregators_match_finite_differences(orc, agg, relu):
    rng, H, indptr, idx, self_idx, G = _case(10 + agg)
    d_in, d_out = H.shape[1], G.shape[1]
    Ws, Wn, b = rng.standard_normal((d_in, d_out)), rng.standard_normal((d_in, d_out)), rng.standard_normal(d_out)
    fwd = lambda H_, Ws_, Wn_, b_: orc.sage_agg_fwd(H_, F64, self_idx, indptr, idx, Ws_, Wn_, b_, agg, relu)
    loss = lambda *a: float((fwd(*a) * G).sum())
    out = fwd(H, Ws, Wn, b)
    gWs, gWn, gb, dH = orc.sage_agg_bwd(H, F64, self_idx, indptr, idx, Ws, Wn, out, agg, relu, G)
    arrs = [H, Ws, Wn, b]
    for got, pos in ((dH, 0), (gWs, 1), (gWn, 2), (gb, 3)):
        np.testing.assert_allclose(got, fd_grad(loss, arrs, pos), rtol=1e-6, atol=1e-7)


def test_mean_aggregator_is_the_mean_layer(orc):
    rng, H, indptr, idx, self_idx, G = _case(3)
    d_in, d_out = H.shape[1], G.shape[1]
    Ws, Wn = rng.standard_normal((d_in, d_out)), rng.standard_normal((d_in, d_out))
    a = orc.sage_agg_bwd(H, F64, self_idx, indptr, idx, Ws, Wn, None, 0, False, G)
    b = orc.sage_bwd(H, F64, self_idx, indptr, idx, Ws, Wn, None, False, G)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=1e-13, atol=1e-13)


def test_sum_and_max_closed_cases(orc):
    rng = np.random.default_rng(5)
    d = 4
    H = rng.standard_normal((6, d))
    I, Z = np.eye(d), np.zeros((d, d))
    G = rng.standard_normal((2, d))
    indptr = np.array([0, 3, 5], np.int32)
    idx = np.array([4, -1, 5, 5, 5], np.int32)
    # sum, W_neigh = I: every valid entry receives the row's gradient once per occurrence
    _, gWn, _, dH = orc.sage_agg_bwd(H, F64, None, indptr, idx, Z, I, None, 1, False, G)
    want = np.zeros_like(H)
    want[4] = G[0]
    want[5] = G[0] + 2 * G[1]
    np.testing.assert_allclose(dH, want)
    np.testing.assert_allclose(gWn, np.outer(H[4] + H[5], G[0]) + np.outer(2 * H[5], G[1]))
    # max, W_neigh = I: per column the larger of rows 4 and 5 takes row 0's gradient; row 1's two
    # equal entries are one vertex, which takes all of it
    _, gWn, _, dH = orc.sage_agg_bwd(H, F64, None, indptr, idx, Z, I, None, 2, False, G)
    want = np.zeros_like(H)
    win = np.where(H[4] >= H[5], 4, 5)
    for k in range(d):
        want[win[k], k] += G[0, k]
    want[5] += G[1]
    np.testing.assert_allclose(dH, want)
    np.testing.assert_allclose(gWn, np.outer(np.maximum(H[4], H[5]), G[0]) + np.outer(H[5], G[1]))
    # max with equal values in two different rows: the first entry in the list takes the gradient
    H2 = H.copy()
    H2[5] = H2[4]
    for order, first in (([4, 5], 4), ([5, 4], 5)):
        _, _, _, dH = orc.sage_agg_bwd(H2, F64, None, np.array([0, 2], np.int32), np.array(order, np.int32), Z, I,
                                       None, 2, False, G[:1])
        want = np.zeros_like(H)
        want[first] = G[0]
        np.testing.assert_allclose(dH, want)
    # an empty segment aggregates to nothing: only the self term
    gWs, gWn, gb, dH = orc.sage_agg_bwd(H, F64, None, np.array([0, 0], np.int32), np.zeros(0, np.int32), I, I, None, 2,
                                        False, G[:1])
    want = np.zeros_like(H)
    want[0] = G[0]
    np.testing.assert_allclose(dH, want)
    np.testing.assert_allclose(gWn, 0)
    np.testing.assert_allclose(gWs, np.outer(H[0], G[0]))


def _dense_adjacency(n_dst, n_src, self_idx, indptr, idx):
    A = np.zeros((n_dst, n_src))
    for r in range(n_dst):
        s = r if self_idx is None else self_idx[r]
        if s >= 0:
            A[r, s] += 1
        for e in range(indptr[r], indptr[r + 1]):
            if idx[e] >= 0:
                A[r, idx[e]] += 1
    return A


@pytest.mark.parametrize("norm", [0, 1])
def test_gcn_against_the_dense_matrix_form(orc, norm):
    """out = A_hat H W with A_hat = (A + I) or D^-1 (A + I) as a dense matrix: gW = (A_hat H)^T dZ,
    dH = A_hat^T dZ W^T (plain numpy)."""
    rng, H, indptr, idx, self_idx, G = _case(20 + norm, n_src=11, n_dst=7)
    d_in, d_out = H.shape[1], G.shape[1]
    W, b = rng.standard_normal((d_in, d_out)), rng.standard_normal(d_out)
    A = _dense_adjacency(7, 11, self_idx, indptr, idx)
    if norm:
        deg = A.sum(1, keepdims=True)
        A = A / np.where(deg > 0, deg, 1.0)
    out = np.maximum(A @ H @ W + b, 0.0)
    np.testing.assert_allclose(orc.gcn_fwd(H, F64, self_idx, indptr, idx, W, b, norm, True), out, rtol=1e-12, atol=1e-12)
    dZ = G * (out > 0)
    gW, gb, dH = orc.gcn_bwd(H, F64, self_idx, indptr, idx, W, out, norm, True, G)
    np.testing.assert_allclose(gW, (A @ H).T @ dZ, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(gb, dZ.sum(0), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dH, A.T @ (dZ @ W.T), rtol=1e-12, atol=1e-12)
    # without the input gradient the others are unchanged
    gW2, gb2, none = orc.gcn_bwd(H, F64, self_idx, indptr, idx, W, out, norm, True, G, want_dH=False)
    assert none is None
    np.testing.assert_array_equal(gW2, gW)
    np.testing.assert_array_equal(gb2, gb)


@pytest.mark.parametrize("norm", [0, 1])
def test_gcn_matches_finite_differences(orc, norm):
    rng, H, indptr, idx, self_idx, G = _case(30 + norm)
    d_in, d_out = H.shape[1], G.shape[1]
    W, b = rng.standard_normal((d_in, d_out)), rng.standard_normal(d_out)
    fwd = lambda H_, W_, b_: orc.gcn_fwd(H_, F64, self_idx, indptr, idx, W_, b_, norm, False)
    loss = lambda *a: float((fwd(*a) * G).sum())
    gW, gb, dH = orc.gcn_bwd(H, F64, self_idx, indptr, idx, W, None, norm, False, G)
    for got, pos in ((dH, 0), (gW, 1), (gb, 2)):
        np.testing.assert_allclose(got, fd_grad(loss, [H, W, b], pos), rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("heads", [1, 2, 3])
@pytest.mark.parametrize("relu", [False, True])
def test_attention_matches_finite_differences(orc, heads, relu):
    rng, H, indptr, idx, self_idx, G = _case(40 + heads)
    d_in, d_out = H.shape[1], G.shape[1]
    W = rng.standard_normal((d_in, d_out))
    a_s, a_d, b = rng.standard_normal(d_out), rng.standard_normal(d_out), rng.standard_normal(d_out)
    fwd = lambda H_, W_, as_, ad_, b_: orc.gat_fwd(H_, F64, self_idx, indptr, idx, W_, as_, ad_, b_, heads, relu)
    loss = lambda *a: float((fwd(*a) * G).sum())
    out = fwd(H, W, a_s, a_d, b)
    gW, gas, gad, gb, dH = orc.gat_bwd(H, F64, self_idx, indptr, idx, W, a_s, a_d, out, heads, relu, G)
    arrs = [H, W, a_s, a_d, b]
    for got, pos in ((dH, 0), (gW, 1), (gas, 2), (gad, 3), (gb, 4)):
        np.testing.assert_allclose(got, fd_grad(loss, arrs, pos), rtol=2e-6, atol=2e-7)


def test_attention_closed_cases(orc):
    """Zero attention vectors make the softmax uniform: the layer is then the mean over the vertex
    and its neighbours of H W, i.e. the normalised GCN-style layer, and so is its backward; the
    attention vectors still receive their gradient through the scores."""
    rng, H, indptr, idx, self_idx, G = _case(50)
    d_in, d_out = H.shape[1], G.shape[1]
    W, b = rng.standard_normal((d_in, d_out)), rng.standard_normal(d_out)
    zero = np.zeros(d_out)
    out = orc.gat_fwd(H, F64, self_idx, indptr, idx, W, zero, zero, b, 2, True)
    np.testing.assert_allclose(out, orc.gcn_fwd(H, F64, self_idx, indptr, idx, W, b, 1, True), rtol=1e-12, atol=1e-12)
    gW, gas, gad, gb, dH = orc.gat_bwd(H, F64, self_idx, indptr, idx, W, zero, zero, out, 2, True, G)
    gW2, gb2, dH2 = orc.gcn_bwd(H, F64, self_idx, indptr, idx, W, out, 1, True, G)
    np.testing.assert_allclose(gW, gW2, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(gb, gb2, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dH, dH2, rtol=1e-11, atol=1e-12)
    assert np.abs(gas).max() > 1e-3          # d/d a_src at a = 0 is not zero in general
    # a destination row without any entry produces act(b): only the bias receives its gradient
    indptr0 = np.zeros(2, np.int32)
    out0 = orc.gat_fwd(H, F64, np.array([-1], np.int32), indptr0, np.zeros(0, np.int32), W, zero + 1, zero + 1, b, 2, False)
    gW, gas, gad, gb, dH = orc.gat_bwd(H, F64, np.array([-1], np.int32), indptr0, np.zeros(0, np.int32), W, zero + 1,
                                       zero + 1, out0, 2, False, G[:1])
    np.testing.assert_allclose(gb, G[0])
    for z in (gW, gas, gad, dH):
        np.testing.assert_allclose(z, 0)
    # accumulators are added to: the C entry twice on the same arrays doubles them
