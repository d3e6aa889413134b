"""Pins of the oracle's GCN-style and graph-attention layers: none of them calls the function
under test to produce its expectation.  Dense textbook formulations ((A+I) H W, D^-1 (A+I) H W,
masked row softmax from scipy), special cases with closed answers, and the link to the
GraphSAGE-mean oracle (itself pinned elsewhere)."""
import numpy as np
import pytest
from scipy.special import softmax

F64 = 3


def _case(rng, n_src, n_dst, d_in, d_out, max_len, p_invalid=0.2, p_self_invalid=0.1):
    H = rng.standard_normal((n_src, d_in))
    W = rng.standard_normal((d_in, d_out)) / np.sqrt(d_in)
    lens = rng.integers(0, max_len + 1, size=n_dst)
    indptr = np.zeros(n_dst + 1, np.int32)
    indptr[1:] = np.cumsum(lens)
    idx = rng.integers(0, n_src, size=int(indptr[-1])).astype(np.int32)
    idx[rng.random(len(idx)) < p_invalid] = -1
    self_idx = rng.integers(0, n_src, size=n_dst).astype(np.int32)
    self_idx[rng.random(n_dst) < p_self_invalid] = -1
    return H, W, self_idx, indptr, idx


def _dense_adjacency(n_dst, n_src, self_idx, indptr, idx):
    """(A + I) of the sampled block with multiplicities: A[r, u] = times u appears in row r's
    segment, plus one for the row's own source vertex."""
    A = np.zeros((n_dst, n_src))
    for r in range(n_dst):
        if self_idx[r] >= 0:
            A[r, self_idx[r]] += 1
        seg = idx[indptr[r]:indptr[r + 1]]
        np.add.at(A[r], seg[seg >= 0], 1)
    return A


@pytest.mark.parametrize("norm", [0, 1])
def test_gcn_equals_dense_normalised_adjacency_product(orc, norm):
    rng = np.random.default_rng(3 + norm)
    H, W, self_idx, indptr, idx = _case(rng, 40, 25, 7, 5, 6)
    b = rng.standard_normal(5)
    A = _dense_adjacency(25, 40, self_idx, indptr, idx)
    if norm:
        deg = A.sum(1, keepdims=True)
        A = np.divide(A, deg, out=np.zeros_like(A), where=deg > 0)
    expect = A @ H @ W + b
    got = orc.gcn_fwd(H, F64, self_idx, indptr, idx, W, b, norm, False)
    np.testing.assert_allclose(got, expect, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(orc.gcn_fwd(H, F64, self_idx, indptr, idx, W, b, norm, True), np.maximum(expect, 0),
                               rtol=1e-12, atol=1e-12)


def test_gcn_special_cases(orc):
    rng = np.random.default_rng(5)
    H = rng.standard_normal((6, 4))
    I = np.eye(4)
    # no neighbours: the vertex's own row comes through (either norm)
    ip0 = np.zeros(4, np.int32)
    for norm in (0, 1):
        np.testing.assert_array_equal(orc.gcn_fwd(H, F64, np.array([2, 0, 5], np.int32), ip0, np.zeros(0, np.int32),
                                                  I, None, norm, False), H[[2, 0, 5]])
    # rows 1 and 4 as neighbours of vertex 0: sum and mean of three rows
    ip = np.array([0, 2], np.int32)
    ix = np.array([1, 4], np.int32)
    s = H[0] + H[1] + H[4]
    np.testing.assert_allclose(orc.gcn_fwd(H, F64, np.array([0], np.int32), ip, ix, I, None, 0, False)[0], s, rtol=1e-15)
    np.testing.assert_allclose(orc.gcn_fwd(H, F64, np.array([0], np.int32), ip, ix, I, None, 1, False)[0], s / 3,
                               rtol=1e-15)
    # an invalid self row is neither added nor counted; an invalid entry likewise
    ix2 = np.array([1, -1], np.int32)
    np.testing.assert_allclose(orc.gcn_fwd(H, F64, np.array([-1], np.int32), ip, ix2, I, None, 1, False)[0], H[1],
                               rtol=1e-15)
    # nothing at all: the bias
    b = np.arange(4.0)
    np.testing.assert_array_equal(orc.gcn_fwd(H, F64, np.array([-1], np.int32), np.array([0, 1], np.int32),
                                              np.array([-1], np.int32), I, b, 1, False)[0], b)
    # identity self rows when self_idx is None
    np.testing.assert_array_equal(orc.gcn_fwd(H, F64, None, np.zeros(3, np.int32), np.zeros(0, np.int32), I, None, 0,
                                              False), H[:2])


def test_gcn_mean_from_the_sage_oracle(orc):
    """(x + c m)/(c+1) W = (x W + c (m W))/(c+1): the GraphSAGE-mean oracle run once with only the
    self weights and once with only the neighbour weights gives the GCN-mean layer."""
    rng = np.random.default_rng(8)
    H, W, self_idx, indptr, idx = _case(rng, 30, 20, 6, 4, 5, p_self_invalid=0.0)
    Z = np.zeros_like(W)
    xs = orc.sage_fwd(H, F64, self_idx, indptr, idx, W, Z, None, False)
    mn = orc.sage_fwd(H, F64, self_idx, indptr, idx, Z, W, None, False)
    c = np.array([(idx[indptr[r]:indptr[r + 1]] >= 0).sum() for r in range(20)], float)[:, None]
    np.testing.assert_allclose(orc.gcn_fwd(H, F64, self_idx, indptr, idx, W, None, 1, False), (xs + c * mn) / (c + 1),
                               rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("heads", [1, 2, 4])
def test_gat_equals_dense_masked_softmax(orc, heads):
    """Dense form: per head, scores s_dst[self_r] + s_src[u] through LeakyReLU(0.2), softmax over the
    row's entries with multiplicities (weights count * exp), times Z."""
    rng = np.random.default_rng(10 + heads)
    n_src, n_dst, d_in, d_out = 30, 22, 6, 8
    H, W, self_idx, indptr, idx = _case(rng, n_src, n_dst, d_in, d_out, 6, p_self_invalid=0.15)
    a_src, a_dst, b = rng.standard_normal(d_out), rng.standard_normal(d_out), rng.standard_normal(d_out)
    dh = d_out // heads
    Z = H @ W
    C = _dense_adjacency(n_dst, n_src, self_idx, indptr, idx)     # entry multiplicities
    expect = np.zeros((n_dst, d_out))
    for h in range(heads):
        sl = slice(h * dh, (h + 1) * dh)
        ssrc = Z[:, sl] @ a_src[sl]
        sdst = Z[:, sl] @ a_dst[sl]
        sd_row = np.where(self_idx >= 0, sdst[np.maximum(self_idx, 0)], 0.0)
        e = sd_row[:, None] + ssrc[None, :]
        e = np.where(e > 0, e, 0.2 * e)
        logits = np.where(C > 0, e + np.log(np.maximum(C, 1)), -np.inf)
        for r in range(n_dst):
            if (C[r] > 0).any():
                expect[r, sl] = softmax(logits[r]) @ Z[:, sl]
    expect += b
    got = orc.gat_fwd(H, F64, self_idx, indptr, idx, W, a_src, a_dst, b, heads, False)
    np.testing.assert_allclose(got, expect, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(orc.gat_fwd(H, F64, self_idx, indptr, idx, W, a_src, a_dst, b, heads, True),
                               np.maximum(expect, 0), rtol=1e-11, atol=1e-12)


def test_gat_special_cases(orc):
    rng = np.random.default_rng(12)
    H, W, self_idx, indptr, idx = _case(rng, 25, 15, 5, 6, 5, p_self_invalid=0.0)
    zero = np.zeros(6)
    # zero attention vectors: uniform weights = mean over the vertex and its neighbours of Z = H W,
    # which the dense normalised adjacency gives directly
    A = _dense_adjacency(15, 25, self_idx, indptr, idx)
    A /= A.sum(1, keepdims=True)
    np.testing.assert_allclose(orc.gat_fwd(H, F64, self_idx, indptr, idx, W, zero, zero, None, 2, False), A @ H @ W,
                               rtol=1e-12, atol=1e-13)
    # attention weights sum to one: identical source rows give that row's projection whatever a is
    Hc = np.tile(H[3], (25, 1))
    a1, a2 = rng.standard_normal(6), rng.standard_normal(6)
    np.testing.assert_allclose(orc.gat_fwd(Hc, F64, self_idx, indptr, idx, W, a1, a2, None, 3, False),
                               np.tile(H[3] @ W, (15, 1)), rtol=1e-12, atol=1e-13)
    # no neighbours: z of the vertex itself
    np.testing.assert_allclose(orc.gat_fwd(H, F64, np.array([4, 7], np.int32), np.zeros(3, np.int32),
                                           np.zeros(0, np.int32), W, a1, a2, None, 1, False), H[[4, 7]] @ W,
                               rtol=1e-13)
    # a dominant score picks out its entry: one neighbour whose s_src is far above the rest
    Hd = H.copy()
    Wi = np.eye(5, 6)
    a_src = np.zeros(6)
    a_src[0] = 1.0
    Hd[:, 0] = 0.0
    Hd[9, 0] = 500.0
    out = orc.gat_fwd(Hd, F64, np.array([2], np.int32), np.array([0, 3], np.int32), np.array([1, 9, 4], np.int32), Wi,
                      a_src, zero, None, 1, False)
    np.testing.assert_allclose(out[0], Hd[9] @ Wi, rtol=1e-12, atol=1e-12)
    # LeakyReLU slope: two entries with scores -10 and -20 -> -2 and -4 -> weights softmax([-2, -4])
    Hs = np.zeros((3, 5))
    Hs[1, 0], Hs[2, 0] = -10.0, -20.0
    Hs[1, 1], Hs[2, 1] = 1.0, 3.0
    out = orc.gat_fwd(Hs, F64, np.array([-1], np.int32), np.array([0, 2], np.int32), np.array([1, 2], np.int32), Wi,
                      a_src, zero, None, 1, False)
    w = softmax(np.array([-2.0, -4.0]))
    np.testing.assert_allclose(out[0, 1], w[0] * 1.0 + w[1] * 3.0, rtol=1e-13)
    # no entries at all: the bias
    b = np.arange(6.0)
    np.testing.assert_array_equal(orc.gat_fwd(H, F64, np.array([-1], np.int32), np.array([0, 1], np.int32),
                                              np.array([-1], np.int32), W, a1, a2, b, 2, False)[0], b)


def test_sage_aggregators_sum_and_max(orc):
    """sum = count x mean (the pinned mean oracle); max against numpy's reduction over the listed
    rows; closed cases."""
    rng = np.random.default_rng(21)
    H, W, self_idx, indptr, idx = _case(rng, 35, 24, 6, 5, 7)
    W2 = rng.standard_normal((6, 5))
    b = rng.standard_normal(5)
    Z = np.zeros_like(W)
    I = np.eye(6, 5)
    # agg 0 is the GraphSAGE-mean layer itself
    np.testing.assert_allclose(orc.sage_agg_fwd(H, F64, self_idx, indptr, idx, W, W2, b, 0, True),
                               orc.sage_fwd(H, F64, self_idx, indptr, idx, W, W2, b, True), rtol=1e-14, atol=1e-15)
    c = np.array([(idx[indptr[r]:indptr[r + 1]] >= 0).sum() for r in range(24)], float)[:, None]
    self_part = orc.sage_fwd(H, F64, self_idx, indptr, idx, W, Z, b, False)
    mean_part = orc.sage_fwd(H, F64, self_idx, indptr, idx, Z, W2, None, False)
    np.testing.assert_allclose(orc.sage_agg_fwd(H, F64, self_idx, indptr, idx, W, W2, b, 1, False),
                               self_part + c * mean_part, rtol=1e-12, atol=1e-12)
    # max: the aggregate itself (W_self = 0, W_neigh = [I | 0]) against numpy over the listed rows
    got = orc.sage_agg_fwd(H, F64, self_idx, indptr, idx, np.zeros((6, 5)), I, None, 2, False)
    for r in range(24):
        seg = idx[indptr[r]:indptr[r + 1]]
        seg = seg[seg >= 0]
        want = H[seg].max(axis=0)[:5] if len(seg) else np.zeros(5)
        np.testing.assert_array_equal(got[r], want)
    # all-negative rows: the maximum is negative, not the 0 the accumulator starts from
    Hn = -np.abs(H) - 1.0
    got = orc.sage_agg_fwd(Hn, F64, None, np.array([0, 3], np.int32), np.array([4, -1, 9], np.int32), np.zeros((6, 5)),
                           I, None, 2, False)
    np.testing.assert_array_equal(got[0], np.maximum(Hn[4], Hn[9])[:5])
    # one neighbour: every aggregator returns that row
    for agg in (0, 1, 2):
        got = orc.sage_agg_fwd(H, F64, None, np.array([0, 1], np.int32), np.array([7], np.int32), np.zeros((6, 5)), I,
                               None, agg, False)
        np.testing.assert_array_equal(got[0], H[7][:5])
