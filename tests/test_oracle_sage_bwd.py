"""Pins for the oracle's layer backward: central finite differences of the oracle's own
forward in float64 (an independent route to the same derivatives), plus special cases."""
import numpy as np

F64 = 3


def rand_csr(rng, n_dst, n_src, max_len, p_invalid=0.15):
    lens = rng.integers(0, max_len + 1, size=n_dst)
    indptr = np.zeros(n_dst + 1, np.int32)
    indptr[1:] = np.cumsum(lens)
    idx = rng.integers(0, n_src, size=int(indptr[-1])).astype(np.int32)
    idx[rng.random(len(idx)) < p_invalid] = -1
    return indptr, idx


def test_gradients_match_finite_differences(orc):
    rng = np.random.default_rng(0)
    n_src, n_dst, d_in, d_out = 9, 6, 4, 3
    H = rng.standard_normal((n_src, d_in))
    Ws = rng.standard_normal((d_in, d_out))
    Wn = rng.standard_normal((d_in, d_out))
    b = rng.standard_normal(d_out)
    indptr, idx = rand_csr(rng, n_dst, n_src, 4)
    self_idx = rng.integers(0, n_src, size=n_dst).astype(np.int32)
    self_idx[1] = -1
    G = rng.standard_normal((n_dst, d_out))           # dL/d out for L = sum(out * G)

    for relu in (False, True):
        fwd = lambda H_, Ws_, Wn_, b_: orc.sage_fwd(H_, F64, self_idx, indptr, idx, Ws_, Wn_, b_, relu)
        loss = lambda H_, Ws_, Wn_, b_: float((fwd(H_, Ws_, Wn_, b_) * G).sum())
        out = fwd(H, Ws, Wn, b)
        gWs, gWn, gb, dH = orc.sage_bwd(H, F64, self_idx, indptr, idx, Ws, Wn, out, relu, G)

        def fd(arr, which):
            g = np.zeros_like(arr)
            eps = 1e-6
            for i in np.ndindex(arr.shape):
                hi, lo = arr.copy(), arr.copy()
                hi[i] += eps
                lo[i] -= eps
                args = {"H": (H, Ws, Wn, b), "Ws": (H, Ws, Wn, b), "Wn": (H, Ws, Wn, b), "b": (H, Ws, Wn, b)}[which]
                a = list(args)
                pos = {"H": 0, "Ws": 1, "Wn": 2, "b": 3}[which]
                a[pos] = hi
                fh = loss(*a)
                a[pos] = lo
                fl = loss(*a)
                g[i] = (fh - fl) / (2 * eps)
            return g

        np.testing.assert_allclose(gWs, fd(Ws, "Ws"), rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(gWn, fd(Wn, "Wn"), rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(gb, fd(b, "b"), rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(dH, fd(H, "H"), rtol=1e-6, atol=1e-7)


def test_special_cases(orc):
    rng = np.random.default_rng(1)
    d = 5
    H = rng.standard_normal((7, d))
    I, Z = np.eye(d), np.zeros((d, d))
    indptr = np.arange(4, dtype=np.int32)          # one neighbour per row
    idx = np.array([6, 2, 2], np.int32)
    G = rng.standard_normal((3, d))
    # W_self = I, W_neigh = 0: dH is G scattered to the self rows (identity self index)
    gWs, gWn, gb, dH = orc.sage_bwd(H, F64, None, indptr, idx, I, Z, None, False, G)
    want = np.zeros_like(H)
    want[:3] = G
    np.testing.assert_allclose(dH, want)
    np.testing.assert_allclose(gWs, H[:3].T @ G)
    np.testing.assert_allclose(gWn, H[idx].T @ G)        # mean of one neighbour = that row
    np.testing.assert_allclose(gb, G.sum(0))
    # W_self = 0, W_neigh = I: the two rows that share neighbour 2 add up there
    _, _, _, dH = orc.sage_bwd(H, F64, None, indptr, idx, Z, I, None, False, G)
    want = np.zeros_like(H)
    want[6] = G[0]
    want[2] = G[1] + G[2]
    np.testing.assert_allclose(dH, want)
    # a mean over f valid entries hands each of them 1/f of the row's gradient
    indptr2 = np.array([0, 4], np.int32)
    idx2 = np.array([1, -1, 3, 1], np.int32)       # three valid entries, vertex 1 twice
    _, _, _, dH = orc.sage_bwd(H, F64, None, indptr2, idx2, Z, I, None, False, G[:1])
    want = np.zeros_like(H)
    want[1] = 2 * G[0] / 3
    want[3] = G[0] / 3
    np.testing.assert_allclose(dH, want)
    # ReLU mask comes from the stored forward output
    out = np.array([[1.0, -1.0, 0.0, 2.0, -3.0]])
    gWs, _, gb, _ = orc.sage_bwd(H, F64, None, indptr2, idx2, I, Z, out, True, G[:1])
    mask = np.array([1, 0, 0, 1, 0.0])
    np.testing.assert_allclose(gb, G[0] * mask)
    np.testing.assert_allclose(gWs, np.outer(H[0], G[0] * mask))
    # accumulation: calling twice on the same accumulators doubles them (checked via the C entry)


def test_sgd_update_closed_cases(orc):
    """W - lr g: exact small cases in every storage type, identity for lr = 0 or g = 0."""
    import numpy as np
    for dt, one, three_q in ((0, np.float32(1.0), np.float32(0.75)), (1, np.uint16(0x3F80), np.uint16(0x3F40)),
                             (2, np.uint16(0x3C00), np.uint16(0x3A00))):
        W = np.full((2, 3), one)
        g = np.ones((2, 3))
        np.testing.assert_array_equal(orc.sgd_update(W, dt, g, 0.25), np.full((2, 3), three_q))
        np.testing.assert_array_equal(orc.sgd_update(W, dt, g, 0.0), W)
        np.testing.assert_array_equal(orc.sgd_update(W, dt, np.zeros((2, 3)), 0.3), W)
    rng = np.random.default_rng(0)
    W = rng.standard_normal((5, 4)).astype(np.float32)
    g = rng.standard_normal((5, 4))
    np.testing.assert_allclose(orc.sgd_update(W, 0, g, 0.01), W - 0.01 * g, rtol=1e-7)
