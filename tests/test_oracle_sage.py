"""Pins for the oracle's GraphSAGE-mean layer and its storage rounding."""
import numpy as np
import pytest
import torch

F32, BF16, F16 = 0, 1, 2


def rand_csr(rng, n_dst, n_src, max_len, p_invalid=0.15):
    lens = rng.integers(0, max_len + 1, size=n_dst)
    indptr = np.zeros(n_dst + 1, np.int32)
    indptr[1:] = np.cumsum(lens)
    idx = rng.integers(0, n_src, size=int(indptr[-1])).astype(np.int32)
    idx[rng.random(len(idx)) < p_invalid] = -1
    return indptr, idx


def test_one_neighbour_mean_is_that_row_and_identity_weights(orc):
    rng = np.random.default_rng(0)
    H = rng.standard_normal((9, 6)).astype(np.float32)
    I = np.eye(6, dtype=np.float32)
    Z = np.zeros((6, 6), np.float32)
    indptr = np.arange(5, dtype=np.int32)
    idx = np.array([8, 2, 2, 0], np.int32)
    self_idx = np.array([1, 3, 5, 7], np.int32)
    # W_self = 0, W_neigh = I: out = mean = the single neighbour's row, exactly
    out = orc.sage_fwd(H, F32, self_idx, indptr, idx, Z, I, None, False)
    np.testing.assert_array_equal(out, H[idx].astype(np.float64))
    # W_self = I, W_neigh = 0: out = x_self exactly
    out = orc.sage_fwd(H, F32, self_idx, indptr, idx, I, Z, None, False)
    np.testing.assert_array_equal(out, H[self_idx].astype(np.float64))
    # identity self index when self_idx is NULL
    out = orc.sage_fwd(H, F32, None, indptr, idx, I, Z, None, False)
    np.testing.assert_array_equal(out, H[:4].astype(np.float64))
    # f copies of one row average to that row
    indptr2 = np.array([0, 5], np.int32)
    out = orc.sage_fwd(H, F32, None, indptr2, np.full(5, 4, np.int32), Z, I, None, False)
    np.testing.assert_allclose(out[0], H[4].astype(np.float64), rtol=1e-15)


def test_all_ones_features_give_column_sums(orc):
    rng = np.random.default_rng(1)
    d_in, d_out = 7, 5
    H = np.ones((10, d_in), np.float32)
    Ws = rng.standard_normal((d_in, d_out)).astype(np.float32)
    Wn = rng.standard_normal((d_in, d_out)).astype(np.float32)
    b = rng.standard_normal(d_out).astype(np.float32)
    indptr, idx = rand_csr(rng, 6, 10, 4, p_invalid=0.0)
    indptr[1:] += 1                       # make every segment non-empty
    idx = np.concatenate([[0], idx]).astype(np.int32)
    out = orc.sage_fwd(H, F32, None, indptr, idx, Ws, Wn, b, False)
    want = Ws.astype(np.float64).sum(0) + Wn.astype(np.float64).sum(0) + b
    np.testing.assert_allclose(out, np.tile(want, (6, 1)), rtol=1e-13, atol=1e-13)


def test_empty_segment_invalid_entries_and_negative_self(orc):
    rng = np.random.default_rng(2)
    H = rng.standard_normal((5, 4)).astype(np.float32)
    Ws = rng.standard_normal((4, 3)).astype(np.float32)
    Wn = rng.standard_normal((4, 3)).astype(np.float32)
    b = rng.standard_normal(3).astype(np.float32)
    indptr = np.array([0, 0, 3, 5, 6], np.int32)
    idx = np.array([-1, -1, -1, 1, -1, 2], np.int32)
    self_idx = np.array([0, 1, -1, 3], np.int32)
    out = orc.sage_fwd(H, F32, self_idx, indptr, idx, Ws, Wn, b, True)
    H64, Ws64, Wn64 = H.astype(np.float64), Ws.astype(np.float64), Wn.astype(np.float64)
    relu = lambda x: np.maximum(x, 0)
    np.testing.assert_allclose(out[0], relu(H64[0] @ Ws64 + b), rtol=1e-14, atol=1e-15)  # empty
    np.testing.assert_allclose(out[1], relu(H64[1] @ Ws64 + b), rtol=1e-14, atol=1e-15)  # all invalid
    # invalid entries do not count in the mean's divisor; negative self -> zero self row
    np.testing.assert_allclose(out[2], relu(H64[1] @ Wn64 + b), rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(out[3], relu(H64[3] @ Ws64 + H64[2] @ Wn64 + b), rtol=1e-14,
                               atol=1e-15)
    assert (out >= 0).all()


@pytest.mark.parametrize("dtype", [F32, BF16, F16])
def test_reduces_to_one_dense_gemm(orc, dtype):
    # out = act([x_self | mean] @ [W_self ; W_neigh] + b): the mean by an explicit
    # python loop, the product by numpy's matmul.
    rng = np.random.default_rng(10 + dtype)
    n_src, n_dst, d_in, d_out = 40, 23, 12, 9
    tdt = {F32: torch.float32, BF16: torch.bfloat16, F16: torch.float16}[dtype]

    def mk(*shape):
        t = torch.from_numpy(rng.standard_normal(shape).astype(np.float32)).to(tdt)
        bits = t.numpy() if dtype == F32 else t.view(torch.int16).numpy().view(np.uint16)
        return bits, t.to(torch.float64).numpy()

    Hb, H = mk(n_src, d_in)
    Wsb, Ws = mk(d_in, d_out)
    Wnb, Wn = mk(d_in, d_out)
    bb, b = mk(d_out)
    indptr, idx = rand_csr(rng, n_dst, n_src, 6)
    self_idx = rng.integers(0, n_src, size=n_dst).astype(np.int32)
    for relu in (False, True):
        out = orc.sage_fwd(Hb, dtype, self_idx, indptr, idx, Wsb, Wnb, bb, relu)
        A = np.zeros((n_dst, 2 * d_in))
        for r in range(n_dst):
            A[r, :d_in] = H[self_idx[r]]
            nb = [u for u in idx[indptr[r]:indptr[r + 1]] if u >= 0]
            if nb:
                A[r, d_in:] = sum(H[u] for u in nb) / len(nb)
        want = A @ np.vstack([Ws, Wn]) + b
        if relu:
            want = np.maximum(want, 0)
        np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-12)
    # a transposed weight would fail: W is [d_in, d_out], row-major, not square here
    assert d_in != d_out


def test_round_store_matches_library_conversions_and_rounds_once(orc):
    rng = np.random.default_rng(7)
    x = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-9, 6, 4000),
                        [0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e-8, 5.9e-8, 2.98e-8, 3e-8,
                         -1e-40, 1e-45, 3.4e38, 1e39]])
    # fp16: numpy converts float64 -> float16 with a single rounding
    with np.errstate(over="ignore"):
        want16 = x.astype(np.float16).view(np.uint16)
    got16 = orc.round_store(x, F16)
    np.testing.assert_array_equal(got16, want16)
    # fp32: C cast = numpy cast
    with np.errstate(over="ignore"):
        np.testing.assert_array_equal(orc.round_store(x, F32).view(np.uint32),
                                      x.astype(np.float32).view(np.uint32))
    # bf16: on values that are exact in fp32 torch's float->bf16 is a single RNE step
    with np.errstate(over="ignore"):
        xf = x.astype(np.float32)
    xf = xf[np.isfinite(xf)]
    want_bf = torch.from_numpy(xf).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(orc.round_store(xf.astype(np.float64), BF16), want_bf)
    # single rounding: 1 + 2^-8 + 2^-40 is above the tie -> rounds up to 1 + 2^-7;
    # rounding through fp32 first would land on the tie and go to 1.0
    v = np.array([1 + 2.0 ** -8 + 2.0 ** -40, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8])
    got = orc.load_f64(orc.round_store(v, BF16), BF16)
    np.testing.assert_array_equal(got, [1 + 2.0 ** -7, 1.0, 1 + 2.0 ** -6])
    # same for fp16 (10 fraction bits)
    v = np.array([1 + 2.0 ** -11 + 2.0 ** -45, 1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11])
    got = orc.load_f64(orc.round_store(v, F16), F16)
    np.testing.assert_array_equal(got, [1 + 2.0 ** -10, 1.0, 1 + 2.0 ** -9])


def test_load_f64_is_exact_for_every_half_and_sampled_bf16(orc):
    bits = np.arange(65536, dtype=np.uint16)
    got = orc.load_f64(bits, F16)
    want = bits.view(np.float16).astype(np.float64)
    np.testing.assert_array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    np.testing.assert_array_equal(got[ok], want[ok])
    gotb = orc.load_f64(bits, BF16)
    wantb = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    okb = ~np.isnan(wantb)
    np.testing.assert_array_equal(gotb[okb], wantb[okb])
    # round trip: every finite half / bf16 value is a fixed point of round_store
    np.testing.assert_array_equal(orc.round_store(want[ok], F16), bits[ok])
    np.testing.assert_array_equal(orc.round_store(wantb[okb], BF16), bits[okb])


def test_forward_chain_on_tiny_batch(orc):
    # two layers end to end against an explicit per-slot recursion in numpy
    rng = np.random.default_rng(3)
    N, D, Hd = 12, 5, 4
    rows = [rng.integers(0, N, size=int(rng.integers(0, 4))).tolist() for _ in range(N)]
    off = np.zeros(N + 1, np.int32)
    off[1:] = np.cumsum([len(r) for r in rows])
    idxs = np.array([x for r in rows for x in r], np.int32)
    X = rng.standard_normal((N, D)).astype(np.float32)
    seeds = np.array([0, 5, 7], np.int32)
    fan = [2, 3]
    ids, indptr = orc.sample(off, idxs, seeds, fan, key=1)
    uniq, remap = orc.pregather(ids)
    Xu = orc.gather(X, uniq)
    W = [tuple(rng.standard_normal(s).astype(np.float32) for s in ((d, Hd), (d, Hd), (Hd,)))
         for d in (D, Hd)]
    outs = orc.forward(Xu, F32, ids, indptr, remap, 3, fan, W)
    assert outs[0][0].shape == (3 + 6, Hd) and outs[1][0].shape == (3, Hd)

    def layer(self_rows, nbr_rows_list, Ws, Wn, b, relu):
        out = []
        for s, nb in zip(self_rows, nbr_rows_list):
            m = np.mean(nb, axis=0) if len(nb) else np.zeros_like(Ws[:, 0], dtype=np.float64)
            s = np.zeros(Ws.shape[0]) if s is None else s
            o = s @ Ws.astype(np.float64) + m @ Wn.astype(np.float64) + b
            out.append(np.maximum(o, 0) if relu else o)
        return out

    X64 = X.astype(np.float64)
    B = 3
    l1 = ids[B:B + 6]
    l2 = ids[B + 6:]
    feat = lambda v: X64[v] if v >= 0 else None
    # hidden rows for level 0 and level 1 slots
    selfs = [feat(v) for v in ids[:B + 6]]
    nbrs = [[X64[v] for v in l1[2 * m:2 * m + 2] if v >= 0] for m in range(B)] + \
           [[X64[v] for v in l2[3 * q:3 * q + 3] if v >= 0] for q in range(6)]
    h1 = layer(selfs, nbrs, *W[0], relu=True)
    np.testing.assert_allclose(outs[0][0], np.array(h1), rtol=1e-12, atol=1e-12)
    h1s = outs[0][1].astype(np.float64)        # stored (fp32-rounded) hidden rows
    selfs2 = [h1s[m] for m in range(B)]
    nbrs2 = [[h1s[B + 2 * m + j] for j in range(2) if l1[2 * m + j] >= 0] for m in range(B)]
    h2 = layer(selfs2, nbrs2, *W[1], relu=False)
    np.testing.assert_allclose(outs[1][0], np.array(h2), rtol=1e-12, atol=1e-12)
