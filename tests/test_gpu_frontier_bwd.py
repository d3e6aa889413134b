"""GPU parity of the backward pass over frontier structures (deduplicated and layer-wise sampled
micrographs) whose row counts only the device knows: weight gradients against the oracle chain."""
import numpy as np
import pytest
import torch

from helpers import ORC_DT, rel_err, to_bits, to_f64, weights_bits
from oracle import dedup as orc_dedup
from oracle import frontier as orc_frontier
from oracle import layerwise as orc_lw

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GRAD_TOL = {torch.float32: 5e-5, torch.bfloat16: 3e-2}


@pytest.fixture(scope="module")
def hb():
    from paper_2409_00657_amd import binding
    binding.load_library()
    return binding


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("sampler,fanouts", [("node", [5, 4]), ("node", [4, 3, 3]), ("layer", [6, 12]), ("layer", [5, 8, 10])])
def test_backward_over_frontiers_vs_oracle_chain(hb, orc, dt, sampler, fanouts):
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import DedupPath
    g = synth.rmat_graph(12, 10.0, device=DEV)
    n, d, hidden, B, L = g.n_vertices, 24, 40, 50, len(fanouts)
    X = synth.features(n, d, dt, device=DEV)
    W = synth.sage_weights(d, hidden, L, dt, device=DEV, bias=True)
    dp = DedupPath(g.offsets, g.indices, X, W, B, fanouts, sampler=sampler)
    dp.enable_backward()
    # whatever lies past the row counts must not reach a gradient
    for t in dp.H + dp.dH:
        t.fill_(float("nan"))
    dp.bwd_ws.fill_(0xFF)
    off_np, idx_np = g.offsets.cpu().numpy(), g.indices.cpu().numpy()
    seeds = synth.seeds(n, B, 3, device=DEV)
    out = dp.run_batch(seeds, 11)
    dp.backward()
    torch.cuda.synchronize()
    sample = orc_dedup.sample_dedup if sampler == "node" else orc_lw.sample_layerwise
    st = sample(off_np, idx_np, seeds.cpu().numpy(), fanouts, 11)
    dOut = to_f64(dp.dHL)
    if dt == torch.float32:
        # end to end: forward and backward chain of the oracle from the same inputs
        ref_out, ref = orc_frontier.layer_chain_grads(orc, to_bits(X), ORC_DT[dt], *st, weights_bits(W), dOut)
        assert rel_err(to_f64(out), ref_out) <= 1e-5 * L
        for k in range(L):
            for part in range(3):
                got = to_f64(dp.gW[k][part])
                assert np.isfinite(got).all()
                assert rel_err(got, ref[k][part]) <= GRAD_TOL[dt] * L, (k, part)
    else:
        # 2-byte activations: a pre-activation that rounds across zero flips its ReLU mask, so every
        # layer is checked on its own from the GPU's stored activations and incoming gradient
        nv, ls, ip, ix = st
        uniq, remap = orc.pregather(nv)
        U = len(uniq)
        Wb = weights_bits(W)
        for k in range(L, 0, -1):
            n_dst, self_idx, ipk, ixk = orc_frontier.layer_inputs(k, L, ls, ip, ix, remap)
            src = to_bits(dp.Xu[:U]) if k == 1 else to_bits(dp.H[k - 2][:int(ls[L - k + 2])])
            d_k = dOut if k == L else to_f64(dp.dH[k - 1][:n_dst])
            ref = orc.sage_bwd(src, ORC_DT[dt], self_idx, ipk, ixk, Wb[k - 1][0], Wb[k - 1][1],
                               to_bits(dp.H[k - 1][:n_dst]) if k < L else None, k < L, d_k, want_dH=(k > 1))
            for part in range(3):
                got = to_f64(dp.gW[k - 1][part])
                assert np.isfinite(got).all()
                assert rel_err(got, ref[part]) <= GRAD_TOL[dt], (k, part)
            if k > 1:
                assert rel_err(to_f64(dp.dH[k - 2][:int(ls[L - k + 2])]), ref[3]) <= GRAD_TOL[dt], k
    # gradients accumulate in place: a second backward of the same batch doubles them
    first = [[t.clone() for t in layer] for layer in dp.gW]
    dp.backward()
    torch.cuda.synchronize()
    for k in range(L):
        for part in range(3):
            assert rel_err(to_f64(dp.gW[k][part]), 2 * to_f64(first[k][part])) <= 1e-6
    # the update takes them and clears the accumulators
    w_before = to_f64(W[0][0]).copy()
    dp.apply_sgd(1e-3)
    torch.cuda.synchronize()
    assert float(dp.gW[0][0].abs().max()) == 0.0
    want = w_before - 1e-3 * 2 * to_f64(first[0][0])
    assert rel_err(to_f64(W[0][0]), want) <= (1e-6 if dt == torch.float32 else 1e-2)


def test_sage_bwd_dev_counts_equal_trimmed_call(hb):
    """With explicit counts the call equals hopgnn_sage_bwd on arrays cut to those counts."""
    rng = np.random.default_rng(4)
    n_dst_cap, n_src_cap, n_dst, n_src, d_in, d_out = 300, 500, 177, 333, 20, 28
    lens = rng.integers(0, 6, size=n_dst_cap)
    lens[n_dst:] = 0
    indptr = np.zeros(n_dst_cap + 1, np.int32)
    indptr[1:] = np.cumsum(lens)
    idx = rng.integers(0, n_src, size=int(indptr[-1])).astype(np.int32)
    t = lambda a, dt=None: torch.as_tensor(a, device=DEV) if dt is None else torch.as_tensor(a, device=DEV, dtype=dt)
    H = t(rng.standard_normal((n_src_cap, d_in)), torch.float32)
    Ws, Wn = t(rng.standard_normal((d_in, d_out)), torch.float32), t(rng.standard_normal((d_in, d_out)), torch.float32)
    out_fwd = t(rng.standard_normal((n_dst_cap, d_out)), torch.float32)
    dOut = t(rng.standard_normal((n_dst_cap, d_out)), torch.float32)
    H[n_src:] = float("nan")
    out_fwd[n_dst:] = float("nan")
    dOut[n_dst:] = float("nan")
    ip, ix = t(indptr), t(idx)
    cnt_dst, cnt_src = t(np.array([n_dst], np.int64)), t(np.array([n_src], np.int64))

    def run(dev_counts):
        gWs, gWn, gb = torch.zeros_like(Ws), torch.zeros_like(Wn), torch.zeros(d_out, device=DEV)
        if dev_counts:
            dH = torch.full((n_src_cap, d_in), 7.0, device=DEV)
            ws = torch.empty(hb.hopgnn_sage_bwd_ws_bytes(torch.float32, n_dst_cap, d_in, d_out, True), dtype=torch.uint8,
                             device=DEV)
            ws.fill_(0xFF)
            hb.hopgnn_sage_bwd_dev(H, n_src_cap, cnt_src, None, ip, ix, n_dst_cap, cnt_dst, Ws, Wn, out_fwd, True, dOut,
                                   gWs, gWn, gb, dH, ws)
        else:
            dH = torch.full((n_src, d_in), 7.0, device=DEV)
            ws = torch.empty(hb.hopgnn_sage_bwd_ws_bytes(torch.float32, n_dst, d_in, d_out, True), dtype=torch.uint8,
                             device=DEV)
            hb.hopgnn_sage_bwd(H[:n_src].contiguous(), n_src, None, ip[:n_dst + 1].contiguous(), ix, n_dst, Ws, Wn,
                               out_fwd[:n_dst].contiguous(), True, dOut[:n_dst].contiguous(), gWs, gWn, gb, dH, ws)
        torch.cuda.synchronize()
        return gWs, gWn, gb, dH
    a, b = run(True), run(False)
    for x, y in zip(a[:3], b[:3]):
        assert rel_err(to_f64(x), to_f64(y)) <= 1e-6
    assert rel_err(to_f64(a[3][:n_src]), to_f64(b[3])) <= 1e-6
    assert bool((a[3][n_src:] == 7.0).all())            # rows past the count are left alone


@pytest.mark.parametrize("sampler", ["node", "layer"])
def test_train_step_equals_the_step_by_step_sequence(hb, sampler):
    """train_step (every call with pre-marshalled arguments) against run_batch + backward +
    apply_sgd on a copy of the weights: the same updated weights."""
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import DedupPath
    g = synth.rmat_graph(11, 8.0, device=DEV)
    n, d, hidden, B, fan = g.n_vertices, 16, 24, 40, [5, 6]
    X = synth.features(n, d, torch.float32, device=DEV)
    W1 = synth.sage_weights(d, hidden, 2, torch.float32, device=DEV, bias=True)
    W2 = [tuple(t.clone() for t in layer) for layer in W1]
    a = DedupPath(g.offsets, g.indices, X, W1, B, fan, sampler=sampler)
    b = DedupPath(g.offsets, g.indices, X, W2, B, fan, sampler=sampler)
    a.enable_backward()
    b.enable_backward()
    for it in range(3):
        seeds = synth.seeds(n, B, 60 + it, device=DEV)
        a.train_step(seeds, 80 + it, 1e-3)
        b.run_batch(seeds, 80 + it)
        b.backward()
        b.apply_sgd(1e-3)
    torch.cuda.synchronize()
    for la, lb in zip(W1, W2):
        for ta, tb in zip(la, lb):
            assert rel_err(to_f64(ta), to_f64(tb)) <= 1e-6      # dH arrives by float atomics: not bit for bit
    assert float(sum(t.abs().sum() for layer in a.gW for t in layer)) == 0.0
