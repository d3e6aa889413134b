"""GPU parity of the backward of the other layer kinds (GraphSAGE with sum / max aggregator, the
GCN-style layer) against the fp64 oracle, for fp32 and 2-byte activations, with and without the
input gradient, ReLU and bias, on shapes that span several tiles and row splits with ragged ends
(and narrow ones that take the element-wise routes).

2-byte activations: the device rounds the masked incoming gradient to the activation type before
the matrix products, so each gradient is compared twice - against the oracle fed the gradient
rounded the same way (both sides take that rounding in the same precision; what is left is fp32
summation order, and the rounding of the aggregate where it is an operand), and against the
oracle fed the unrounded gradient at the bound derived for that rounding."""
import numpy as np
import pytest
import torch

from helpers import GRAD_TOL, GRAD_TOL_SAME, ORC_DT, TOL, rel_err, round_like, to_bits, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

SHAPES = [(1500, 1111, 128, 128, 12), (4000, 777, 100, 256, 16), (300, 65, 7, 5, 4), (2500, 3000, 136, 132, 6)]


@pytest.fixture(scope="module")
def hb():
    from paper_2409_00657_amd import binding
    binding.load_library()
    return binding


def _rand_csr(rng, n_dst, n_src, max_len, p_invalid=0.15):
    lens = rng.integers(0, max_len + 1, size=n_dst)
    indptr = np.zeros(n_dst + 1, np.int32)
    indptr[1:] = np.cumsum(lens)
    idx = rng.integers(0, n_src, size=int(indptr[-1])).astype(np.int32)
    idx[rng.random(len(idx)) < p_invalid] = -1
    return indptr, idx


def _inputs(rng, dt, shape, quantise=False):
    n_src, n_dst, d_in, d_out, max_len = shape
    f = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float32))
    H = f(n_src, d_in)
    if quantise:        # few distinct values: equal maxima in different rows are common
        H = torch.round(H * 2) / 2
    H = H.to(dt).to(DEV)
    W1 = (f(d_in, d_out) / np.sqrt(d_in)).to(dt).to(DEV)
    W2 = (f(d_in, d_out) / np.sqrt(d_in)).to(dt).to(DEV)
    dOut = rng.standard_normal((n_dst, d_out)).astype(np.float32)
    indptr, idx = _rand_csr(rng, n_dst, n_src, max_len)
    self_idx = rng.integers(0, n_src, size=n_dst).astype(np.int32)
    self_idx[rng.random(n_dst) < 0.05] = -1
    return H, W1, W2, dOut, indptr, idx, self_idx


def _stored(orc, out64, dt):
    """The forward output as the device stores it (rounded to dt): what decides the ReLU mask."""
    bits = orc.round_store(out64, ORC_DT[dt])
    t = torch.from_numpy(bits if dt == torch.float32 else bits.view(np.int16))
    return bits, (t if dt == torch.float32 else t.view(dt)).to(DEV)


def _t(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("agg", [1, 2])
@pytest.mark.parametrize("shape", SHAPES)
def test_sage_aggregator_backward_vs_oracle(hb, orc, dt, agg, shape):
    n_src, n_dst, d_in, d_out, _ = shape
    rng = np.random.default_rng(n_src * 7 + d_in + agg)
    H, Ws, Wn, dOut, indptr, idx, self_idx = _inputs(rng, dt, shape, quantise=(agg == 2 and d_in == 7))
    odt = ORC_DT[dt]
    Hb, Wsb, Wnb = to_bits(H), to_bits(Ws), to_bits(Wn)
    out_bits, out_fwd = _stored(orc, orc.sage_agg_fwd(Hb, odt, self_idx, indptr, idx, Wsb, Wnb, None, agg, True), dt)
    on16 = dt != torch.float32 and d_in % 8 == 0 and d_out % 4 == 0     # weight gradient on the 2-byte instructions
    for relu, want_dh, use_bias in [(True, True, True), (False, False, False)]:
        ref = orc.sage_agg_bwd(Hb, odt, self_idx, indptr, idx, Wsb, Wnb, out_bits if relu else None, agg, relu,
                               dOut.astype(np.float64), want_dH=want_dh)
        same = ref if dt == torch.float32 else orc.sage_agg_bwd(Hb, odt, self_idx, indptr, idx, Wsb, Wnb,
                                                                 out_bits if relu else None, agg, relu,
                                                                 round_like(dOut, dt), want_dH=want_dh)
        w_ref = same if on16 else ref
        gWs = torch.zeros((d_in, d_out), device=DEV)
        gWn = torch.zeros((d_in, d_out), device=DEV)
        gb = torch.zeros(d_out, device=DEV) if use_bias else None
        dH = torch.full((n_src, d_in), 7.0, device=DEV) if want_dh else None
        ws = torch.empty(hb.hopgnn_sage_bwd_ws_bytes(dt, n_dst, d_in, d_out, want_dh), dtype=torch.uint8, device=DEV)
        ws.fill_(0x5A)
        hb.hopgnn_sage_bwd_agg(H, n_src, _t(self_idx), _t(indptr), _t(idx), n_dst, Ws, Wn, out_fwd if relu else None, agg,
                               relu, _t(dOut), gWs, gWn, gb, dH, ws)
        torch.cuda.synchronize()
        assert rel_err(to_f64(gWs), w_ref[0]) <= GRAD_TOL_SAME, (shape, relu)
        # the aggregate is rounded to the activation type before it is an operand
        assert rel_err(to_f64(gWn), w_ref[1]) <= (GRAD_TOL_SAME if dt == torch.float32 else TOL[dt]), (shape, relu)
        assert rel_err(to_f64(gWs), ref[0]) <= GRAD_TOL[dt] and rel_err(to_f64(gWn), ref[1]) <= GRAD_TOL[dt]
        if use_bias:
            assert rel_err(to_f64(gb), ref[2]) <= 2e-5
        if want_dh:
            assert rel_err(to_f64(dH), same[3]) <= GRAD_TOL_SAME
            assert rel_err(to_f64(dH), ref[3]) <= GRAD_TOL[dt]


def test_sage_aggregator_backward_mean_is_the_mean_call(hb):
    rng = np.random.default_rng(3)
    shape = (1500, 1111, 128, 128, 12)
    n_src, n_dst, d_in, d_out, _ = shape
    H, Ws, Wn, dOut, indptr, idx, self_idx = _inputs(rng, torch.float32, shape)
    res = []
    for call in ("agg", "mean"):
        gWs, gWn = torch.zeros((d_in, d_out), device=DEV), torch.zeros((d_in, d_out), device=DEV)
        gb, dH = torch.zeros(d_out, device=DEV), torch.empty((n_src, d_in), device=DEV)
        ws = torch.empty(hb.hopgnn_sage_bwd_ws_bytes(torch.float32, n_dst, d_in, d_out, True), dtype=torch.uint8, device=DEV)
        if call == "agg":
            hb.hopgnn_sage_bwd_agg(H, n_src, _t(self_idx), _t(indptr), _t(idx), n_dst, Ws, Wn, None, 0, False, _t(dOut),
                                   gWs, gWn, gb, dH, ws)
        else:
            hb.hopgnn_sage_bwd(H, n_src, _t(self_idx), _t(indptr), _t(idx), n_dst, Ws, Wn, None, False, _t(dOut), gWs, gWn,
                               gb, dH, ws)
        torch.cuda.synchronize()
        res.append((gWs, gWn, gb, dH))
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1]) and torch.equal(res[0][2], res[1][2])
    assert rel_err(to_f64(res[0][3]), to_f64(res[1][3])) <= 1e-6      # atomic order


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("norm", [0, 1])
@pytest.mark.parametrize("shape", SHAPES)
def test_gcn_backward_vs_oracle(hb, orc, dt, norm, shape):
    n_src, n_dst, d_in, d_out, _ = shape
    rng = np.random.default_rng(n_src * 5 + d_in + norm)
    H, W, _, dOut, indptr, idx, self_idx = _inputs(rng, dt, shape)
    odt = ORC_DT[dt]
    Hb, Wb = to_bits(H), to_bits(W)
    out_bits, out_fwd = _stored(orc, orc.gcn_fwd(Hb, odt, self_idx, indptr, idx, Wb, None, norm, True), dt)
    on16 = dt != torch.float32 and d_in % 8 == 0 and d_out % 4 == 0
    for relu, want_dh, use_bias in [(True, True, True), (False, False, False)]:
        ref = orc.gcn_bwd(Hb, odt, self_idx, indptr, idx, Wb, out_bits if relu else None, norm, relu,
                          dOut.astype(np.float64), want_dH=want_dh)
        same = ref if dt == torch.float32 else orc.gcn_bwd(Hb, odt, self_idx, indptr, idx, Wb, out_bits if relu else None,
                                                            norm, relu, round_like(dOut, dt), want_dH=want_dh)
        w_ref = same if on16 else ref
        gW = torch.zeros((d_in, d_out), device=DEV)
        gb = torch.zeros(d_out, device=DEV) if use_bias else None
        dH = torch.full((n_src, d_in), 7.0, device=DEV) if want_dh else None
        ws = torch.empty(hb.hopgnn_sage_bwd_ws_bytes(dt, n_dst, d_in, d_out, want_dh), dtype=torch.uint8, device=DEV)
        ws.fill_(0x5A)
        hb.hopgnn_gcn_bwd(H, n_src, _t(self_idx), _t(indptr), _t(idx), n_dst, W, out_fwd if relu else None, norm, relu,
                          _t(dOut), gW, gb, dH, ws)
        torch.cuda.synchronize()
        assert rel_err(to_f64(gW), w_ref[0]) <= (GRAD_TOL_SAME if dt == torch.float32 else TOL[dt]), (shape, relu)
        assert rel_err(to_f64(gW), ref[0]) <= GRAD_TOL[dt]
        if use_bias:
            assert rel_err(to_f64(gb), ref[1]) <= 2e-5
        if want_dh:
            assert rel_err(to_f64(dH), same[2]) <= GRAD_TOL_SAME
            assert rel_err(to_f64(dH), ref[2]) <= GRAD_TOL[dt]
        # accumulation: a second call on the same accumulators doubles them (powers of two: exact)
        if not relu:
            g1 = gW.clone()
            hb.hopgnn_gcn_bwd(H, n_src, _t(self_idx), _t(indptr), _t(idx), n_dst, W, None, norm, False, _t(dOut), gW, gb,
                              None, ws)
            torch.cuda.synchronize()
            assert torch.equal(gW, 2 * g1)


def test_layer_backward_argument_errors(hb):
    from paper_2409_00657_amd.binding import HopgnnError
    rng = np.random.default_rng(0)
    shape = (40, 30, 8, 8, 3)
    n_src, n_dst, d_in, d_out, _ = shape
    H, W, W2, dOut, indptr, idx, self_idx = _inputs(rng, torch.float32, shape)
    g = lambda: torch.zeros((d_in, d_out), device=DEV)
    ws = torch.empty(hb.hopgnn_sage_bwd_ws_bytes(torch.float32, n_dst, d_in, d_out, True), dtype=torch.uint8, device=DEV)
    with pytest.raises(HopgnnError):
        hb.hopgnn_sage_bwd_agg(H, n_src, _t(self_idx), _t(indptr), _t(idx), n_dst, W, W2, None, 3, False, _t(dOut), g(), g(),
                               None, None, ws)
    with pytest.raises(HopgnnError):
        hb.hopgnn_gcn_bwd(H, n_src, _t(self_idx), _t(indptr), _t(idx), n_dst, W, None, 2, False, _t(dOut), g(), None, None, ws)
    with pytest.raises(HopgnnError):     # ReLU without the stored forward output
        hb.hopgnn_gcn_bwd(H, n_src, _t(self_idx), _t(indptr), _t(idx), n_dst, W, None, 1, True, _t(dOut), g(), None, None, ws)
    with pytest.raises(HopgnnError):     # workspace too small
        hb.hopgnn_gcn_bwd(H, n_src, _t(self_idx), _t(indptr), _t(idx), n_dst, W, None, 1, False, _t(dOut), g(), None, None,
                          ws[:256])


GAT_SHAPES = [  # n_src, n_dst, d_in, d_out, longest segment, heads
    (1500, 1111, 128, 128, 12, 4), (4000, 777, 100, 256, 16, 2), (300, 65, 7, 6, 4, 3), (2500, 900, 136, 132, 6, 1),
    (600, 40, 32, 64, 150, 8)]      # the last: segments longer than a wavefront


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("shape", GAT_SHAPES)
def test_attention_backward_vs_oracle(hb, orc, dt, shape):
    """The forward call runs first on the device (its workspace holds z and the scores the backward
    call reads; its stored output decides the ReLU mask on both sides)."""
    n_src, n_dst, d_in, d_out, max_len, heads = shape
    rng = np.random.default_rng(n_src * 3 + d_in + heads)
    H, W, _, dOut, indptr, idx, self_idx = _inputs(rng, dt, (n_src, n_dst, d_in, d_out, max_len))
    f = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float32))
    a_s, a_d, b = (f(d_out) * 0.3).to(dt).to(DEV), (f(d_out) * 0.3).to(dt).to(DEV), (f(d_out) * 0.1).to(dt).to(DEV)
    odt = ORC_DT[dt]
    for relu, want_dh, use_bias in [(True, True, True), (False, False, False)]:
        fwd_ws = torch.empty(hb.hopgnn_gat_fwd_ws_bytes(dt, n_src, d_in, d_out, heads), dtype=torch.uint8, device=DEV)
        out = torch.empty((n_dst, d_out), dtype=dt, device=DEV)
        hb.hopgnn_gat_fwd(H, n_src, _t(self_idx), _t(indptr), _t(idx), n_dst, W, a_s, a_d, b if use_bias else None, heads,
                          relu, out, fwd_ws)
        gW = torch.zeros((d_in, d_out), device=DEV)
        gas, gad = torch.zeros(d_out, device=DEV), torch.zeros(d_out, device=DEV)
        gb = torch.zeros(d_out, device=DEV) if use_bias else None
        dH = torch.full((n_src, d_in), 7.0, device=DEV) if want_dh else None
        ws = torch.empty(hb.hopgnn_gat_bwd_ws_bytes(dt, n_src, n_dst, d_in, d_out, heads), dtype=torch.uint8, device=DEV)
        ws.fill_(0x5A)
        hb.hopgnn_gat_bwd(H, n_src, _t(self_idx), _t(indptr), _t(idx), n_dst, W, a_s, a_d, out if relu else None, fwd_ws,
                          relu, _t(dOut), heads, gW, gas, gad, gb, dH, ws)
        torch.cuda.synchronize()
        ref = orc.gat_bwd(to_bits(H), odt, self_idx, indptr, idx, to_bits(W), to_bits(a_s), to_bits(a_d),
                          to_bits(out) if relu else None, heads, relu, dOut.astype(np.float64), want_dH=want_dh)
        # fp32: everything is fp32 arithmetic (exp, sums in another order); 2-byte: the gradient with
        # respect to z is rounded to the activation type before the two matrix products
        tol = 1e-4 if dt == torch.float32 else GRAD_TOL[dt]
        assert rel_err(to_f64(gW), ref[0]) <= tol, (shape, relu)
        assert rel_err(to_f64(gas), ref[1]) <= 1e-4 and rel_err(to_f64(gad), ref[2]) <= 1e-4, (shape, relu)
        if use_bias:
            assert rel_err(to_f64(gb), ref[3]) <= 2e-5
        if want_dh:
            assert rel_err(to_f64(dH), ref[4]) <= tol, (shape, relu)


def test_attention_backward_argument_errors(hb):
    from paper_2409_00657_amd.binding import HopgnnError
    rng = np.random.default_rng(0)
    n_src, n_dst, d_in, d_out, heads = 40, 30, 8, 8, 2
    H, W, _, dOut, indptr, idx, self_idx = _inputs(rng, torch.float32, (n_src, n_dst, d_in, d_out, 3))
    a = torch.zeros(d_out, device=DEV)
    fwd_ws = torch.zeros(hb.hopgnn_gat_fwd_ws_bytes(torch.float32, n_src, d_in, d_out, heads), dtype=torch.uint8, device=DEV)
    ws = torch.empty(hb.hopgnn_gat_bwd_ws_bytes(torch.float32, n_src, n_dst, d_in, d_out, heads), dtype=torch.uint8, device=DEV)
    g = lambda: torch.zeros((d_in, d_out), device=DEV)
    v = lambda: torch.zeros(d_out, device=DEV)
    call = lambda **k: hb.hopgnn_gat_bwd(H, n_src, _t(self_idx), _t(indptr), _t(idx), n_dst, W, a, a, k.get("out"),
                                         k.get("fwd_ws", fwd_ws), k.get("relu", False), _t(dOut), k.get("heads", heads), g(),
                                         v(), v(), None, None, k.get("ws", ws))
    call()                                        # the valid call
    torch.cuda.synchronize()
    for bad in (dict(heads=3), dict(heads=0), dict(relu=True), dict(ws=ws[:256])):
        with pytest.raises(HopgnnError):
            call(**bad)
    assert hb.hopgnn_gat_bwd_ws_bytes(torch.float32, n_src, n_dst, d_in, d_out, 3) == 0


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_attention_backward_with_a_device_row_count(hb, dt):
    """Source rows past the device-side count (here NaN, as unwritten memory may be) are neither read
    nor written: same gradients as the call on exactly the rows that exist."""
    n_src, n_dst, d_in, d_out, max_len, heads = 1500, 1111, 128, 128, 12, 4
    extra = 77
    rng = np.random.default_rng(17)
    H, W, _, dOut, indptr, idx, self_idx = _inputs(rng, dt, (n_src, n_dst, d_in, d_out, max_len))
    a_s = torch.from_numpy(rng.standard_normal(d_out).astype(np.float32) * 0.3).to(dt).to(DEV)
    a_d = torch.from_numpy(rng.standard_normal(d_out).astype(np.float32) * 0.3).to(dt).to(DEV)
    Hcap = torch.cat([H, torch.full((extra, d_in), float("nan"), dtype=dt, device=DEV)])
    n_dev = torch.tensor([n_src], dtype=torch.int64, device=DEV)
    res = []
    for Hin, cap, cnt in ((H, n_src, None), (Hcap, n_src + extra, n_dev)):
        fwd_ws = torch.empty(hb.hopgnn_gat_fwd_ws_bytes(dt, cap, d_in, d_out, heads), dtype=torch.uint8, device=DEV)
        fwd_ws.fill_(0xFF)          # NaN patterns where nothing is written
        out = torch.empty((n_dst, d_out), dtype=dt, device=DEV)
        hb.hopgnn_gat_fwd(Hin, cap, _t(self_idx), _t(indptr), _t(idx), n_dst, W, a_s, a_d, None, heads, True, out, fwd_ws,
                          n_src_dev=cnt)
        gW, gas, gad = torch.zeros((d_in, d_out), device=DEV), torch.zeros(d_out, device=DEV), torch.zeros(d_out, device=DEV)
        dH = torch.full((cap, d_in), 7.0, device=DEV)
        ws = torch.empty(hb.hopgnn_gat_bwd_ws_bytes(dt, cap, n_dst, d_in, d_out, heads), dtype=torch.uint8, device=DEV)
        ws.fill_(0xFF)
        hb.hopgnn_gat_bwd(Hin, cap, _t(self_idx), _t(indptr), _t(idx), n_dst, W, a_s, a_d, out, fwd_ws, True, _t(dOut), heads,
                          gW, gas, gad, None, dH, ws, n_src_dev=cnt)
        torch.cuda.synchronize()
        res.append((gW, gas, gad, dH))
    (gW0, gas0, gad0, dH0), (gW1, gas1, gad1, dH1) = res
    assert torch.isfinite(gW1).all() and torch.isfinite(gas1).all() and torch.isfinite(gad1).all()
    # float atomics inside: equal up to summation order
    assert rel_err(to_f64(gW1), to_f64(gW0)) <= 1e-4 and rel_err(to_f64(gas1), to_f64(gas0)) <= 1e-4
    assert rel_err(to_f64(gad1), to_f64(gad0)) <= 1e-4 and rel_err(to_f64(dH1[:n_src]), to_f64(dH0)) <= 1e-4
    assert bool((dH1[n_src:] == 7.0).all())        # rows that do not exist stay untouched


@pytest.mark.parametrize("model", ["gcn", "gat"])
def test_pipeline_backward_chain_vs_oracle_and_training(hb, orc, model):
    """A sampled batch of the small workload through HotPath: forward, then the pipeline's own backward
    calls (last layer first).  Every layer's gradients against the oracle from the device's stored
    activations and incoming gradient; then SGD iterations on a fixed pair of batches lower
    1/2 |H_L|^2."""
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import HotPath
    cfg = synth.CONFIGS[1]
    g = cfg.make_graph(device=DEV)
    X = cfg.make_features(device=DEV)
    W = cfg.make_weights(device=DEV)
    hp = HotPath(g.offsets, g.indices, X, W, cfg.batch, cfg.fanouts, model=model)
    hp.enable_backward()
    seeds = synth.seeds(cfg.n_vertices, cfg.batch, 5, device=DEV)
    out = hp.run_batch(seeds, 5)
    hp.backward(0)
    torch.cuda.synchronize()
    sh = hp.shape
    B, L = sh.n_seeds, sh.n_layers
    assert L == 2
    U = int(hp.n_uniq.item())
    remap, indptr, slot_idx = hp.remap.cpu().numpy(), hp.indptr.cpu().numpy(), hp.slot_idx[0].cpu().numpy()
    n2, n1 = sh.n_dst(2), sh.n_dst(1)
    H1, Xu = to_bits(hp.H[0]), to_bits(hp.Xu[:U])
    dOut2 = to_f64(out)                               # dL/dH_L = H_L for fp32 activations
    w = lambda k: to_bits(W[k][0])
    if model == "gcn":
        ref2 = orc.gcn_bwd(H1, 0, None, indptr[:n2 + 1], slot_idx[:sh.nnz(2)], w(1), None, 1, False, dOut2)
        dH1 = to_f64(hp.dH[0])
        ref1 = orc.gcn_bwd(Xu, 0, remap[:n1], indptr[:n1 + 1], remap[B:B + sh.nnz(1)], w(0), H1, 1, True, dH1, want_dH=False)
        got2, got1 = (hp.gW[1][0], hp.gW[1][2]), (hp.gW[0][0], hp.gW[0][2])
        ref2_dH, names = ref2[2], ("gW", "gbias")
    else:
        a = lambda k, j: to_bits(hp.attn[k][j])
        ref2 = orc.gat_bwd(H1, 0, None, indptr[:n2 + 1], slot_idx[:sh.nnz(2)], w(1), a(1, 0), a(1, 1), None, hp.gat_heads,
                           False, dOut2)
        dH1 = to_f64(hp.dH[0])
        ref1 = orc.gat_bwd(Xu, 0, remap[:n1], indptr[:n1 + 1], remap[B:B + sh.nnz(1)], w(0), a(0, 0), a(0, 1), H1,
                           hp.gat_heads, True, dH1, want_dH=False)
        got2 = (hp.gW[1][0], hp.g_attn[1][0], hp.g_attn[1][1], hp.gW[1][2])
        got1 = (hp.gW[0][0], hp.g_attn[0][0], hp.g_attn[0][1], hp.gW[0][2])
        ref2_dH, names = ref2[4], ("gW", "ga_src", "ga_dst", "gbias")
    tol = 1e-4
    for k, (got, ref) in ((2, (got2, ref2)), (1, (got1, ref1))):
        for name, gt, rf in zip(names, got, ref):
            if gt is not None:
                assert rel_err(to_f64(gt), rf.reshape(gt.shape)) <= tol, (model, k, name)
    assert rel_err(dH1, ref2_dH) <= tol

    # training: gradients of two batches accumulate, one update per iteration
    hp.apply_sgd(0.0)                                  # clears the accumulators
    batches = [(synth.seeds(cfg.n_vertices, cfg.batch, s, device=DEV), s) for s in (3, 4)]
    losses = []
    for it in range(6):
        loss = 0.0
        for sd, key in batches:
            o = hp.run_batch(sd, key)
            loss += 0.5 * float((o.double() ** 2).sum().item())
            hp.backward(0)
        losses.append(loss)
        hp.apply_sgd(3e-4)
    torch.cuda.synchronize()
    assert all(b < a for a, b in zip(losses, losses[1:])), losses
