"""GPU parity of the layer backward against the fp64 oracle."""
import numpy as np
import pytest
import torch

from helpers import ORC_DT, rel_err, to_bits, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
F32 = 0


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


def _run_gpu(hb, H, self_idx, indptr, idx, Ws, Wn, out_fwd, relu, dOut, want_dh, use_bias, acc_init=None):
    n_src, d_in = H.shape
    d_out = Ws.shape[1]
    n_dst = len(indptr) - 1
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    gWs = torch.zeros((d_in, d_out), device=DEV) if acc_init is None else acc_init[0].clone()
    gWn = torch.zeros((d_in, d_out), device=DEV) if acc_init is None else acc_init[1].clone()
    gb = (torch.zeros(d_out, device=DEV) if acc_init is None else acc_init[2].clone()) if use_bias else None
    dH = torch.full((n_src, d_in), 7.0, device=DEV) if want_dh else None     # must be overwritten
    ws = torch.empty(hb.hopgnn_sage_bwd_ws_bytes(torch.float32, n_dst, d_in, d_out, want_dh), dtype=torch.uint8,
                     device=DEV)
    ws.fill_(0x5A)
    hb.hopgnn_sage_bwd(t(H), n_src, t(self_idx), t(indptr), t(idx), n_dst, t(Ws), t(Wn), t(out_fwd), relu, t(dOut),
                       gWs, gWn, gb, dH, ws)
    torch.cuda.synchronize()
    return gWs, gWn, gb, dH


@pytest.mark.parametrize("shape", [(300, 200, 32, 32, 6), (1500, 1111, 128, 128, 12), (4000, 777, 100, 256, 16),
                                   (500, 129, 20, 12, 5), (300, 65, 7, 5, 4), (3000, 9000, 64, 128, 3)])
def test_sage_bwd_vs_oracle(hb, orc, shape):
    n_src, n_dst, d_in, d_out, max_len = shape
    rng = np.random.default_rng(n_src * 7 + d_in)
    f = lambda *s: rng.standard_normal(s).astype(np.float32)
    H = f(n_src, d_in)
    Ws = f(d_in, d_out) / np.float32(np.sqrt(d_in))
    Wn = f(d_in, d_out) / np.float32(np.sqrt(d_in))
    dOut = f(n_dst, d_out)
    indptr, idx = _rand_csr(rng, n_dst, n_src, max_len)
    self_idx = rng.integers(0, n_src, size=n_dst).astype(np.int32)
    self_idx[rng.random(n_dst) < 0.05] = -1
    out_fwd = orc.round_store(orc.sage_fwd(H, F32, self_idx, indptr, idx, Ws, Wn, None, True), F32)
    for relu, want_dh, use_bias in [(True, True, True), (False, False, False)]:
        ref = orc.sage_bwd(H, F32, self_idx, indptr, idx, Ws, Wn, out_fwd if relu else None, relu,
                           dOut.astype(np.float64), want_dH=want_dh)
        gWs, gWn, gb, dH = _run_gpu(hb, H, self_idx, indptr, idx, Ws, Wn, out_fwd if relu else None, relu, dOut,
                                    want_dh, use_bias)
        assert rel_err(to_f64(gWs), ref[0]) <= 2e-5, (shape, relu)
        assert rel_err(to_f64(gWn), ref[1]) <= 2e-5, (shape, relu)
        if use_bias:
            assert rel_err(to_f64(gb), ref[2]) <= 2e-5
        if want_dh:
            assert rel_err(to_f64(dH), ref[3]) <= 2e-5
        if relu:
            unfused = (gWs, gWn, gb)
    # accumulation in place: a second call adds the same amount again, bit for bit
    g1 = _run_gpu(hb, H, self_idx, indptr, idx, Ws, Wn, out_fwd, True, dOut, False, True)
    # without an input gradient the ReLU mask is applied inside the weight-gradient kernel: same bits
    for a, b in zip(g1[:3], unfused):
        assert torch.equal(a, b)
    g2 = _run_gpu(hb, H, self_idx, indptr, idx, Ws, Wn, out_fwd, True, dOut, False, True, acc_init=g1[:3])
    for a, b in zip(g1[:3], g2[:3]):
        assert torch.equal(b, a + a)
    # weight gradients are bit-stable from run to run
    g3 = _run_gpu(hb, H, self_idx, indptr, idx, Ws, Wn, out_fwd, True, dOut, False, True)
    for a, b in zip(g1[:3], g3[:3]):
        assert torch.equal(a, b)


def test_backward_chain_on_a_sampled_batch(hb, orc):
    """Two layers of config 1: forward on the GPU, then backward from a given output gradient,
    layer 2 then layer 1; gradients against the oracle, layer by layer from the same inputs."""
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import HotPath
    cfg = synth.CONFIGS[1]
    g = cfg.make_graph(device=DEV)
    X = cfg.make_features(device=DEV)
    W = cfg.make_weights(device=DEV)
    hp = HotPath(g.offsets, g.indices, X, W, cfg.batch, cfg.fanouts)
    seeds = synth.seeds(cfg.n_vertices, cfg.batch, 5, device=DEV)
    hp.run_batch(seeds, 5)
    torch.cuda.synchronize()
    sh = hp.shape
    B, L = sh.n_seeds, sh.n_layers
    U = int(hp.n_uniq.item())
    ids = hp.ids.cpu().numpy()
    remap = hp.remap.cpu().numpy()
    indptr = hp.indptr.cpu().numpy()
    slot_idx = hp.slot_idx[0].cpu().numpy()
    rng = np.random.default_rng(0)
    dOut2 = rng.standard_normal((B, cfg.hidden)).astype(np.float32)
    # layer 2 (last, no ReLU): input H1 (slot rows), identity self, idx = slot_idx
    n_dst2, nnz2 = sh.n_dst(2), sh.nnz(2)
    H1 = hp.H[0]
    n_src2 = sh.n_dst(1)
    g2 = _run_gpu(hb, H1.cpu().numpy(), None, indptr[:n_dst2 + 1], slot_idx[:nnz2], W[1][0].cpu().numpy(),
                  W[1][1].cpu().numpy(), None, False, dOut2, True, False)
    ref2 = orc.sage_bwd(to_bits(H1), F32, None, indptr[:n_dst2 + 1], slot_idx[:nnz2], to_bits(W[1][0]),
                        to_bits(W[1][1]), None, False, dOut2.astype(np.float64))
    assert rel_err(to_f64(g2[0]), ref2[0]) <= 2e-5 and rel_err(to_f64(g2[1]), ref2[1]) <= 2e-5
    assert rel_err(to_f64(g2[3]), ref2[3]) <= 2e-5
    # every source slot has at most one parent and one self term: dH1 is bit-stable
    g2b = _run_gpu(hb, H1.cpu().numpy(), None, indptr[:n_dst2 + 1], slot_idx[:nnz2], W[1][0].cpu().numpy(),
                   W[1][1].cpu().numpy(), None, False, dOut2, True, False)
    assert torch.equal(g2[3], g2b[3])
    # layer 1 (ReLU): input Xu through remap; the feature gradient is not needed
    n_dst1, nnz1 = sh.n_dst(1), sh.nnz(1)
    dH1 = g2[3].cpu().numpy()
    Xu = hp.Xu[:U]
    g1 = _run_gpu(hb, Xu.cpu().numpy(), remap[:n_dst1], indptr[:n_dst1 + 1], remap[B:B + nnz1],
                  W[0][0].cpu().numpy(), W[0][1].cpu().numpy(), H1.cpu().numpy(), True, dH1, False, False)
    ref1 = orc.sage_bwd(to_bits(Xu), F32, remap[:n_dst1], indptr[:n_dst1 + 1], remap[B:B + nnz1],
                        to_bits(W[0][0]), to_bits(W[0][1]), to_bits(H1), True, dH1.astype(np.float64), want_dH=False)
    assert rel_err(to_f64(g1[0]), ref1[0]) <= 2e-5 and rel_err(to_f64(g1[1]), ref1[1]) <= 2e-5


@pytest.mark.parametrize("dt", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("shape", [(1500, 1111, 128, 128, 12), (4000, 777, 100, 256, 16), (300, 65, 7, 5, 4),
                                   (6000, 5000, 136, 132, 9), (700, 2100, 512, 64, 5), (900, 300, 8, 260, 3)])
def test_sage_bwd_two_byte_activations_vs_oracle(hb, orc, dt, shape):
    """bf16 / fp16 rows, weights and stored forward output; fp32 gradients in and out.  The shapes
    cover both routes of the contractions: the 2-byte matrix instructions (feature widths that are
    multiples of 8: several tiles each way with ragged last ones, row splits that do not fill the
    last group of eight, a ragged last chunk) and the fp32 ones (any width)."""
    from helpers import GRAD_TOL, GRAD_TOL_SAME, ORC_DT, TOL, round_like
    n_src, n_dst, d_in, d_out, max_len = shape
    rng = np.random.default_rng(n_src * 11 + d_in)
    f = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float32))
    H = f(n_src, d_in).to(dt).to(DEV)
    Ws = (f(d_in, d_out) / np.sqrt(d_in)).to(dt).to(DEV)
    Wn = (f(d_in, d_out) / np.sqrt(d_in)).to(dt).to(DEV)
    dOut = rng.standard_normal((n_dst, d_out)).astype(np.float32)
    indptr, idx = _rand_csr(rng, n_dst, n_src, max_len)
    self_idx = rng.integers(0, n_src, size=n_dst).astype(np.int32)
    self_idx[rng.random(n_dst) < 0.05] = -1
    odt = ORC_DT[dt]
    Hb, Wsb, Wnb = to_bits(H), to_bits(Ws), to_bits(Wn)
    out_bits = orc.round_store(orc.sage_fwd(Hb, odt, self_idx, indptr, idx, Wsb, Wnb, None, True), odt)
    out_fwd = torch.from_numpy(out_bits.view(np.int16)).view(dt).to(DEV)
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    for relu, want_dh, use_bias in [(True, True, True), (False, False, False)]:
        ref = orc.sage_bwd(Hb, odt, self_idx, indptr, idx, Wsb, Wnb, out_bits if relu else None, relu,
                           dOut.astype(np.float64), want_dH=want_dh)
        gWs = torch.zeros((d_in, d_out), device=DEV)
        gWn = torch.zeros((d_in, d_out), device=DEV)
        gb = torch.zeros(d_out, device=DEV) if use_bias else None
        dH = torch.full((n_src, d_in), 7.0, device=DEV) if want_dh else None
        ws = torch.empty(hb.hopgnn_sage_bwd_ws_bytes(dt, n_dst, d_in, d_out, want_dh), dtype=torch.uint8, device=DEV)
        ws.fill_(0x5A)
        hb.hopgnn_sage_bwd(H, n_src, t(self_idx), t(indptr), t(idx), n_dst, Ws, Wn, out_fwd if relu else None, relu,
                           t(dOut), gWs, gWn, gb, dH, ws)
        torch.cuda.synchronize()
        # the contractions take the incoming gradient rounded to the activation type (products of two
        # 2-byte values, fp32 sums): against the oracle fed the gradient rounded the same way only the
        # summation order is left (and the rounding of the mean, where it is an operand); against the
        # oracle fed the unrounded gradient, the bound derived for that rounding.  Widths that are not
        # multiples of 8 keep fp32 products in the weight gradient.  The bias gradient sums fp32 values.
        same = orc.sage_bwd(Hb, odt, self_idx, indptr, idx, Wsb, Wnb, out_bits if relu else None, relu,
                            round_like(dOut, dt), want_dH=want_dh)
        w_ref = same if d_in % 8 == 0 and d_out % 4 == 0 else ref
        assert rel_err(to_f64(gWs), w_ref[0]) <= GRAD_TOL_SAME, (shape, relu)
        assert rel_err(to_f64(gWn), w_ref[1]) <= TOL[dt], (shape, relu)
        assert rel_err(to_f64(gWs), ref[0]) <= GRAD_TOL[dt] and rel_err(to_f64(gWn), ref[1]) <= GRAD_TOL[dt]
        if use_bias:
            assert rel_err(to_f64(gb), ref[2]) <= 2e-5
        if want_dh:
            assert rel_err(to_f64(dH), same[3]) <= GRAD_TOL_SAME
            assert rel_err(to_f64(dH), ref[3]) <= GRAD_TOL[dt]
        if relu:    # the same call without an input gradient masks inside the weight-gradient kernel: same bits
            g2 = [torch.zeros_like(gWs), torch.zeros_like(gWn), torch.zeros(d_out, device=DEV)]
            hb.hopgnn_sage_bwd(H, n_src, t(self_idx), t(indptr), t(idx), n_dst, Ws, Wn, out_fwd, True, t(dOut), g2[0],
                               g2[1], g2[2], None, ws)
            torch.cuda.synchronize()
            assert torch.equal(g2[0], gWs) and torch.equal(g2[1], gWn) and torch.equal(g2[2], gb)


def test_sage_bwd_rejects_identity_self_without_rows(hb):
    H = torch.zeros((4, 8), device=DEV)
    W = torch.zeros((8, 8), device=DEV)
    z = torch.zeros((8, 8), device=DEV)
    ip = torch.zeros(7, dtype=torch.int32, device=DEV)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    with pytest.raises(hb.HopgnnError):     # 6 destination rows with identity self, but only 4 source rows
        hb.hopgnn_sage_bwd(H, 4, None, ip, ip, 6, W, W, None, False, torch.zeros((6, 8), device=DEV), z, z, None,
                           None, ws)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16, torch.float16])
def test_sgd_update_vs_oracle(hb, orc, dt):
    from helpers import ORC_DT
    rng = np.random.default_rng(5)
    for n in (1, 7, 1000, 100_003):
        W = torch.from_numpy(rng.standard_normal(n).astype(np.float32)).to(dt).to(DEV)
        g = torch.from_numpy(rng.standard_normal(n).astype(np.float32)).to(DEV)
        ref = orc.sgd_update(to_bits(W), ORC_DT[dt], g.cpu().numpy(), 0.05)
        hb.hopgnn_sgd_update(W, g, 0.05, True)
        torch.cuda.synchronize()
        got = to_f64(W)
        want = orc.load_f64(ref, ORC_DT[dt])
        # fp32 arithmetic against fp64, then one rounding: within a place or so of the stored
        # type at the size of the operands (W and lr*g are O(1); their difference may be tiny)
        if dt == torch.float32:
            assert np.max(np.abs(got - want)) <= 1e-6
        else:
            assert np.max(np.abs(got - want) / np.maximum(np.abs(want), 0.05)) <= 2.0 ** -7
        assert float(g.abs().max().item()) == 0.0
    W0 = torch.ones(33, dtype=dt, device=DEV)
    hb.hopgnn_sgd_update(W0, torch.ones(33, device=DEV), 0.25, False)
    torch.cuda.synchronize()
    assert torch.equal(W0, torch.full((33,), 0.75, dtype=dt, device=DEV))


def test_training_iterations_lower_the_loss(hb):
    """Forward, backward with accumulation over two batches, one SGD update per iteration: the loss
    1/2 |H_L|^2 of a fixed pair of batches falls from iteration to iteration."""
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import HotPath
    cfg = synth.CONFIGS[1]
    g = cfg.make_graph(device=DEV)
    X = cfg.make_features(device=DEV)
    W = cfg.make_weights(device=DEV)
    hp = HotPath(g.offsets, g.indices, X, W, cfg.batch, cfg.fanouts)
    hp.enable_backward()
    batches = [(synth.seeds(cfg.n_vertices, cfg.batch, s, device=DEV), s) for s in (3, 4)]
    losses = []
    for it in range(6):
        loss = 0.0
        for seeds, key in batches:            # gradients of both batches accumulate in place
            out = hp.run_batch(seeds, key)
            loss += 0.5 * float((out.double() ** 2).sum().item())
            hp.backward(0)
        losses.append(loss)
        hp.apply_sgd(3e-4)
        torch.cuda.synchronize()
        assert all(float(gw.abs().max().item()) == 0.0 for gw in hp.gW[0][:2])
    assert all(b < a for a, b in zip(losses, losses[1:])), losses
    assert losses[-1] < 0.8 * losses[0], losses


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("case", range(6))
def test_slot_order_backward_equals_the_general_call(hb, orc, dt, case):
    """Neighbour lists in slot order (entry e is source row first + e, or -1): the atomic-free pull
    gives the general call's gradients bit for bit (every row has at most two contributions there,
    so the general call is exact too), and the oracle's within tolerance."""
    rng = np.random.default_rng(50 + case)
    n_dst = [1, 7, 64, 300, 300, 1000][case]
    first = [0, 3, 64, 0, 120, 1000][case]            # 0: every row can be a child; n_dst: none is
    d_in, d_out = [(4, 4), (12, 20), (32, 32), (100, 64), (33, 7), (16, 128)][case]
    lens = rng.integers(0, 6, size=n_dst)
    if case == 1:
        lens[:] = 0                                   # no entries at all
    indptr = np.zeros(n_dst + 1, np.int32)
    indptr[1:] = np.cumsum(lens)
    nnz = int(indptr[-1])
    n_src = max(first + nnz, n_dst) + [0, 5, 0, 17, 1, 0][case]     # some rows past the last entry
    idx = (first + np.arange(nnz)).astype(np.int32)
    idx[rng.random(nnz) < 0.2] = -1
    f32 = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float32)).to(DEV)
    H, Ws, Wn = f32(n_src, d_in).to(dt), (f32(d_in, d_out) / 3).to(dt), (f32(d_in, d_out) / 3).to(dt)
    out_fwd, dOut = f32(n_dst, d_out).to(dt), f32(n_dst, d_out)
    ip, ix = torch.from_numpy(indptr).to(DEV), torch.from_numpy(idx if nnz else np.zeros(1, np.int32)).to(DEV)

    def run(slots):
        g = [torch.zeros((d_in, d_out), device=DEV), torch.zeros((d_in, d_out), device=DEV), torch.zeros(d_out, device=DEV)]
        dH = torch.full((n_src, d_in), float("nan"), device=DEV)
        ws = torch.empty(hb.hopgnn_sage_bwd_ws_bytes(dt, n_dst, d_in, d_out, True), dtype=torch.uint8, device=DEV)
        ws.fill_(0xFF)
        if slots:
            hb.hopgnn_sage_bwd_slots(H, n_src, ip, ix, n_dst, first, Ws, Wn, out_fwd, True, dOut, g[0], g[1], g[2], dH, ws)
        else:
            hb.hopgnn_sage_bwd(H, n_src, None, ip, ix, n_dst, Ws, Wn, out_fwd, True, dOut, g[0], g[1], g[2], dH, ws)
        torch.cuda.synchronize()
        return g + [dH]
    a, b, a2 = run(True), run(False), run(True)
    for x, y, z in zip(a, b, a2):
        assert torch.equal(x, y) and torch.equal(x, z)
    ref = orc.sage_bwd(to_bits(H), ORC_DT[dt], None, indptr, idx, to_bits(Ws), to_bits(Wn), to_bits(out_fwd), True,
                       dOut.cpu().numpy().astype(np.float64))
    tol = 2e-5 if dt == torch.float32 else 2e-2
    assert rel_err(to_f64(a[3]), ref[3]) <= tol
    assert rel_err(to_f64(a[0]), ref[0]) <= tol and rel_err(to_f64(a[1]), ref[1]) <= tol


def test_slot_order_backward_argument_errors(hb):
    one = torch.zeros(64, device=DEV)
    i32 = torch.zeros(8, dtype=torch.int32, device=DEV)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    W = torch.zeros((4, 4), device=DEV)
    for first in (-1, 5):
        with pytest.raises(hb.HopgnnError):
            hb.hopgnn_sage_bwd_slots(one.view(16, 4), 16, i32, i32, 4, first, W, W, None, False, one.view(16, 4)[:4],
                                     W.clone(), W.clone(), None, torch.zeros((16, 4), device=DEV), ws)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16, torch.float16])
def test_sgd_update_multi_equals_one_call_per_tensor(hb, dt):
    rng = np.random.default_rng(8)
    sizes = [1, 1023, 1024, 1025, 4096 * 3 + 5, 100 * 256, 7]
    Ws = [torch.from_numpy(rng.standard_normal(n).astype(np.float32)).to(DEV).to(dt) for n in sizes]
    gs = [torch.from_numpy(rng.standard_normal(n).astype(np.float32)).to(DEV) for n in sizes]
    W1, g1 = [w.clone() for w in Ws], [g.clone() for g in gs]
    for w, g in zip(W1, g1):
        hb.hopgnn_sgd_update(w, g, 0.05, True)
    W2, g2 = [w.clone() for w in Ws], [g.clone() for g in gs]
    hb.SgdTensors(list(zip(W2, g2)) + [(None, None)]).update(0.05, True)
    W3, g3 = [w.clone() for w in Ws], [g.clone() for g in gs]
    hb.SgdTensors(list(zip(W3, g3))).update(0.05, False)
    torch.cuda.synchronize()
    for a, b, c, ga, gb, gc, g0 in zip(W1, W2, W3, g1, g2, g3, gs):
        assert torch.equal(a, b) and torch.equal(a, c)
        assert float(ga.abs().max()) == 0.0 and float(gb.abs().max()) == 0.0
        assert torch.equal(gc, g0)                                    # not cleared when not asked to


@pytest.mark.parametrize("dt", [torch.float32, torch.float16])
def test_backward_with_the_forward_calls_means(hb, dt):
    """The forward call leaves the neighbour means at the start of its workspace; handing them to
    the backward call instead of computing them again gives the same bits."""
    rng = np.random.default_rng(12)
    n_src, n_dst, d_in, d_out = 400, 250, 24, 40
    indptr, idx = _rand_csr(rng, n_dst, n_src, 6)
    self_idx = rng.integers(-1, n_src, size=n_dst).astype(np.int32)
    f32 = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float32)).to(DEV)
    H, Ws, Wn = f32(n_src, d_in).to(dt), (f32(d_in, d_out) / 4).to(dt), (f32(d_in, d_out) / 4).to(dt)
    dOut = f32(n_dst, d_out)
    ip, ix, si = (torch.from_numpy(a).to(DEV) for a in (indptr, idx, self_idx))
    out = torch.empty((n_dst, d_out), dtype=dt, device=DEV)
    ws_f = torch.empty(hb.hopgnn_sage_fwd_ws_bytes(dt, n_dst, d_in, d_out), dtype=torch.uint8, device=DEV)
    hb.hopgnn_sage_fwd(H, n_src, si, ip, ix, n_dst, Ws, Wn, None, True, out, ws_f)

    def run(mean):
        g = [torch.zeros((d_in, d_out), device=DEV), torch.zeros((d_in, d_out), device=DEV), torch.zeros(d_out, device=DEV)]
        dH = torch.empty((n_src, d_in), device=DEV)
        ws = torch.empty(hb.hopgnn_sage_bwd_ws_bytes(dt, n_dst, d_in, d_out, True), dtype=torch.uint8, device=DEV)
        ws.fill_(0xFF)
        hb.hopgnn_sage_bwd_dev(H, n_src, None, si, ip, ix, n_dst, None, Ws, Wn, out, True, dOut, g[0], g[1], g[2], dH, ws,
                               mean_fwd=mean)
        torch.cuda.synchronize()
        return g + [dH]
    a, b = run(None), run(ws_f)
    for x, y in zip(a[:3], b[:3]):
        assert torch.equal(x, y)
    assert rel_err(to_f64(a[3]), to_f64(b[3])) <= 1e-6          # float atomics: order of arrival
