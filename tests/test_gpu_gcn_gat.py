"""GPU parity of the GCN-style and graph-attention layers against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from helpers import ORC_DT, TOL, rel_err, to_bits, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
DTYPES = [torch.float32, torch.bfloat16, torch.float16]


@pytest.fixture(scope="module")
def hb():
    from paper_2409_00657_amd import binding
    binding.load_library()
    return binding


def _case(rng, n_src, n_dst, d_in, d_out, max_len, dt, identity_self=False):
    f = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float32))
    H = f(n_src, d_in).to(dt)
    W = (f(d_in, d_out) / np.sqrt(d_in)).to(dt)
    b = f(d_out).to(dt)
    lens = rng.integers(0, max_len + 1, size=n_dst)
    indptr = np.zeros(n_dst + 1, np.int32)
    indptr[1:] = np.cumsum(lens)
    idx = rng.integers(0, n_src, size=int(indptr[-1])).astype(np.int32)
    idx[rng.random(len(idx)) < 0.15] = -1
    if identity_self:
        self_idx = None
    else:
        self_idx = rng.integers(0, n_src, size=n_dst).astype(np.int32)
        self_idx[rng.random(n_dst) < 0.05] = -1
    return H, W, b, self_idx, indptr, idx


def _dev(a):
    return None if a is None else (a.to(DEV) if isinstance(a, torch.Tensor) else torch.from_numpy(a).to(DEV))


SHAPES = [(300, 200, 32, 32, 6), (1500, 1111, 128, 128, 12), (4000, 777, 100, 256, 16), (500, 129, 20, 12, 5),
          (300, 65, 7, 5, 4), (9000, 3000, 64, 128, 3)]
# enough rows for the 128 x 128 (fp32) and 256 x 256 (2-byte) projection tiles
LARGE_GCN = (3000, 66000, 64, 256, 3)
LARGE_GAT = (66000, 2000, 64, 256, 6)
# enough source rows for fp32 attention scores to come from the skinny product
MANY_ROWS_GAT = (132000, 500, 16, 32, 4)


@pytest.mark.parametrize("dt", DTYPES)
@pytest.mark.parametrize("shape", SHAPES + [LARGE_GCN])
def test_gcn_fwd_vs_oracle(hb, orc, dt, shape):
    n_src, n_dst, d_in, d_out, max_len = shape
    rng = np.random.default_rng(n_src + 3 * d_in)
    variants = [(1, True, True, False), (0, False, False, n_src >= n_dst)]
    for norm, relu, use_bias, ident in variants[:1] if shape == LARGE_GCN else variants:
        H, W, b, self_idx, indptr, idx = _case(rng, n_src, n_dst, d_in, d_out, max_len, dt, identity_self=ident)
        ref = orc.gcn_fwd(to_bits(H), ORC_DT[dt], self_idx, indptr, idx, to_bits(W), to_bits(b) if use_bias else None,
                          norm, relu)
        out = torch.full((n_dst, d_out), float("nan"), dtype=dt, device=DEV)
        ws = torch.empty(hb.hopgnn_gcn_fwd_ws_bytes(dt, n_dst, d_in, d_out), dtype=torch.uint8, device=DEV)
        ws.fill_(0x5A)
        hb.hopgnn_gcn_fwd(_dev(H), n_src, _dev(self_idx), _dev(indptr), _dev(idx), n_dst, _dev(W),
                          _dev(b) if use_bias else None, norm, relu, out, ws)
        torch.cuda.synchronize()
        assert rel_err(to_f64(out), ref) <= TOL[dt], (shape, norm)


@pytest.mark.parametrize("dt", DTYPES)
@pytest.mark.parametrize("shape", SHAPES + [(600, 300, 40, 96, 5), LARGE_GAT, MANY_ROWS_GAT])
def test_gat_fwd_vs_oracle(hb, orc, dt, shape):
    n_src, n_dst, d_in, d_out, max_len = shape
    rng = np.random.default_rng(n_src + 5 * d_in)
    head_options = [h for h in (1, 2, 4, 8) if d_out % h == 0]
    variants = [(head_options[-1], True, True, False), (head_options[0], False, False, n_src >= n_dst)]
    if d_out == 96:     # three heads of 32: rows of 24 words, packed two to a wavefront
        variants = [(3, True, True, False)]
    for heads, relu, use_bias, ident in variants[1:] if shape == LARGE_GAT else variants:
        H, W, b, self_idx, indptr, idx = _case(rng, n_src, n_dst, d_in, d_out, max_len, dt, identity_self=ident)
        f = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float32))
        a_src = (f(d_out) / np.sqrt(d_out // heads)).to(dt)
        a_dst = (f(d_out) / np.sqrt(d_out // heads)).to(dt)
        ref = orc.gat_fwd(to_bits(H), ORC_DT[dt], self_idx, indptr, idx, to_bits(W), to_bits(a_src), to_bits(a_dst),
                          to_bits(b) if use_bias else None, heads, relu)
        out = torch.full((n_dst, d_out), float("nan"), dtype=dt, device=DEV)
        ws = torch.empty(hb.hopgnn_gat_fwd_ws_bytes(dt, n_src, d_in, d_out, heads), dtype=torch.uint8, device=DEV)
        ws.fill_(0x5A)
        hb.hopgnn_gat_fwd(_dev(H), n_src, _dev(self_idx), _dev(indptr), _dev(idx), n_dst, _dev(W), _dev(a_src),
                          _dev(a_dst), _dev(b) if use_bias else None, heads, relu, out, ws)
        torch.cuda.synchronize()
        assert rel_err(to_f64(out), ref) <= TOL[dt], (shape, heads)


@pytest.mark.parametrize("dt", DTYPES)
@pytest.mark.parametrize("agg", [1, 2])
@pytest.mark.parametrize("shape", [(300, 200, 32, 32, 6), (1500, 1111, 128, 128, 12), (300, 65, 7, 5, 4)])
def test_sage_sum_and_max_aggregators_vs_oracle(hb, orc, dt, agg, shape):
    n_src, n_dst, d_in, d_out, max_len = shape
    rng = np.random.default_rng(n_src + 13 * agg)
    H, W, b, self_idx, indptr, idx = _case(rng, n_src, n_dst, d_in, d_out, max_len, dt)
    W2 = (torch.from_numpy(rng.standard_normal((d_in, d_out)).astype(np.float32)) / np.sqrt(d_in)).to(dt)
    if agg == 2:      # all-negative rows too: the maximum must not start from zero
        H = (-H.float().abs() - 0.5).to(dt) if n_src == 300 else H
    ref = orc.sage_agg_fwd(to_bits(H), ORC_DT[dt], self_idx, indptr, idx, to_bits(W), to_bits(W2), to_bits(b), agg, True)
    out = torch.full((n_dst, d_out), float("nan"), dtype=dt, device=DEV)
    ws = torch.empty(hb.hopgnn_sage_fwd_ws_bytes(dt, n_dst, d_in, d_out), dtype=torch.uint8, device=DEV)
    ws.fill_(0x5A)
    hb.hopgnn_sage_fwd_agg(_dev(H), n_src, _dev(self_idx), _dev(indptr), _dev(idx), n_dst, _dev(W), _dev(W2), _dev(b),
                           agg, True, out, ws)
    torch.cuda.synchronize()
    assert rel_err(to_f64(out), ref) <= TOL[dt], (shape, agg)


def test_layers_on_a_sampled_batch(hb, orc):
    """Config 1, first layer over the pre-gathered rows (self and neighbours through remap): the
    attention layer projects each UNIQUE row once."""
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import HotPath
    cfg = synth.CONFIGS[1]
    g = cfg.make_graph(device=DEV)
    X = cfg.make_features(device=DEV)
    W = cfg.make_weights(device=DEV)
    hp = HotPath(g.offsets, g.indices, X, W, cfg.batch, cfg.fanouts)
    seeds = synth.seeds(cfg.n_vertices, cfg.batch, 9, device=DEV)
    hp.sample(0, seeds, 9)
    hp.pregather()
    hp.gather()
    torch.cuda.synchronize()
    sh = hp.shape
    B, U = sh.n_seeds, int(hp.n_uniq.item())
    n_dst, nnz = sh.n_dst(1), sh.nnz(1)
    remap = hp.remap.cpu().numpy()
    indptr = hp.indptr.cpu().numpy()[:n_dst + 1]
    Xu = hp.Xu[:U]
    W1 = W[0][0]
    d_in, d_out = W1.shape
    rng = np.random.default_rng(4)
    a_src = torch.from_numpy(rng.standard_normal(d_out).astype(np.float32)).to(DEV)
    a_dst = torch.from_numpy(rng.standard_normal(d_out).astype(np.float32)).to(DEV)
    out = torch.empty((n_dst, d_out), device=DEV)
    ws = torch.empty(max(hb.hopgnn_gat_fwd_ws_bytes(torch.float32, hp.cap, d_in, d_out, 4),
                         hb.hopgnn_gcn_fwd_ws_bytes(torch.float32, n_dst, d_in, d_out)), dtype=torch.uint8, device=DEV)
    # the whole pre-gather buffer with its row count left on the device, as the pipeline passes it
    hp.Xu[U:].fill_(float("nan"))
    hb.hopgnn_gat_fwd(hp.Xu, hp.cap, hp.remap[:n_dst], hp.indptr[:n_dst + 1], hp.remap[B:B + nnz], n_dst, W1, a_src,
                      a_dst, None, 4, True, out, ws, n_src_dev=hp.n_uniq)
    torch.cuda.synchronize()
    ref = orc.gat_fwd(to_bits(Xu), 0, remap[:n_dst], indptr, remap[B:B + nnz], to_bits(W1), to_bits(a_src),
                      to_bits(a_dst), None, 4, True)
    assert rel_err(to_f64(out), ref) <= 1e-5
    hb.hopgnn_gcn_fwd(Xu, U, hp.remap[:n_dst], hp.indptr[:n_dst + 1], hp.remap[B:B + nnz], n_dst, W1, None, 1, True,
                      out, ws)
    torch.cuda.synchronize()
    ref = orc.gcn_fwd(to_bits(Xu), 0, remap[:n_dst], indptr, remap[B:B + nnz], to_bits(W1), None, 1, True)
    assert rel_err(to_f64(out), ref) <= 1e-5


def test_layer_argument_errors(hb):
    H = torch.zeros((4, 8), device=DEV)
    W = torch.zeros((8, 8), device=DEV)
    ip = torch.zeros(5, dtype=torch.int32, device=DEV)
    out = torch.zeros((4, 8), device=DEV)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    with pytest.raises(hb.HopgnnError):          # norm must be 0 or 1
        hb.hopgnn_gcn_fwd(H, 4, None, ip, ip, 4, W, None, 2, False, out, ws)
    with pytest.raises(hb.HopgnnError):          # heads must divide d_out
        hb.hopgnn_gat_fwd(H, 4, None, ip, ip, 4, W, W[0], W[0], None, 3, False, out, ws)
    with pytest.raises(hb.HopgnnError):          # workspace too small
        hb.hopgnn_gat_fwd(H, 4, None, ip, ip, 4, W, W[0], W[0], None, 2, False, out, ws[:256])
    assert hb.hopgnn_gat_fwd_ws_bytes(torch.float32, 4, 8, 8, 3) == 0


@pytest.mark.parametrize("model", ["gcn", "gat"])
@pytest.mark.parametrize("merge", [False, True])
def test_layer_kinds_through_the_single_call_path(hb, orc, model, merge):
    """hopgnn_batch_fwd with GCN-style / attention layers: the same bits as the step-by-step
    sequence, and the last layer's rows against the oracle's chain of that layer type."""
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import HotPath
    cfg = synth.CONFIGS[1]
    g = cfg.make_graph(device=DEV)
    X = cfg.make_features(device=DEV)
    W = cfg.make_weights(device=DEV)
    G, B, L = 3, cfg.batch, len(cfg.fanouts)
    hp = HotPath(g.offsets, g.indices, X, W, B, cfg.fanouts, group=G, model=model, merge=merge)
    seeds = synth.seeds(cfg.n_vertices, B * G, 21, device=DEV)
    keys = [5, 6, 7]
    out = torch.full((G * B, cfg.hidden), float("nan"), device=DEV)
    hp.forward(seeds, keys, out)
    torch.cuda.synchronize()
    outs2 = [torch.empty((B, cfg.hidden), device=DEV) for _ in range(G)]
    hp.run_group([seeds[b * B:(b + 1) * B] for b in range(G)], keys, outs2)
    torch.cuda.synchronize()
    assert torch.equal(torch.cat(outs2), out)
    # oracle: per batch, chain the layer type over the batch's own slot arrays
    off_np, idx_np = g.offsets.cpu().numpy(), g.indices.cpu().numpy()
    ref_ids = [orc.sample(off_np, idx_np, seeds[b * B:(b + 1) * B].cpu().numpy(), cfg.fanouts, keys[b]) for b in range(G)]
    ru, rr = orc.pregather(np.concatenate([i for i, _ in ref_ids]))
    Xu = orc.gather(to_bits(X), ru)
    T = len(ref_ids[0][0])
    from paper_2409_00657_amd.pipeline import BatchShape
    shb = BatchShape(B, list(cfg.fanouts))
    for b in range(G):
        ids_b, ip = ref_ids[b]
        remap_b = rr[b * T:(b + 1) * T]
        H = Xu
        for k in range(1, L + 1):
            n_dst, nnz = shb.n_dst(k), shb.nnz(k)
            if k == 1:
                self_idx, idx = remap_b[:n_dst], remap_b[B:B + nnz]
            else:
                e = np.arange(nnz, dtype=np.int32)
                self_idx, idx = None, np.where(ids_b[B:B + nnz] >= 0, B + e, -1).astype(np.int32)
            Wk = to_bits(W[k - 1][0])
            if model == "gcn":
                o = orc.gcn_fwd(H, 0, self_idx, ip[:n_dst + 1], idx, Wk, None, 1, k < L)
            else:
                a_s, a_d = hp.attn[k - 1]
                o = orc.gat_fwd(H, 0, self_idx, ip[:n_dst + 1], idx, Wk, to_bits(a_s), to_bits(a_d), None, hp.gat_heads,
                                k < L)
            H = orc.round_store(o, 0)
        assert rel_err(to_f64(out[b * B:(b + 1) * B]), o) <= 1e-5, (model, merge, b)
