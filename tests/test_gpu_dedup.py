"""GPU parity of the deduplicated-frontier sampler (bit-exact against the oracle) and of the layer
chain over it (the tree oracle's root rows)."""
import numpy as np
import pytest
import torch

from helpers import ORC_DT, TOL, rel_err, to_bits, to_f64, weights_bits, chain_tol
from oracle import dedup as orc_dedup

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def hb():
    from paper_2409_00657_amd import binding
    binding.load_library()
    return binding


def _run_sampler(hb, g, seeds, fanouts, key, seeds_per_key=0):
    B = seeds.numel()
    t_seed = hb.hopgnn_slots_per_seed(fanouts)
    T = B * t_seed
    P = 1
    for f in fanouts:
        P *= f
    S = T - B * P
    i32 = dict(dtype=torch.int32, device=DEV)
    nv = torch.full((T,), -9, **i32)
    ls = torch.full((len(fanouts) + 2,), -9, dtype=torch.int64, device=DEV)
    ip = torch.full((S + 1,), -9, **i32)
    ix = torch.full((max(T - B, 1),), -9, **i32)
    ws = torch.empty(hb.hopgnn_sample_dedup_ws_bytes(B, fanouts), dtype=torch.uint8, device=DEV)
    ws.fill_(0x5A)
    hb.hopgnn_sample_dedup(g.offsets, g.indices, seeds, fanouts, key, nv, ls, ip, ix, ws, seeds_per_key=seeds_per_key)
    torch.cuda.synchronize()
    return nv, ls, ip, ix, T, S


@pytest.mark.parametrize("case", range(6))
def test_sample_dedup_bit_exact(hb, case):
    from paper_2409_00657_amd import synth
    graphs = [lambda: synth.uniform_graph(500, 1, 6, seed=3, device=DEV),
              lambda: synth.rmat_graph(11, 8.0, seed=4, device=DEV),
              lambda: synth.chung_lu_graph(3000, 12.0, 2.1, seed=5, device=DEV, offsets_i64=True),
              lambda: synth.rmat_graph(10, 3.0, seed=6, device=DEV, offsets_i64=True),
              lambda: synth.uniform_graph(40, 1, 3, seed=7, device=DEV),
              lambda: synth.rmat_graph(12, 16.0, seed=8, device=DEV)]
    fans = [[5, 5], [10, 10], [15, 10, 5], [4, 3, 2, 2], [7], [16, 16, 16]]
    Bs = [64, 100, 33, 50, 300, 5]
    g = graphs[case]()
    fan, B = fans[case], Bs[case]
    seeds = synth.seeds(g.n_vertices, B, case, device=DEV)
    key = 1000 + case
    nv, ls, ip, ix, T, S = _run_sampler(hb, g, seeds, fan, key)
    r_nv, r_ls, r_ip, r_ix = orc_dedup.sample_dedup(g.offsets.cpu().numpy(), g.indices.cpu().numpy(),
                                                    seeds.cpu().numpy(), fan, key)
    np.testing.assert_array_equal(ls.cpu().numpy(), r_ls)
    n_nodes, n_nonleaf, nnz = len(r_nv), int(r_ls[len(fan)]), len(r_ix)
    np.testing.assert_array_equal(nv[:n_nodes].cpu().numpy(), r_nv)
    assert bool((nv[n_nodes:] == -1).all())
    np.testing.assert_array_equal(ip[:n_nonleaf + 1].cpu().numpy(), r_ip)
    assert bool((ip[n_nonleaf:] == nnz).all())
    np.testing.assert_array_equal(ix[:nnz].cpu().numpy(), r_ix)
    assert bool((ix[nnz:T - B] == -1).all())
    assert n_nodes <= T


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("fanouts", [[6, 5], [5, 4, 3]])
def test_layers_over_deduplicated_nodes_give_the_tree_rows(hb, orc, dt, fanouts):
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import DedupPath
    g = synth.rmat_graph(12, 10.0, device=DEV)
    n, d, hidden, B, L = g.n_vertices, 24, 40, 60, len(fanouts)
    X = synth.features(n, d, dt, device=DEV)
    W = synth.sage_weights(d, hidden, L, dt, device=DEV, bias=True)
    dp = DedupPath(g.offsets, g.indices, X, W, B, fanouts)
    off_np, idx_np = g.offsets.cpu().numpy(), g.indices.cpu().numpy()
    for it in range(2):
        seeds = synth.seeds(n, B, 30 + it, device=DEV)
        out = dp.run_batch(seeds, 400 + it).clone()
        torch.cuda.synchronize()
        # the same sequence from one library call: the same bits
        out2 = torch.full_like(out, float("nan"))
        dp.remap.fill_(-7)
        dp.forward(seeds, 400 + it, out2)
        torch.cuda.synchronize()
        assert to_bits(out2).tobytes() == to_bits(out).tobytes()
        # the tree oracle's rows for the same seeds and key
        ids, ip = orc.sample(off_np, idx_np, seeds.cpu().numpy(), fanouts, 400 + it)
        uniq, remap = orc.pregather(ids)
        U = int(dp.n_uniq.item())
        assert U == len(uniq)
        np.testing.assert_array_equal(dp.uniq[:U].cpu().numpy(), uniq)      # the same rows are fetched
        Xu = orc.gather(to_bits(X), uniq)
        ref = orc.forward(Xu, ORC_DT[dt], ids, ip, remap, B, fanouts, weights_bits(W))[-1][0]
        assert rel_err(to_f64(out), ref) <= chain_tol(dt, L)
        # fewer rows than slots
        n_nodes = int(dp.level_start[L + 1].item())
        assert n_nodes < dp.capacity


def test_grouped_dedup_equals_per_batch_oracle(hb, orc):
    """A group as one merged batch with a key per block of seeds: block b's nodes are those of the
    oracle's batch b, and the layer chain gives every seed the tree oracle's row."""
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import DedupPath
    g = synth.rmat_graph(12, 10.0, device=DEV)
    n, d, hidden, B, G, fan = g.n_vertices, 16, 24, 10, 70, [4, 3]
    off_np, idx_np = g.offsets.cpu().numpy(), g.indices.cpu().numpy()
    seeds = synth.seeds(n, B * G, 77, device=DEV)
    keys = [900 + 3 * b for b in range(G)]
    nv, ls, ip, ix, T, S = _run_sampler(hb, g, seeds, fan, keys, seeds_per_key=B)
    nv_np, ls_np = nv.cpu().numpy(), ls.cpu().numpy()
    # level 1 of the merged batch = level 1 of every batch in turn
    pos = int(ls_np[1])
    for b in range(G):
        r_nv, r_ls, _, _ = orc_dedup.sample_dedup(off_np, idx_np, seeds[b * B:(b + 1) * B].cpu().numpy(), fan, keys[b])
        lvl1 = r_nv[r_ls[1]:r_ls[2]]
        np.testing.assert_array_equal(nv_np[pos:pos + len(lvl1)], lvl1)
        pos += len(lvl1)
    assert pos == ls_np[2]
    X = synth.features(n, d, torch.float32, device=DEV)
    W = synth.sage_weights(d, hidden, 2, torch.float32, device=DEV)
    dp = DedupPath(g.offsets, g.indices, X, W, B, fan, group=G)
    out = torch.empty((G * B, hidden), device=DEV)
    dp.forward(seeds, keys, out)
    torch.cuda.synchronize()
    for b in (0, 1, 63, 64, 69):
        sb = seeds[b * B:(b + 1) * B].cpu().numpy()
        ids, tip = orc.sample(off_np, idx_np, sb, fan, keys[b])
        uniq, remap = orc.pregather(ids)
        ref = orc.forward(orc.gather(to_bits(X), uniq), 0, ids, tip, remap, B, fan, weights_bits(W))[-1][0]
        assert rel_err(to_f64(out[b * B:(b + 1) * B]), ref) <= 1e-5, b


def test_sample_dedup_argument_errors(hb):
    from paper_2409_00657_amd import synth
    g = synth.uniform_graph(100, 2, 4, device=DEV)
    seeds = synth.seeds(100, 4, 0, device=DEV)
    z = torch.zeros(1 << 16, dtype=torch.int32, device=DEV)
    ls = torch.zeros(8, dtype=torch.int64, device=DEV)
    ws = torch.empty(1 << 22, dtype=torch.uint8, device=DEV)
    with pytest.raises(hb.HopgnnError):          # 17^3 = 4913 slots in one micrograph's last level
        hb.hopgnn_sample_dedup(g.offsets, g.indices, seeds, [17, 17, 17], 0, z, ls, z, z, ws)
    with pytest.raises(hb.HopgnnError):          # workspace too small
        hb.hopgnn_sample_dedup(g.offsets, g.indices, seeds, [4, 4], 0, z, ls, z, z, ws[:256])
    assert hb.hopgnn_sample_dedup_ws_bytes(4, [3, 0]) == 0
