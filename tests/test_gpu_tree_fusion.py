"""The single-call path with the slot tree's shape put to use (plan.fuse_tree: every projection
but the last also forms the next layer's neighbour means, the rows only those means read are
never written, layers >= 2 run no aggregation kernel) against the same call without it: the
last layer's rows must come out bit for bit the same, and so must the rows it does store.
The unfused path is the one the other tests hold against the oracle; two cases here are checked
against the oracle directly as well."""
import numpy as np
import pytest
import torch

from helpers import ORC_DT, TOL, chain_tol, rel_err, to_bits, to_f64, weights_bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

CASES = [
    # fanouts, seeds per batch, group, merge, dtype, feature dim, hidden
    ([10, 10], 300, 1, False, torch.float32, 128, 128),       # 64-row tiles, 6 groups of 10 per tile
    ([15, 10, 5], 120, 1, False, torch.float32, 100, 256),    # three layers; 128-row tiles on layer 1; 400-byte rows
    ([25, 10], 500, 1, False, torch.bfloat16, 256, 256),      # 256-row tiles: 10 groups of 25
    ([10, 10, 10], 64, 4, True, torch.float16, 128, 512),     # a merged group, N = 512
    ([10, 10, 10], 40, 3, False, torch.float16, 64, 64),      # batches of a group run one after the other
    ([64, 3], 50, 1, False, torch.float32, 32, 40),           # the widest group a tile can hold
    ([1, 1, 7], 90, 2, True, torch.bfloat16, 16, 24),         # groups of one
    ([7, 33, 2], 17, 1, False, torch.float32, 24, 8),         # ragged everything
    ([10, 10, 10], 300, 1, False, torch.float16, 128, 512),   # 256 x 256 tiles, two column tiles, four K tiles
    ([25, 10], 2600, 1, False, torch.bfloat16, 256, 256),     # 256 x 256 tiles, one column tile, eight K tiles
    ([10, 10], 1500, 2, True, torch.float16, 64, 256),        # 256 x 256 tiles, two K tiles, a merged group
    # enough 256 x 256 tiles (four and more per CU) for the workgroups that walk over their tiles; the
    # oracle's chain is left to the full-size tests at these sizes
    ([10, 10, 10], 1200, 1, False, torch.float16, 128, 512),  # four K tiles, two column tiles
    ([25, 10], 5400, 2, True, torch.bfloat16, 256, 256),      # eight K tiles, one column tile, a merged group
    ([10, 10], 13000, 1, False, torch.float16, 64, 512),      # two K tiles: the K loop is its last step only
    ([10, 10, 10], 1200, 1, False, torch.bfloat16, 192, 512), # six K tiles, exchanged operands
]


@pytest.mark.parametrize("fan,B,G,merge,dt,d,hidden", CASES)
def test_fused_tree_layers_give_the_unfused_bits(orc, fan, B, G, merge, dt, d, hidden):
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import HotPath
    g = synth.rmat_graph(13, 9.0, seed=11, device=DEV)        # 42 % of the vertices have no neighbours
    n, L = g.n_vertices, len(fan)
    X = synth.features(n, d, dt, device=DEV)
    W = synth.sage_weights(d, hidden, L, dt, device=DEV, bias=True)
    fused = HotPath(g.offsets, g.indices, X, W, B, fan, group=G, merge=merge, fuse_tree=True)
    plain = HotPath(g.offsets, g.indices, X, W, B, fan, group=G, merge=merge, fuse_tree=False)
    assert fused.fused and not plain.fused
    for it in range(2):
        seeds = synth.seeds(n, B * G, 300 + it, device=DEV)
        keys = [17 * it + b for b in range(G)]
        out_f = torch.full((G * B, hidden), float("nan"), dtype=dt, device=DEV)
        out_p = torch.full((G * B, hidden), float("nan"), dtype=dt, device=DEV)
        for h in fused.H:
            h.fill_(float("nan"))
        fused.forward(seeds, keys, out_f)
        plain.forward(seeds, keys, out_p)
        torch.cuda.synchronize()
        assert not torch.isnan(out_f.float()).any()
        assert to_bits(out_f).tobytes() == to_bits(out_p).tobytes()
        assert torch.equal(fused.ids, plain.ids) and torch.equal(fused.remap, plain.remap)
        # the rows a layer stores are the next layer's destinations: the same bits as without the flag
        # (with batches run one after the other the buffers hold the group's last batch on both sides)
        sh = fused.shape
        for k in range(1, L):
            keep = sh.n_dst(k + 1)
            assert to_bits(fused.H[k - 1][:keep]).tobytes() == to_bits(plain.H[k - 1][:keep]).tobytes(), k
            assert torch.isnan(fused.H[k - 1][keep:].float()).all()      # and nothing else is written
    if B * G * int(np.prod(fan)) > 1_000_000:
        return
    # against the oracle's own chain (first batch of the last group run)
    off_np, idx_np = g.offsets.cpu().numpy(), g.indices.cpu().numpy()
    ref_ids = [orc.sample(off_np, idx_np, seeds[b * B:(b + 1) * B].cpu().numpy(), fan, keys[b]) for b in range(G)]
    ru, rr = orc.pregather(np.concatenate([i for i, _ in ref_ids]))
    Xu_ref = orc.gather(to_bits(X), ru)
    T = len(ref_ids[0][0])
    outs = orc.forward(Xu_ref, ORC_DT[dt], ref_ids[0][0], ref_ids[0][1], rr[:T], B, fan, weights_bits(W))
    assert rel_err(to_f64(out_f[:B]), outs[-1][0]) <= chain_tol(dt, L)


def test_the_flag_is_ignored_where_the_tree_path_does_not_apply():
    """Groups of siblings wider than a tile, one layer only, widths that are no multiple of 8: the
    plan reports no scratch need and the call is the plain one."""
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import HotPath
    g = synth.rmat_graph(11, 8.0, seed=2, device=DEV)
    n = g.n_vertices
    for fan, d, hidden in (([70, 2], 16, 16), ([5], 16, 16), ([5, 5], 16, 18), ([5, 5], 10, 16)):
        X = synth.features(n, d, torch.float32, device=DEV)
        W = synth.sage_weights(d, hidden, len(fan), torch.float32, device=DEV)
        a = HotPath(g.offsets, g.indices, X, W, 30, fan, fuse_tree=True)
        b = HotPath(g.offsets, g.indices, X, W, 30, fan, fuse_tree=False)
        assert not a.fused
        seeds = synth.seeds(n, 30, 1, device=DEV)
        oa = torch.empty((30, hidden), device=DEV)
        ob = torch.empty((30, hidden), device=DEV)
        a.forward(seeds, [5], oa)
        b.forward(seeds, [5], ob)
        torch.cuda.synchronize()
        assert torch.equal(oa, ob)
