"""Whole chains at full size against the oracle's OWN chain (not isolated layers): a micrograph's
rows depend only on its root and key (the draws hash (key, root, vertex, hop, draw); nothing in a
batch couples micrographs), so for a handful of seeds of a full-size batch the oracle runs
everything itself on a mini-batch of just those seeds - sampling, pre-gather, gather of the rows it
asks for, every layer from its own rounded activations - and its root rows must equal the rows the
benchmark's single call (fused slot-tree layers, merged groups) produced for those seeds."""
import numpy as np
import pytest
import torch

from helpers import ORC_DT, chain_tol, rel_err, to_bits, to_f64, weights_bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _oracle_roots(orc, graph_np, X, wb, roots, fanouts, key):
    off_np, idx_np = graph_np
    ids, indptr = orc.sample(off_np, idx_np, np.asarray(roots, np.int64), fanouts, key)
    uniq, remap = orc.pregather(ids)
    rows = to_bits(X[torch.from_numpy(uniq).long().to(X.device)])      # input plumbing: the rows it asks for
    Xu = orc.gather(rows, np.arange(len(uniq), dtype=np.int32))
    outs = orc.forward(Xu, ORC_DT[X.dtype], ids, indptr, remap, len(roots), fanouts, wb)
    return outs[-1][0]            # last layer, unrounded float64, one row per root


@pytest.mark.timeout(900)
@pytest.mark.parametrize("cfg_id,group", [(3, 1), (4, 1), (5, 8)])
def test_root_rows_of_the_benched_call_vs_the_oracles_own_chain(orc, cfg_id, group):
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import HotPath
    cfg = synth.CONFIGS[cfg_id]
    g = cfg.make_graph(device=DEV)
    X = cfg.make_features(device=DEV)
    W = cfg.make_weights(device=DEV)
    fan, B, L = list(cfg.fanouts), cfg.batch, len(cfg.fanouts)
    hp = HotPath(g.offsets, g.indices, X, W, B, fan, group=group, merge=group > 1)      # as bench.py builds it
    assert hp.fused
    seeds = torch.cat([synth.seeds(cfg.n_vertices, B, 40 + b, device=DEV) for b in range(group)])
    keys = [900 + 7 * b for b in range(group)]
    out = torch.full((group * B, cfg.hidden), float("nan"), dtype=X.dtype, device=DEV)
    hp.forward(seeds, keys, out)
    torch.cuda.synchronize()
    graph_np = (g.offsets.cpu().numpy(), g.indices.cpu().numpy())
    wb = weights_bits(W)
    seeds_np = seeds.cpu().numpy()
    deg = graph_np[0][seeds_np + 1] - graph_np[0][seeds_np]
    rng = np.random.default_rng(cfg_id)
    n_checked = 0
    for b in sorted(set([0, group - 1, group // 2])):
        # first and last seed of the block, a few in between, and one dead micrograph if the block has one
        pos = sorted(set([0, B - 1] + [int(x) for x in rng.integers(1, B - 1, size=4)]))
        dead = np.nonzero(deg[b * B:(b + 1) * B] == 0)[0]
        if len(dead):
            pos = sorted(set(pos + [int(dead[0])]))
        want = _oracle_roots(orc, graph_np, X, wb, seeds_np[b * B + np.asarray(pos)], fan, keys[b])
        got = to_f64(out[b * B + torch.tensor(pos, device=DEV)])
        err = rel_err(got, want)
        assert err <= chain_tol(X.dtype, L), (cfg.name, b, pos, err)
        n_checked += len(pos)
    assert n_checked >= 6
