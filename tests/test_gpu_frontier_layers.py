"""GCN-style and attention layers over frontier structures (deduplicated and layer-wise sampled
micrographs) against the oracle chain, step by step and through the single-call entry point."""
import numpy as np
import pytest
import torch

from helpers import ORC_DT, TOL, rel_err, to_bits, to_f64, weights_bits, chain_tol
from oracle import dedup as orc_dedup
from oracle import frontier as orc_frontier
from oracle import layerwise as orc_lw

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("model", ["gcn", "gat"])
@pytest.mark.parametrize("sampler,fanouts", [("node", [5, 4]), ("layer", [5, 8, 10])])
def test_layer_kinds_over_frontiers(orc, dt, model, sampler, fanouts):
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import DedupPath
    g = synth.rmat_graph(12, 10.0, device=DEV)
    n, d, hidden, B, L, G = g.n_vertices, 24, 40, 30, len(fanouts), 2
    X = synth.features(n, d, dt, device=DEV)
    W = synth.sage_weights(d, hidden, L, dt, device=DEV, bias=True)
    dp = DedupPath(g.offsets, g.indices, X, W, B, fanouts, group=G, sampler=sampler, model=model)
    for t in dp.H:
        t.fill_(float("nan"))
    seeds = synth.seeds(n, B * G, 7, device=DEV)
    keys = [31, 32]
    out = dp.run_batch(seeds, keys).clone()
    torch.cuda.synchronize()
    out2 = torch.full_like(out, float("nan"))
    dp.forward(seeds, keys, out2)
    torch.cuda.synchronize()
    assert to_bits(out2).tobytes() == to_bits(out).tobytes()      # the same launches issued from C
    off_np, idx_np = g.offsets.cpu().numpy(), g.indices.cpu().numpy()
    sample = orc_dedup.sample_dedup if sampler == "node" else orc_lw.sample_layerwise
    wb = weights_bits(W)
    odt = ORC_DT[dt]

    def layer(k, H, self_idx, ip, ix, relu):
        Wk, _, bk = wb[k - 1]
        if model == "gcn":
            return orc.gcn_fwd(H, odt, self_idx, ip, ix, Wk, bk, 1, relu)
        a_s, a_d = dp.attn[k - 1]
        return orc.gat_fwd(H, odt, self_idx, ip, ix, Wk, to_bits(a_s), to_bits(a_d), bk, dp.gat_heads, relu)
    for b in range(G):
        st = sample(off_np, idx_np, seeds[b * B:(b + 1) * B].cpu().numpy(), fanouts, keys[b])
        ref = orc_frontier.layer_chain(orc, to_bits(X), odt, *st, wb, layer=layer)
        assert rel_err(to_f64(out[b * B:(b + 1) * B]), ref) <= chain_tol(dt, L), b
