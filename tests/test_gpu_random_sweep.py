"""Seeded random sweeps (valid inputs only) of the layer entry points and of whole batches
against the oracle: odd widths, one-row inputs, empty segments, all-invalid self rows, every
dtype, every pre-gather algorithm, groups, one to four hops."""
import numpy as np
import pytest
import torch

import oracle as orc
from helpers import ORC_DT, TOL, rel_err, to_bits, to_f64, weights_bits, chain_tol

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(a):
    return None if a is None else (a.to(DEV) if isinstance(a, torch.Tensor)
                                   else torch.from_numpy(np.ascontiguousarray(a)).to(DEV))


@pytest.mark.parametrize("seed", [1, 2])
def test_random_layer_shapes(seed):
    from paper_2409_00657_amd import binding as hb
    hb.load_library()
    rng = np.random.default_rng(seed)
    N_CASES = 40
    dts = [torch.float32, torch.bfloat16, torch.float16]
    dev = _dev
    failures = []
    for case in range(N_CASES):
        dt = dts[rng.integers(0, 3)]
        n_src = int(rng.choice([1, 2, 5, 33, 64, 65, 200, 1000, 5000]))
        n_dst = int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 257, 700, 3000]))
        d_in = int(rng.choice([1, 2, 3, 4, 7, 8, 12, 16, 31, 32, 33, 60, 64, 100, 128, 130, 200, 256, 300]))
        d_out = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 24, 32, 40, 64, 65, 96, 128, 129, 200, 256, 320]))
        max_len = int(rng.choice([0, 1, 2, 5, 9, 30]))
        ident = bool(rng.integers(0, 2)) and n_src >= n_dst
        f = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float32))
        H = f(n_src, d_in).to(dt); Ws = (f(d_in, d_out) / np.sqrt(d_in)).to(dt); Wn = (f(d_in, d_out) / np.sqrt(d_in)).to(dt)
        b = f(d_out).to(dt) if rng.integers(0, 2) else None
        lens = rng.integers(0, max_len + 1, size=n_dst)
        indptr = np.zeros(n_dst + 1, np.int32); indptr[1:] = np.cumsum(lens)
        idx = rng.integers(0, n_src, size=int(indptr[-1])).astype(np.int32)
        idx[rng.random(len(idx)) < rng.choice([0.0, 0.2, 0.9])] = -1
        self_idx = None if ident else rng.integers(0, n_src, size=n_dst).astype(np.int32)
        if self_idx is not None: self_idx[rng.random(n_dst) < rng.choice([0.0, 0.1, 1.0])] = -1
        relu = bool(rng.integers(0, 2))
        odt = ORC_DT[dt]
        Hb, Wsb, Wnb, bb = to_bits(H), to_bits(Ws), to_bits(Wn), (None if b is None else to_bits(b))
        tag = (case, str(dt), n_src, n_dst, d_in, d_out, max_len, ident, relu, b is not None)
        def check(name, got, ref, tol):
            e = rel_err(to_f64(got), ref)
            if not (e <= tol):
                failures.append((name, e, tag))
        out = torch.full((n_dst, d_out), float("nan"), dtype=dt, device=DEV)
        ws = torch.empty(max(hb.hopgnn_sage_fwd_ws_bytes(dt, n_dst, d_in, d_out), 256), dtype=torch.uint8, device=DEV); ws.fill_(0x5A)
        agg = int(rng.integers(0, 3))
        hb.hopgnn_sage_fwd_agg(dev(H), n_src, dev(self_idx), dev(indptr), dev(idx), n_dst, dev(Ws), dev(Wn), dev(b), agg, relu, out, ws)
        torch.cuda.synchronize()
        check("sage_agg%d" % agg, out, orc.sage_agg_fwd(Hb, odt, self_idx, indptr, idx, Wsb, Wnb, bb, agg, relu), TOL[dt])
        # gcn
        norm = int(rng.integers(0, 2))
        ws = torch.empty(max(hb.hopgnn_gcn_fwd_ws_bytes(dt, n_dst, d_in, d_out), 256), dtype=torch.uint8, device=DEV); ws.fill_(0x5A)
        out.fill_(float("nan"))
        hb.hopgnn_gcn_fwd(dev(H), n_src, dev(self_idx), dev(indptr), dev(idx), n_dst, dev(Ws), dev(b), norm, relu, out, ws)
        torch.cuda.synchronize()
        check("gcn%d" % norm, out, orc.gcn_fwd(Hb, odt, self_idx, indptr, idx, Wsb, bb, norm, relu), TOL[dt])
        # gat
        heads = int(rng.choice([h for h in (1, 2, 3, 4, 5, 8, 16) if d_out % h == 0]))
        a_s = (f(d_out) / np.sqrt(d_out // heads)).to(dt); a_d = (f(d_out) / np.sqrt(d_out // heads)).to(dt)
        ws = torch.empty(max(hb.hopgnn_gat_fwd_ws_bytes(dt, n_src, d_in, d_out, heads), 256), dtype=torch.uint8, device=DEV); ws.fill_(0x5A)
        out.fill_(float("nan"))
        hb.hopgnn_gat_fwd(dev(H), n_src, dev(self_idx), dev(indptr), dev(idx), n_dst, dev(Ws), dev(a_s), dev(a_d), dev(b), heads, relu, out, ws)
        torch.cuda.synchronize()
        check("gat%d" % heads, out, orc.gat_fwd(Hb, odt, self_idx, indptr, idx, Wsb, to_bits(a_s), to_bits(a_d), bb, heads, relu), TOL[dt])
        # backward
        dOut = rng.standard_normal((n_dst, d_out)).astype(np.float32)
        out_bits = orc.round_store(orc.sage_fwd(Hb, odt, self_idx, indptr, idx, Wsb, Wnb, bb, True), odt)
        out_fwd = torch.from_numpy(out_bits if dt == torch.float32 else out_bits.view(np.int16)).view(dt).to(DEV) if dt != torch.float32 else torch.from_numpy(out_bits).to(DEV)
        want_dh = bool(rng.integers(0, 2))
        ref = orc.sage_bwd(Hb, odt, self_idx, indptr, idx, Wsb, Wnb, out_bits if relu else None, relu, dOut.astype(np.float64), want_dH=want_dh)
        gWs = torch.zeros((d_in, d_out), device=DEV); gWn = torch.zeros((d_in, d_out), device=DEV); gb = torch.zeros(d_out, device=DEV)
        dH = torch.full((n_src, d_in), 7.0, device=DEV) if want_dh else None
        ws = torch.empty(max(hb.hopgnn_sage_bwd_ws_bytes(dt, n_dst, d_in, d_out, want_dh), 256), dtype=torch.uint8, device=DEV); ws.fill_(0x5A)
        hb.hopgnn_sage_bwd(dev(H), n_src, dev(self_idx), dev(indptr), dev(idx), n_dst, dev(Ws), dev(Wn), out_fwd if relu else None, relu, dev(dOut), gWs, gWn, gb, dH, ws)
        torch.cuda.synchronize()
        gtol = 3e-5 if dt == torch.float32 else TOL[dt]     # 2-byte: the contractions round dOut to the activation type
        check("gWs", gWs, ref[0], gtol); check("gWn", gWn, ref[1], gtol); check("gb", gb, ref[2], 3e-5)
        if want_dh: check("dH", dH, ref[3], gtol)
    assert not failures, failures


@pytest.mark.parametrize("seed", [1, 2])
def test_random_whole_batches(seed):
    from paper_2409_00657_amd import binding as hb, synth
    from paper_2409_00657_amd.pipeline import HotPath
    rng = np.random.default_rng(seed)
    N_CASES = 12
    dts = [torch.float32, torch.bfloat16, torch.float16]
    failures = []
    for case in range(N_CASES):
        kind = rng.integers(0, 3)
        scale = int(rng.integers(6, 15))
        if kind == 0: g = synth.uniform_graph(int(rng.integers(10, 5000)), 1, int(rng.integers(1, 20)), seed=case, device=DEV, offsets_i64=bool(rng.integers(0, 2)))
        elif kind == 1: g = synth.rmat_graph(scale, float(rng.uniform(0.5, 20)), seed=case, device=DEV, offsets_i64=bool(rng.integers(0, 2)))
        else: g = synth.chung_lu_graph(int(rng.integers(50, 20000)), float(rng.uniform(1, 30)), 2.1, seed=case, device=DEV, offsets_i64=bool(rng.integers(0, 2)))
        n = g.n_vertices
        L = int(rng.integers(1, 5))
        fan = [int(rng.integers(1, 7 if L > 2 else 16)) for _ in range(L)]
        B = int(rng.choice([1, 2, 7, 64, 100, 300]))
        G = int(rng.choice([1, 1, 2, 3, 5]))
        dt = dts[rng.integers(0, 3)]
        d = int(rng.choice([1, 3, 4, 8, 20, 32, 100, 128]))
        hidden = int(rng.choice([1, 4, 7, 16, 32, 64, 130]))
        algo = int(rng.integers(0, 3))
        tag = (case, kind, n, fan, B, G, str(dt), d, hidden, algo)
        t_seed = hb.hopgnn_slots_per_seed(fan)
        if B * t_seed * G > 3_000_000: continue
        X = synth.features(n, d, dt, seed=case, device=DEV)
        W = synth.sage_weights(d, hidden, L, dt, seed=case, device=DEV, bias=bool(rng.integers(0, 2)))
        hp = HotPath(g.offsets, g.indices, X, W, B, fan, group=G, pg_algo=algo)
        off_np, idx_np = g.offsets.cpu().numpy(), g.indices.cpu().numpy()
        T = hp.shape.n_slots
        for it in range(2):
            seeds = synth.seeds(n, B * G, case * 10 + it, device=DEV)
            keys = [int(rng.integers(0, 2 ** 63)) for _ in range(G)]
            out = torch.full((G * B, hidden), float("nan"), dtype=dt, device=DEV)
            hp.forward(seeds, keys, out)
            torch.cuda.synchronize()
            ref_ids = []
            for b in range(G):
                i, ip = orc.sample(off_np, idx_np, seeds[b * B:(b + 1) * B].cpu().numpy(), fan, keys[b])
                ref_ids.append(i)
            all_ids = np.concatenate(ref_ids)
            ru, rr = orc.pregather(all_ids)
            ok = np.array_equal(hp.ids.cpu().numpy()[:G * T], all_ids) and np.array_equal(hp.indptr.cpu().numpy(), ip) \
                and int(hp.n_uniq.item()) == len(ru) and np.array_equal(hp.uniq[:len(ru)].cpu().numpy(), ru) \
                and np.array_equal(hp.remap.cpu().numpy()[:G * T], rr)
            Xu_ref = orc.gather(to_bits(X), ru)
            ok = ok and to_bits(hp.Xu[:len(ru)]).tobytes() == Xu_ref.tobytes()
            if not ok:
                failures.append(("integer path", tag, it))
                continue
            wb = weights_bits(W)
            for b in range(G):
                outs = orc.forward(Xu_ref, ORC_DT[dt], ref_ids[b], ip, rr[b * T:(b + 1) * T], B, fan, wb)
                e = rel_err(to_f64(out[b * B:(b + 1) * B]), outs[-1][0])
                # chained layers: the oracle chains its own rounded activations, so allow the depth
                if not (e <= chain_tol(dt, L)):
                    failures.append(("forward", e, tag, it, b))
    assert not failures, failures


@pytest.mark.parametrize("seed", [1, 2])
def test_random_frontier_batches(seed):
    """Deduplicated and layer-wise sampled micrographs on random graphs, shapes, groups and types:
    structure bit-exact, root rows and (fp32) weight gradients against the oracle chain."""
    from paper_2409_00657_amd import binding as hb, synth
    from paper_2409_00657_amd.pipeline import DedupPath
    from oracle import dedup as orc_dedup, frontier as orc_frontier, layerwise as orc_lw
    rng = np.random.default_rng(100 + seed)
    dts = [torch.float32, torch.bfloat16, torch.float16]
    failures = []
    for case in range(10):
        kind = rng.integers(0, 3)
        if kind == 0: g = synth.uniform_graph(int(rng.integers(10, 3000)), 0, int(rng.integers(1, 12)), seed=case, device=DEV, offsets_i64=bool(rng.integers(0, 2)))
        elif kind == 1: g = synth.rmat_graph(int(rng.integers(6, 13)), float(rng.uniform(0.5, 12)), seed=case, device=DEV, offsets_i64=bool(rng.integers(0, 2)))
        else: g = synth.chung_lu_graph(int(rng.integers(50, 8000)), float(rng.uniform(1, 20)), 2.1, seed=case, device=DEV, offsets_i64=bool(rng.integers(0, 2)))
        n = g.n_vertices
        sampler = ["node", "layer"][rng.integers(0, 2)]
        L = int(rng.integers(1, 4))
        fan = [int(rng.integers(1, 9 if sampler == "node" else 20)) for _ in range(L)]
        B = int(rng.choice([1, 3, 17, 64, 90]))
        G = int(rng.choice([1, 1, 2, 4]))
        dt = dts[rng.integers(0, 3)]
        d = int(rng.choice([1, 4, 12, 32, 100]))
        hidden = int(rng.choice([1, 4, 20, 64]))
        algo = int(rng.integers(0, 3))
        tag = (case, kind, n, sampler, fan, B, G, str(dt), d, hidden, algo)
        X = synth.features(n, d, dt, seed=case, device=DEV)
        W = synth.sage_weights(d, hidden, L, dt, seed=case, device=DEV, bias=bool(rng.integers(0, 2)))
        dp = DedupPath(g.offsets, g.indices, X, W, B, fan, pg_algo=algo, group=G, sampler=sampler)
        dp.enable_backward()
        for t in dp.H + dp.dH:
            t.fill_(float("nan"))
        off_np, idx_np = g.offsets.cpu().numpy(), g.indices.cpu().numpy()
        sample = orc_dedup.sample_dedup if sampler == "node" else orc_lw.sample_layerwise
        for it in range(2):
            seeds = synth.seeds(n, B * G, case * 10 + it, device=DEV)
            keys = [int(rng.integers(0, 2 ** 63)) for _ in range(G)]
            out = torch.full((G * B, hidden), float("nan"), dtype=dt, device=DEV)
            dp.forward(seeds, keys, out)
            torch.cuda.synchronize()
            if sampler == "node":       # the node-wise oracle takes one key: batch by batch, then the level-major merge is checked through the rows
                parts = [sample(off_np, idx_np, seeds[b * B:(b + 1) * B].cpu().numpy(), fan, keys[b]) for b in range(G)]
            else:
                parts = [sample(off_np, idx_np, seeds.cpu().numpy(), fan, [k for k in keys for _ in range(B)])]
            if len(parts) == 1:
                nv, ls, ip, ix = parts[0]
                n_nodes, n_nonleaf, nnz = len(nv), int(ls[L]), len(ix)
                ok = np.array_equal(dp.level_start.cpu().numpy(), ls) and np.array_equal(dp.node_vertex[:n_nodes].cpu().numpy(), nv) \
                    and np.array_equal(dp.indptr[:n_nonleaf + 1].cpu().numpy(), ip) and np.array_equal(dp.idx[:nnz].cpu().numpy(), ix) \
                    and bool((dp.node_vertex[n_nodes:] == -1).all())
                if not ok:
                    failures.append(("structure", tag, it))
                    continue
            wb = weights_bits(W)
            for b, st in enumerate(parts):
                ref = orc_frontier.layer_chain(orc, to_bits(X), ORC_DT[dt], *st, wb)
                got = out if len(parts) == 1 else out[b * B:(b + 1) * B]
                e = rel_err(to_f64(got), ref)
                if not (e <= chain_tol(dt, L)):
                    failures.append(("forward", e, tag, it, b))
            if dt == torch.float32 and len(parts) == 1:
                dp.run_batch(seeds, keys)
                dp.backward()
                torch.cuda.synchronize()
                _, grads = orc_frontier.layer_chain_grads(orc, to_bits(X), 0, *parts[0], wb, to_f64(dp.dHL))
                for k in range(L):
                    for part in range(3):
                        if W[k][part] is None:
                            continue
                        e = rel_err(to_f64(dp.gW[k][part]), grads[k][part])
                        if not (e <= 5e-5 * L):
                            failures.append(("grad", e, k, part, tag, it))
                for layer in dp.gW:
                    for t in layer:
                        if t is not None:
                            t.zero_()
    assert not failures, failures
