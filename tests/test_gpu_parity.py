"""GPU parity: every step through the C ABI against the CPU oracle, element by
element, on seeded inputs spanning several tiles and ragged tails."""
import numpy as np
import pytest
import torch

from helpers import ORC_DT, TOL, rel_err, to_bits, to_f64

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def hb():
    from paper_2409_00657_amd import binding
    binding.load_library()
    return binding


def _csr(rows, dtype=torch.int32):
    off = np.zeros(len(rows) + 1, np.int64)
    off[1:] = np.cumsum([len(r) for r in rows])
    idx = np.array([x for r in rows for x in r], np.int32)
    if len(idx) == 0:
        idx = np.zeros(0, np.int32)
    return torch.from_numpy(off).to(dtype), torch.from_numpy(idx)


def _gpu_sample(hb, off, idx, seeds, fan, key, with_slot_idx=True):
    B = len(seeds)
    lv = [B]
    for f in fan:
        lv.append(lv[-1] * f)
    T, S = sum(lv), sum(lv[:-1])
    ids = torch.full((T,), -7, dtype=torch.int32, device=DEV)
    indptr = torch.full((S + 1,), -7, dtype=torch.int32, device=DEV)
    slot_idx = torch.full((max(S - B, 1),), -7, dtype=torch.int32, device=DEV)
    hb.hopgnn_sample(off.to(DEV), idx.to(DEV), torch.as_tensor(seeds, dtype=torch.int32).to(DEV), fan,
                     key, ids, indptr, slot_idx if (with_slot_idx and len(fan) > 1) else None)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), indptr.cpu().numpy(), slot_idx.cpu().numpy()[:S - B], (B, T, S)


@pytest.mark.parametrize("case", range(6))
def test_sample_bit_exact(hb, orc, case):
    rng = np.random.default_rng(100 + case)
    N = [3, 50, 1000, 5000, 257, 20000][case]
    maxdeg = [3, 6, 40, 9, 300, 17][case]
    rows = [rng.integers(0, N, size=int(rng.integers(0, maxdeg))).tolist() for _ in range(N)]
    fan = [[2], [3, 2], [5, 5], [4, 3, 2], [10, 10], [7, 1, 6]][case]
    B = [1, 7, 64, 130, 33, 300][case]
    seeds = rng.integers(0, N, size=B).astype(np.int32)
    key = int(rng.integers(0, 2 ** 63))
    for dt in (torch.int32, torch.int64):
        off, idx = _csr(rows, dt)
        ids, indptr, slot_idx, (B_, T, S) = _gpu_sample(hb, off, idx, seeds, fan, key)
        ref_ids, ref_indptr = orc.sample(off.numpy(), idx.numpy(), seeds, fan, key)
        np.testing.assert_array_equal(ids, ref_ids)
        np.testing.assert_array_equal(indptr, ref_indptr)
        if len(fan) > 1:
            e = np.arange(S - B, dtype=np.int32)
            np.testing.assert_array_equal(slot_idx, np.where(ref_ids[B:S] >= 0, B + e, -1))


def test_sample_group_equals_separate_calls(hb, orc):
    """Several batches in one launch: bit for bit the per-batch calls, and the oracle's."""
    from paper_2409_00657_amd import synth
    g = synth.rmat_graph(12, 9.0, device=DEV)
    off_np, idx_np = g.offsets.cpu().numpy(), g.indices.cpu().numpy()
    B, fan, G = 37, [4, 3, 5], 5
    t_seed = hb.hopgnn_slots_per_seed(fan)
    T = B * t_seed
    S = T - B * 4 * 3 * 5
    seeds = synth.seeds(g.n_vertices, B * G, 3, device=DEV)
    keys = [11, 0, 2 ** 63 + 5, 7, 7]
    ids = torch.full((G * T,), -9, dtype=torch.int32, device=DEV)
    indptr = torch.full((S + 1,), -9, dtype=torch.int32, device=DEV)
    stride = S - B + 3          # a stride with slack: the gaps stay untouched
    slot_idx = torch.full((G * stride,), -9, dtype=torch.int32, device=DEV)
    hb.hopgnn_sample_group(g.offsets, g.indices, seeds, B, fan, keys, ids, indptr, slot_idx, stride)
    torch.cuda.synchronize()
    for b in range(G):
        ids1 = torch.empty(T, dtype=torch.int32, device=DEV)
        ip1 = torch.empty(S + 1, dtype=torch.int32, device=DEV)
        si1 = torch.empty(S - B, dtype=torch.int32, device=DEV)
        hb.hopgnn_sample(g.offsets, g.indices, seeds[b * B:(b + 1) * B], fan, keys[b], ids1, ip1, si1)
        torch.cuda.synchronize()
        assert torch.equal(ids[b * T:(b + 1) * T], ids1)
        assert torch.equal(indptr, ip1)
        assert torch.equal(slot_idx[b * stride:b * stride + S - B], si1)
        assert bool((slot_idx[b * stride + S - B:(b + 1) * stride] == -9).all())
        ref_ids, ref_ip = orc.sample(off_np, idx_np, seeds[b * B:(b + 1) * B].cpu().numpy(), fan, keys[b])
        np.testing.assert_array_equal(ids1.cpu().numpy(), ref_ids)
        np.testing.assert_array_equal(ip1.cpu().numpy(), ref_ip)
    # 70 batches: more than one launch's worth of keys
    G2 = 70
    seeds2 = synth.seeds(g.n_vertices, 8 * G2, 4, device=DEV)
    keys2 = list(range(100, 100 + G2))
    t2 = 8 * hb.hopgnn_slots_per_seed([3, 2])
    ids2 = torch.empty(G2 * t2, dtype=torch.int32, device=DEV)
    hb.hopgnn_sample_group(g.offsets, g.indices, seeds2, 8, [3, 2], keys2, ids2)
    torch.cuda.synchronize()
    for b in (0, 63, 64, 69):
        ref_ids, _ = orc.sample(off_np, idx_np, seeds2[b * 8:(b + 1) * 8].cpu().numpy(), [3, 2], keys2[b])
        np.testing.assert_array_equal(ids2[b * t2:(b + 1) * t2].cpu().numpy(), ref_ids)
    # overlapping neighbour lists are refused
    with pytest.raises(hb.HopgnnError):
        hb.hopgnn_sample_group(g.offsets, g.indices, seeds, B, fan, keys, ids, indptr, slot_idx, S - B - 1)


def test_sample_edge_cases(hb, orc):
    # zero seeds: no-op; all-isolated graph: every child invalid
    off, idx = _csr([[], [], []])
    ids, indptr, _, _ = _gpu_sample(hb, off, idx, np.array([2, 0], np.int32), [3, 2], 5)
    ref_ids, ref_indptr = orc.sample(off.numpy(), idx.numpy(), np.array([2, 0], np.int32), [3, 2], 5)
    np.testing.assert_array_equal(ids, ref_ids)
    np.testing.assert_array_equal(indptr, ref_indptr)
    assert (ids[2:] == -1).all()
    empty = torch.zeros(0, dtype=torch.int32, device=DEV)
    hb.hopgnn_sample(off.to(DEV), idx.to(DEV), empty, [3, 2], 0, empty, None, None)
    with pytest.raises(hb.HopgnnError):
        hb.hopgnn_sample(off.to(DEV), idx.to(DEV), empty, [3, 0], 0, empty, None, None)
    # a vertex of huge degree and degree 1 (remainder by 1 and by a large number)
    rows = [[1] * 1 , list(range(2, 70002)) ] + [[0]] * 70000
    off, idx = _csr(rows, torch.int64)
    seeds = np.array([1, 0, 1], np.int32)
    ids, _, _, _ = _gpu_sample(hb, off, idx, seeds, [64, 2], 99)
    ref_ids, _ = orc.sample(off.numpy(), idx.numpy(), seeds, [64, 2], 99)
    np.testing.assert_array_equal(ids, ref_ids)


def _gpu_pregather(hb, ids_np, n_vertices, algo=0):
    ids = torch.from_numpy(ids_np).to(DEV)
    n = len(ids_np)
    uniq = torch.full((max(min(n, n_vertices), 1),), -7, dtype=torch.int32, device=DEV)
    remap = torch.full((max(n, 1),), -7, dtype=torch.int32, device=DEV)
    n_uniq = torch.full((1,), -7, dtype=torch.int64, device=DEV)
    ws = torch.empty(hb.hopgnn_pregather_ws_bytes(n, n_vertices, algo), dtype=torch.uint8, device=DEV)
    ws.fill_(0xAB)      # the call may not rely on workspace contents
    hb.hopgnn_pregather(ids, n_vertices, uniq, n_uniq, remap, ws, algo)
    torch.cuda.synchronize()
    U = int(n_uniq.item())
    return uniq.cpu().numpy()[:U], remap.cpu().numpy()[:n], U


@pytest.mark.parametrize("algo", [0, 1, 2])
@pytest.mark.parametrize("case", range(8))
def test_pregather_bit_exact(hb, orc, case, algo):
    rng = np.random.default_rng(200 + case)
    n, N = [(0, 10), (1, 1), (5, 33), (1984, 20000), (113664, 1 << 20), (300001, 70000),
            (4096, (1 << 31) - 1), (200000, 100)][case]
    ids = rng.integers(0, N, size=n).astype(np.int32)
    if n > 3:
        ids[rng.random(n) < 0.25] = -1
        ids[-1] = N - 1          # the last vertex, in the bitmap's ragged last word
        ids[0] = 0
    if case == 2:
        ids[:] = -1              # nothing valid
    uniq, remap, U = _gpu_pregather(hb, ids, N, algo)
    ref_uniq, ref_remap = orc.pregather(ids)
    assert U == len(ref_uniq)
    np.testing.assert_array_equal(uniq, ref_uniq)
    np.testing.assert_array_equal(remap, ref_remap)


def test_pregather_leaves_its_workspace_clean(hb, orc):
    """Whatever the workspace held, after a bitmap pre-gather the presence map (one byte per vertex
    at the start of the workspace) is zero again, and a prepared workspace stays prepared."""
    rng = np.random.default_rng(77)
    N, T = 100_000, 30_000
    ids_np = rng.integers(0, N, size=T).astype(np.int32)
    ids_np[rng.random(T) < 0.1] = -1
    ids = torch.from_numpy(ids_np).to(DEV)
    ws = torch.empty(hb.hopgnn_pregather_ws_bytes(T, N, 1), dtype=torch.uint8, device=DEV)
    ws.fill_(0x5A)
    uniq = torch.empty(T, dtype=torch.int32, device=DEV)
    remap = torch.empty(T, dtype=torch.int32, device=DEV)
    n_uniq = torch.zeros(1, dtype=torch.int64, device=DEV)
    ref_u, ref_r = orc.pregather(ids_np)
    for _ in range(2):
        hb.hopgnn_pregather(ids, N, uniq, n_uniq, remap, ws, algo=1)
        torch.cuda.synchronize()
        assert int(n_uniq.item()) == len(ref_u)
        np.testing.assert_array_equal(uniq[:len(ref_u)].cpu().numpy(), ref_u)
        np.testing.assert_array_equal(remap.cpu().numpy(), ref_r)
        assert int(ws[:N].to(torch.int64).sum().item()) == 0
    ws.fill_(0x33)
    hb.hopgnn_pregather_ws_init(ws, T, N, 1)
    torch.cuda.synchronize()
    assert int(ws[:N].to(torch.int64).sum().item()) == 0


def test_pregather_hub_heavy_and_repeatable(hb, orc):
    # power-law-like multiset: a few IDs repeated tens of thousands of times
    rng = np.random.default_rng(7)
    N = 1 << 22
    ids = np.minimum((N * rng.random(500000) ** 6).astype(np.int64), N - 1).astype(np.int32)
    ref_uniq, ref_remap = orc.pregather(ids)
    for algo in (1, 1, 2, 2):
        uniq, remap, U = _gpu_pregather(hb, ids, N, algo)
        np.testing.assert_array_equal(uniq, ref_uniq)
        np.testing.assert_array_equal(remap, ref_remap)


@pytest.mark.parametrize("dtype,dim,ld", [(torch.float32, 32, 32), (torch.float32, 128, 128),
                                          (torch.float32, 100, 100), (torch.bfloat16, 256, 256),
                                          (torch.float16, 128, 128), (torch.float32, 7, 7),
                                          (torch.float16, 5, 5), (torch.float16, 6, 6),
                                          (torch.float32, 64, 80), (torch.bfloat16, 24, 40)])
def test_gather_byte_exact(hb, orc, dtype, dim, ld):
    rng = np.random.default_rng(dim)
    n_rows = 5003
    big = torch.from_numpy(rng.standard_normal((n_rows, ld)).astype(np.float32)).to(dtype).to(DEV)
    X = big[:, :dim]
    uniq_np = np.unique(rng.integers(0, n_rows, size=3001)).astype(np.int32)
    uniq_np[-1] = n_rows - 1
    uniq = torch.from_numpy(uniq_np).to(DEV)
    U = len(uniq_np)
    ref = orc.gather(to_bits(big)[:, :dim], uniq_np)
    # host-count mode
    Xu = torch.zeros((U, dim), dtype=dtype, device=DEV)
    hb.hopgnn_gather(X, uniq, U, None, Xu)
    torch.cuda.synchronize()
    assert to_bits(Xu).tobytes() == ref.tobytes()
    # device-count mode: capacity larger than U, rows past U untouched
    cap = U + 100
    Xu2 = torch.full((cap, dim), 3.0, dtype=dtype, device=DEV)
    uniq_cap = torch.cat([uniq, torch.zeros(100, dtype=torch.int32, device=DEV)])
    n_dev = torch.tensor([U], dtype=torch.int64, device=DEV)
    hb.hopgnn_gather(X, uniq_cap, cap, n_dev, Xu2)
    torch.cuda.synchronize()
    assert to_bits(Xu2[:U]).tobytes() == ref.tobytes()
    assert (Xu2[U:] == 3.0).all()


def _rand_csr(rng, n_dst, n_src, max_len, p_invalid=0.15):
    lens = rng.integers(0, max_len + 1, size=n_dst)
    indptr = np.zeros(n_dst + 1, np.int32)
    indptr[1:] = np.cumsum(lens)
    idx = rng.integers(0, n_src, size=int(indptr[-1])).astype(np.int32)
    idx[rng.random(len(idx)) < p_invalid] = -1
    return indptr, idx


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("shape", [(700, 333, 32, 32, 6), (3000, 1111, 128, 128, 12),
                                   (5000, 777, 100, 256, 16), (900, 300, 256, 256, 30),
                                   (400, 129, 20, 12, 5), (300, 65, 7, 5, 4),
                                   (2000, 40000, 64, 128, 3), (1500, 600, 512, 64, 8),
                                   (900, 4000, 136, 520, 7)])
def test_sage_fwd_within_tolerance(hb, orc, dtype, shape):
    n_src, n_dst, d_in, d_out, max_len = shape
    rng = np.random.default_rng(n_src + d_in)
    mk = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float32))
    H = mk(n_src, d_in).to(dtype)
    Ws = (mk(d_in, d_out) / np.sqrt(d_in)).to(dtype)
    Wn = (mk(d_in, d_out) / np.sqrt(d_in)).to(dtype)
    b = (mk(d_out) * 0.1).to(dtype)
    indptr, idx = _rand_csr(rng, n_dst, n_src, max_len)
    self_idx = rng.integers(0, n_src, size=n_dst).astype(np.int32)
    self_idx[rng.random(n_dst) < 0.05] = -1
    for relu, use_bias, use_self in [(True, True, True), (False, False, False)]:
        if not use_self and n_dst > n_src:
            continue
        ws = torch.empty(hb.hopgnn_sage_fwd_ws_bytes(dtype, n_dst, d_in, d_out), dtype=torch.uint8, device=DEV)
        out = torch.full((n_dst, d_out), 9.0, dtype=dtype, device=DEV)
        hb.hopgnn_sage_fwd(H.to(DEV), n_src, torch.from_numpy(self_idx).to(DEV) if use_self else None,
                           torch.from_numpy(indptr).to(DEV), torch.from_numpy(idx).to(DEV), n_dst,
                           Ws.to(DEV), Wn.to(DEV), b.to(DEV) if use_bias else None, relu, out, ws)
        torch.cuda.synchronize()
        ref = orc.sage_fwd(to_bits(H), ORC_DT[dtype], self_idx if use_self else None, indptr, idx,
                           to_bits(Ws), to_bits(Wn), to_bits(b) if use_bias else None, relu)
        err = rel_err(to_f64(out), ref)
        assert err <= TOL[dtype], (err, shape, relu)
        # run-to-run bit stability
        out2 = torch.empty_like(out)
        hb.hopgnn_sage_fwd(H.to(DEV), n_src, torch.from_numpy(self_idx).to(DEV) if use_self else None,
                           torch.from_numpy(indptr).to(DEV), torch.from_numpy(idx).to(DEV), n_dst,
                           Ws.to(DEV), Wn.to(DEV), b.to(DEV) if use_bias else None, relu, out2, ws)
        torch.cuda.synchronize()
        assert to_bits(out).tobytes() == to_bits(out2).tobytes()


def _oracle_rows_parallel(orc, H_bits, odt, self_idx, indptr, idx, Ws, Wn, b, relu, chunk=4096, threads=16):
    """orc.sage_fwd over all rows, in chunks of rows on several host threads (the oracle is a loop
    over independent rows and its C calls release the interpreter lock)."""
    from concurrent.futures import ThreadPoolExecutor
    n_dst = len(indptr) - 1

    def run(lo):
        hi = min(n_dst, lo + chunk)
        ip = indptr[lo:hi + 1].astype(np.int64)
        e0, e1 = int(ip[0]), int(ip[-1])
        return orc.sage_fwd(H_bits, odt, None if self_idx is None else self_idx[lo:hi], (ip - e0).astype(np.int32),
                            idx[e0:e1], Ws, Wn, b, relu)
    with ThreadPoolExecutor(max_workers=threads) as pool:
        return np.concatenate(list(pool.map(run, range(0, n_dst, chunk))))


@pytest.mark.timeout(300)
@pytest.mark.parametrize("dtype,d_out", [(torch.float32, 256), (torch.bfloat16, 512), (torch.float16, 512),
                                         (torch.bfloat16, 256)])
def test_sage_fwd_every_row_through_the_large_tiles(hb, orc, dtype, d_out):
    """The two-matrix layer (K = 2*d_in, self rows through self_idx) at a size that takes the largest
    projection tiles - 128 x 128 for fp32, 256 x 256 for 2-byte types - with EVERY output row checked
    against the oracle: 66,000 rows span 258 to 516 row tiles, a ragged last tile, and many rounds
    over the 8 XCDs."""
    n_src, n_dst, d_in, max_len = 9000, 66_000, 128, 9
    rng = np.random.default_rng(d_out + n_dst)
    mk = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float32))
    H = mk(n_src, d_in).to(dtype)
    Ws = (mk(d_in, d_out) / np.sqrt(d_in)).to(dtype)
    Wn = (mk(d_in, d_out) / np.sqrt(d_in)).to(dtype)
    b = (mk(d_out) * 0.1).to(dtype)
    indptr, idx = _rand_csr(rng, n_dst, n_src, max_len)
    self_idx = rng.integers(0, n_src, size=n_dst).astype(np.int32)
    self_idx[rng.random(n_dst) < 0.03] = -1
    ws = torch.empty(hb.hopgnn_sage_fwd_ws_bytes(dtype, n_dst, d_in, d_out), dtype=torch.uint8, device=DEV)
    out = torch.full((n_dst, d_out), 9.0, dtype=dtype, device=DEV)
    hb.hopgnn_sage_fwd(H.to(DEV), n_src, torch.from_numpy(self_idx).to(DEV), torch.from_numpy(indptr).to(DEV),
                       torch.from_numpy(idx).to(DEV), n_dst, Ws.to(DEV), Wn.to(DEV), b.to(DEV), True, out, ws)
    torch.cuda.synchronize()
    ref = _oracle_rows_parallel(orc, to_bits(H), ORC_DT[dtype], self_idx, indptr, idx, to_bits(Ws), to_bits(Wn),
                                to_bits(b), True)
    got = to_f64(out)
    # the tolerance per block of rows as well as overall, so that one bad tile cannot hide in the rms
    assert rel_err(got, ref) <= TOL[dtype]
    worst = max(rel_err(got[lo:lo + 256], ref[lo:lo + 256]) for lo in range(0, n_dst, 256))
    assert worst <= 2 * TOL[dtype], worst


def test_sage_fwd_special_cases_exact(hb):
    # one neighbour -> mean is that row; identity weights -> output is the row (exact in fp32)
    rng = np.random.default_rng(1)
    d = 64
    H = torch.from_numpy(rng.standard_normal((50, d)).astype(np.float32)).to(DEV)
    I = torch.eye(d, device=DEV)
    Z = torch.zeros((d, d), device=DEV)
    n_dst = 40
    indptr = torch.arange(n_dst + 1, dtype=torch.int32, device=DEV)
    idx = torch.from_numpy(rng.integers(0, 50, size=n_dst).astype(np.int32)).to(DEV)
    ws = torch.empty(hb.hopgnn_sage_fwd_ws_bytes(torch.float32, n_dst, d, d), dtype=torch.uint8, device=DEV)
    out = torch.empty((n_dst, d), device=DEV)
    hb.hopgnn_sage_fwd(H, 50, None, indptr, idx, n_dst, Z, I, None, False, out, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, H[idx.long()])
    hb.hopgnn_sage_fwd(H, 50, None, indptr, idx, n_dst, I, Z, None, False, out, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, H[:n_dst])


@pytest.mark.parametrize("case", range(4))
def test_micrograph_locality_and_owner_split_bit_exact(hb, orc, case):
    rng = np.random.default_rng(300 + case)
    N = [40, 3000, 20000, 500][case]
    fan = [[2, 2], [10, 10], [15, 10, 5], [3]][case]
    B = [5, 70, 33, 9][case]
    S = [2, 4, 8, 16][case]
    rows = [rng.integers(0, N, size=int(rng.integers(0, 9))).tolist() for _ in range(N)]
    off, idx = _csr(rows)
    seeds = rng.integers(0, N, size=B).astype(np.int32)
    owner = rng.integers(0, S, size=N).astype(np.int32)
    ids, _, _, _ = _gpu_sample(hb, off, idx, seeds, fan, 77)
    ref_tot, ref_col = orc.micrograph_locality(ids, B, fan, owner)
    n_total = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    n_coloc = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    d_owner = torch.from_numpy(owner).to(DEV)
    hb.hopgnn_micrograph_locality(torch.from_numpy(ids).to(DEV), B, fan, d_owner, n_total, n_coloc)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(n_total.cpu().numpy(), ref_tot)
    np.testing.assert_array_equal(n_coloc.cpu().numpy(), ref_col)
    # owner split of the batch's pre-gathered set, with U on the device and on the host
    uniq_np, _ = orc.pregather(ids)
    U = len(uniq_np)
    cap = U + 37
    uniq = torch.zeros(cap, dtype=torch.int32, device=DEV)
    uniq[:U] = torch.from_numpy(uniq_np).to(DEV)
    ws = torch.empty(hb.hopgnn_split_ws_bytes(cap), dtype=torch.uint8, device=DEV)
    for server in range(min(S, 3)):
        want = orc.split_by_owner(uniq_np, owner, server)
        for n_arg, n_dev in ((cap, torch.tensor([U], dtype=torch.int64, device=DEV)), (U, None)):
            remote = torch.full((cap,), -7, dtype=torch.int32, device=DEV)
            n_remote = torch.full((1,), -7, dtype=torch.int64, device=DEV)
            hb.hopgnn_split_by_owner(uniq, n_arg, n_dev, d_owner, server, remote, n_remote, ws)
            torch.cuda.synchronize()
            assert int(n_remote.item()) == len(want)
            np.testing.assert_array_equal(remote.cpu().numpy()[:len(want)], want)
            assert (remote[len(want):] == -7).all()
