"""The entry point that allocates nothing (hopgnn_pregather_static) against hopgnn_pregather:
the same ids, bit for bit the same uniq / n_uniq / remap, on two calls in a row, the second with
a smaller input (the static scratch keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _ids(n_ids, n_vertices, seed, invalid_every=7):
    g = torch.Generator().manual_seed(seed)
    # hub-heavy multiset: squares of uniforms concentrate on low IDs, as power-law graphs do
    u = torch.rand(n_ids, generator=g, dtype=torch.float64)
    ids = (u * u * n_vertices).to(torch.int64).clamp_(0, n_vertices - 1).to(torch.int32)
    ids[::invalid_every] = -1
    return ids.to(DEV)


def _both(lib, ids, n_vertices):
    from paper_2409_00657_amd import binding as hb
    n = ids.numel()
    st = torch.cuda.current_stream().cuda_stream
    out = []
    ws = torch.empty(hb.hopgnn_pregather_ws_bytes(n, n_vertices, hb.PG_BITMAP), dtype=torch.uint8, device=DEV)
    for static in (False, True):
        uniq = torch.full((max(min(n, n_vertices), 1),), -7, dtype=torch.int32, device=DEV)
        remap = torch.full((max(n, 1),), -7, dtype=torch.int32, device=DEV)
        n_uniq = torch.full((1,), -7, dtype=torch.int64, device=DEV)
        if static:
            rc = lib.hopgnn_pregather_static(ids.data_ptr(), n, n_vertices, uniq.data_ptr(), n_uniq.data_ptr(),
                                             remap.data_ptr(), st)
        else:
            rc = lib.hopgnn_pregather(ids.data_ptr(), n, n_vertices, hb.PG_BITMAP, uniq.data_ptr(), n_uniq.data_ptr(),
                                      remap.data_ptr(), ws.data_ptr(), ws.numel(), st)
        assert rc == 0, rc
        torch.cuda.synchronize()
        U = int(n_uniq.item())
        out.append((U, uniq[:U].cpu().numpy(), remap[:n].cpu().numpy()))
    return out


def test_static_scratch_pregather_matches_workspace_pregather_twice():
    from paper_2409_00657_amd import binding as hb
    lib = hb.load_library()                      # the raw C ABI
    assert lib.hopgnn_pregather_static_max_vertices() == 1 << 24
    # first call: large (2^24 vertices, the limit); second call: smaller input over fewer vertices,
    # so stale marks of the first call would show up as extra IDs if they were not cleared
    for n_ids, n_vertices, seed in ((1_130_496, 1 << 24, 1), (113_664, 1 << 20, 2), (1_984, 20_000, 3), (0, 5_000, 4)):
        ids = _ids(n_ids, n_vertices, seed) if n_ids else torch.empty(0, dtype=torch.int32, device=DEV)
        (U0, uniq0, remap0), (U1, uniq1, remap1) = _both(lib, ids, n_vertices)
        assert U0 == U1
        np.testing.assert_array_equal(uniq0, uniq1)
        np.testing.assert_array_equal(remap0, remap1)
        if n_ids:                                # and both are the plain definition
            h = ids.cpu().numpy()
            ref = np.unique(h[h >= 0])
            np.testing.assert_array_equal(uniq1, ref)
            pos = np.where(h >= 0, np.searchsorted(ref, np.maximum(h, 0)), -1)
            np.testing.assert_array_equal(remap1, pos)


def test_static_scratch_pregather_rejects_sizes_beyond_its_scratch():
    from paper_2409_00657_amd import binding as hb
    lib = hb.load_library()
    ids = torch.zeros(16, dtype=torch.int32, device=DEV)
    uniq = torch.empty(16, dtype=torch.int32, device=DEV)
    remap = torch.empty(16, dtype=torch.int32, device=DEV)
    n_uniq = torch.zeros(1, dtype=torch.int64, device=DEV)
    rc = lib.hopgnn_pregather_static(ids.data_ptr(), 16, (1 << 24) + 1, uniq.data_ptr(), n_uniq.data_ptr(),
                                     remap.data_ptr(), None)
    assert rc == 3                               # HOPGNN_ERANGE, before any launch
    assert lib.hopgnn_pregather_static(None, 16, 100, uniq.data_ptr(), n_uniq.data_ptr(), remap.data_ptr(), None) == 1
    torch.cuda.synchronize()
