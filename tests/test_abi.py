"""CPU-side checks of the boundary: the library loads, exports every function the
header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "hopgnn.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(hopgnn_[a-z0-9_]+)\s*\(", src)))


@pytest.fixture(scope="module")
def lib():
    from paper_2409_00657_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_2409_00657_amd.build import build_library
        build_library()
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert {"hopgnn_sample", "hopgnn_pregather", "hopgnn_gather", "hopgnn_sage_fwd"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    from paper_2409_00657_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_host_only_queries(lib):
    from paper_2409_00657_amd import binding as hb
    assert hb.hopgnn_slots_per_seed([5, 5]) == 31
    assert hb.hopgnn_slots_per_seed([15, 10, 5]) == 916
    assert hb.hopgnn_slots_per_seed([10, 10, 10]) == 1111
    assert hb.hopgnn_slots_per_seed([3, 0]) == -1
    assert hb.hopgnn_slots_per_seed([2] * 9) == -1
    assert hb.hopgnn_pregather_ws_bytes(1000, 1 << 20) >= (1 << 20) // 8
    assert hb.hopgnn_sage_fwd_ws_bytes(__import__("torch").float32, 100, 64, 32) >= 100 * 64 * 4
    assert lib.hopgnn_status_str(0) == b"ok"
    assert lib.hopgnn_status_str(2) == b"workspace too small"


def test_argument_errors_are_reported_before_any_launch(lib):
    c = ctypes
    fan = (c.c_int32 * 2)(5, 5)
    # NULL graph
    assert lib.hopgnn_sample(None, None, 4, fan, 2, 0, None, None, None, None) == 1
    # negative sizes / NULL outputs
    assert lib.hopgnn_pregather(None, -1, 10, 0, None, None, None, None, 0, None) == 1
    assert lib.hopgnn_pregather(None, 5, 10, 0, None, None, None, None, 0, None) == 1
    assert lib.hopgnn_gather(None, 0, 10, 0, 4, None, 3, None, None, None) == 1
    assert lib.hopgnn_gather(None, 7, 10, 4, 4, None, 3, None, None, None) == 1
    assert lib.hopgnn_gather(None, 0, 10, 4, 4, None, 3, None, None, None) == 1
    assert lib.hopgnn_gather(None, 0, 10, 4, 4, None, 0, None, None, None) == 0   # empty: no-op
    assert lib.hopgnn_sage_fwd(None, 0, 5, 0, None, None, None, 3, None, None, None, 4, 0,
                               None, None, 0, None) == 1
    assert lib.hopgnn_sage_fwd(None, 0, 5, 4, None, None, None, 0, None, None, None, 4, 0,
                               None, None, 0, None) == 0                          # n_dst = 0


def test_batch_plan_errors_and_layout(lib):
    from paper_2409_00657_amd import binding as hb
    c = ctypes
    # the ctypes mirror must have the C struct's size: compile a one-line probe with the same header
    import subprocess
    import tempfile
    with tempfile.TemporaryDirectory() as d:
        src = os.path.join(d, "p.c")
        open(src, "w").write('#include <stdio.h>\n#include <stddef.h>\n#include "hopgnn.h"\nint main(void){printf("%zu %zu %zu",'
                             'sizeof(hopgnn_batch_plan),offsetof(hopgnn_batch_plan,W_self),'
                             'offsetof(hopgnn_batch_plan,dd_ws_bytes));return 0;}\n')
        exe = os.path.join(d, "p")
        subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), src, "-o", exe], check=True)
        size, off_w, off_m = map(int, subprocess.run([exe], capture_output=True, text=True, check=True).stdout.split())
    assert c.sizeof(hb.BatchPlan) == size
    assert hb.BatchPlan.W_self.offset == off_w
    assert hb.BatchPlan.dd_ws_bytes.offset == off_m
    plan = hb.BatchPlan()
    keys = (c.c_uint64 * 1)(0)
    one = c.c_void_p(8)    # any non-NULL address: the checks below fail before it is used
    assert lib.hopgnn_batch_fwd(None, one, keys, 1, one, None) == 1
    plan.group, plan.n_layers, plan.n_seeds = 1, 2, 4
    assert lib.hopgnn_batch_fwd(c.byref(plan), one, keys, 0, one, None) == 1      # no batches
    assert lib.hopgnn_batch_fwd(c.byref(plan), one, keys, 2, one, None) == 1      # more than the plan's group
    assert lib.hopgnn_batch_fwd(c.byref(plan), one, keys, 1, one, None) == 1      # fanouts are zero
    plan.n_layers = 9
    assert lib.hopgnn_batch_fwd(c.byref(plan), one, keys, 1, one, None) == 1


def test_newer_entry_points_reject_bad_arguments(lib):
    c = ctypes
    fan = (c.c_int32 * 2)(5, 5)
    keys = (c.c_uint64 * 2)(1, 2)
    one = c.c_void_p(8)
    from paper_2409_00657_amd import binding as hb
    g = hb._Csr(10, 20, 8, 0, 8)
    # grouped / merged sampling
    assert lib.hopgnn_sample_group(None, one, 4, fan, 2, keys, 2, one, None, None, 0, None) == 1
    assert lib.hopgnn_sample_group(c.byref(g), one, 4, fan, 2, keys, -1, one, None, None, 0, None) == 1
    assert lib.hopgnn_sample_group(c.byref(g), one, 4, fan, 2, keys, 0, one, None, None, 0, None) == 0   # no batches
    assert lib.hopgnn_sample_group(c.byref(g), one, 4, fan, 2, None, 2, one, None, None, 0, None) == 1   # no keys
    assert lib.hopgnn_sample_merged(c.byref(g), one, 8, 0, fan, 2, keys, one, None, None, None) == 1     # seeds_per_key < 1
    assert lib.hopgnn_sample_merged(c.byref(g), one, 0, 4, fan, 2, keys, one, None, None, None) == 0     # no seeds
    big = (c.c_int32 * 3)(1000, 1000, 1000)
    assert lib.hopgnn_sample_merged(c.byref(g), one, 4, 4, big, 3, keys, one, None, None, None) == 3     # 4e9 slots
    # workspace preparation
    assert lib.hopgnn_pregather_ws_init(None, 1 << 20, 10, 1000, 0, None) == 1
    assert lib.hopgnn_pregather_ws_init(one, 1 << 20, 10, 1000, 0, None) == 1          # not 256-byte aligned
    assert lib.hopgnn_pregather_ws_init(c.c_void_p(256), 16, 10, 1000, 1, None) == 2   # too small
    # aggregator and layer variants
    assert lib.hopgnn_sage_fwd_agg(None, 0, 5, 4, None, None, None, 3, None, None, None, 4, 7, 0, None, None, 0,
                                   None) == 1                                          # unknown aggregator
    assert lib.hopgnn_gcn_fwd(None, 0, 5, 4, None, None, None, 0, None, None, 4, 1, 0, None, None, 0, None) == 0
    assert lib.hopgnn_gcn_fwd(None, 0, 5, 4, None, None, None, 3, None, None, 4, 2, 0, None, None, 0, None) == 1
    assert lib.hopgnn_gat_fwd(None, 0, 5, None, 4, None, None, None, 3, None, None, None, None, 6, 4, 0, None, None,
                              0, None) == 1                                            # 4 heads do not divide 6
    assert lib.hopgnn_gat_fwd_ws_bytes(0, 100, 8, 8, 17) == 0
    assert lib.hopgnn_sage_bwd_ws_bytes(5, 100, 8, 8, 1) == 0


def test_sage_bwd_dev_rejects_bad_arguments(lib):
    c = ctypes
    one = c.c_void_p(256)
    args = lambda dt=0, n_src=8, n_dst=4, d_in=4, d_out=4, ws=one, ws_bytes=1 << 30, self_idx=one: (
        one, dt, n_src, None, d_in, self_idx, one, one, n_dst, None, one, one, one, None, 1, one, d_out, one, one, None,
        None, ws, ws_bytes, None)
    assert lib.hopgnn_sage_bwd_dev(*args(dt=7)) == 1
    assert lib.hopgnn_sage_bwd_dev(*args(n_dst=-1)) == 1
    assert lib.hopgnn_sage_bwd_dev(*args(d_in=0)) == 1
    assert lib.hopgnn_sage_bwd_dev(*args(n_dst=0)) == 0                       # nothing to do
    assert lib.hopgnn_sage_bwd_dev(*args(ws=None)) == 1
    assert lib.hopgnn_sage_bwd_dev(*args(ws=c.c_void_p(8))) == 1              # not 256-byte aligned
    assert lib.hopgnn_sage_bwd_dev(*args(ws_bytes=16)) == 2
    assert lib.hopgnn_sage_bwd_dev(*args(n_src=2, self_idx=None)) == 1        # identity self rows must exist
    assert lib.hopgnn_sage_bwd_dev(*args(n_dst=1 << 31)) == 3


def test_sgd_update_multi_rejects_bad_arguments(lib):
    c = ctypes
    W = (c.c_void_p * 2)(256, 512)
    g = (c.c_void_p * 2)(1024, 2048)
    n = (c.c_int64 * 2)(4, 4)
    assert lib.hopgnn_sgd_update_multi(W, 0, g, n, 0, 0.1, 1, None) == 0           # no tensors
    assert lib.hopgnn_sgd_update_multi(W, 0, g, n, 33, 0.1, 1, None) == 1
    assert lib.hopgnn_sgd_update_multi(W, 0, g, n, -1, 0.1, 1, None) == 1
    assert lib.hopgnn_sgd_update_multi(W, 4, g, n, 2, 0.1, 1, None) == 1
    assert lib.hopgnn_sgd_update_multi(None, 0, g, n, 2, 0.1, 1, None) == 1
    assert lib.hopgnn_sgd_update_multi(W, 0, g, (c.c_int64 * 2)(4, -1), 2, 0.1, 1, None) == 1
    assert lib.hopgnn_sgd_update_multi((c.c_void_p * 2)(256, None), 0, g, n, 2, 0.1, 1, None) == 1
    assert lib.hopgnn_sgd_update_multi(W, 0, g, (c.c_int64 * 2)(0, 0), 2, 0.1, 1, None) == 0     # all empty


def test_slot_order_backward_rejects_bad_arguments(lib):
    c = ctypes
    one = c.c_void_p(256)
    args = lambda first=2, n_dst=4, n_src=8, idx=one, dt=0: (
        one, dt, n_src, 4, one, idx, n_dst, first, one, one, None, None, 0, one, 4, one, one, None, None, one, 1 << 30,
        None)
    assert lib.hopgnn_sage_bwd_slots(*args(first=-1)) == 1
    assert lib.hopgnn_sage_bwd_slots(*args(first=5)) == 1            # past the destination rows
    assert lib.hopgnn_sage_bwd_slots(*args(idx=None)) == 1
    assert lib.hopgnn_sage_bwd_slots(*args(dt=5)) == 1
    assert lib.hopgnn_sage_bwd_slots(*args(n_src=2)) == 1            # self rows are the rows themselves
    assert lib.hopgnn_sage_bwd_slots(*args(n_dst=0, first=0)) == 0


def test_layer_calls_with_device_counts_reject_bad_arguments(lib):
    c = ctypes
    one = c.c_void_p(256)
    gcn = lambda dt=0, n_dst=4, norm=1, ws_bytes=1 << 30, self_idx=one, n_src=8: (
        one, dt, n_src, 4, self_idx, one, one, n_dst, None, one, None, 4, norm, 0, one, one, ws_bytes, None)
    assert lib.hopgnn_gcn_fwd_dev(*gcn(dt=9)) == 1
    assert lib.hopgnn_gcn_fwd_dev(*gcn(norm=2)) == 1
    assert lib.hopgnn_gcn_fwd_dev(*gcn(n_dst=0)) == 0
    assert lib.hopgnn_gcn_fwd_dev(*gcn(ws_bytes=8)) == 2
    assert lib.hopgnn_gcn_fwd_dev(*gcn(self_idx=None, n_src=2)) == 1
    gat = lambda heads=2, n_dst=4, ws_bytes=1 << 30: (
        one, 0, 8, None, 4, one, one, one, n_dst, None, one, one, one, None, 4, heads, 0, one, one, ws_bytes, None)
    assert lib.hopgnn_gat_fwd_dev(*gat(heads=3)) == 1          # 3 heads do not divide 4
    assert lib.hopgnn_gat_fwd_dev(*gat(heads=0)) == 1
    assert lib.hopgnn_gat_fwd_dev(*gat(n_dst=0)) == 0
    assert lib.hopgnn_gat_fwd_dev(*gat(ws_bytes=8)) == 2


def test_frontier_locality_rejects_bad_arguments(lib):
    c = ctypes
    one = c.c_void_p(256)
    ok = (one, one, one, one, 4, 2, 31, one, one, one, None)
    sub = lambda i, v: ok[:i] + (v,) + ok[i + 1:]
    assert lib.hopgnn_frontier_locality(*sub(4, -1)) == 1
    assert lib.hopgnn_frontier_locality(*sub(5, 0)) == 1
    assert lib.hopgnn_frontier_locality(*sub(5, 9)) == 1
    assert lib.hopgnn_frontier_locality(*sub(6, 0)) == 1
    assert lib.hopgnn_frontier_locality(*sub(6, 16385)) == 3           # the hash set would not fit LDS
    assert lib.hopgnn_frontier_locality(*sub(4, 0)) == 0               # no seeds
    for i in (0, 1, 2, 3, 7, 8, 9):
        assert lib.hopgnn_frontier_locality(*sub(i, None)) == 1


def test_layerwise_capacities_and_errors(lib):
    c = ctypes
    from paper_2409_00657_amd import binding as hb
    assert hb.hopgnn_layerwise_caps([10, 25]) == (36, 11, 260)
    assert hb.hopgnn_layerwise_caps([7]) == (8, 1, 7)
    assert hb.hopgnn_layerwise_caps([4, 3, 2]) == (10, 8, 4 + 12 + 6)
    caps = (c.c_int64 * 3)()
    ok = (c.c_int32 * 2)(10, 25)
    assert lib.hopgnn_layerwise_caps(ok, 2, None) == 1
    assert lib.hopgnn_layerwise_caps(None, 2, caps) == 1
    assert lib.hopgnn_layerwise_caps(ok, 0, caps) == 1
    assert lib.hopgnn_layerwise_caps(ok, 9, caps) == 1
    assert lib.hopgnn_layerwise_caps((c.c_int32 * 2)(10, 0), 2, caps) == 1
    assert lib.hopgnn_layerwise_caps((c.c_int32 * 1)(1025), 1, caps) == 3            # a budget above 1024
    assert lib.hopgnn_layerwise_caps((c.c_int32 * 2)(300, 300), 2, caps) == 3        # 90000 pairs
    assert lib.hopgnn_layerwise_caps((c.c_int32 * 2)(256, 256), 2, caps) == 0
    assert lib.hopgnn_sample_layerwise_ws_bytes(4, (c.c_int32 * 2)(300, 300), 2) == 0
    assert lib.hopgnn_sample_layerwise_ws_bytes(-1, ok, 2) == 0
    assert lib.hopgnn_sample_layerwise_ws_bytes(100, ok, 2) >= 100 * (36 + 11 + 260) * 4
    one = c.c_void_p(256)
    keys = (c.c_uint64 * 1)(1)
    g = hb._Csr(10, 20, 8, 0, 8)
    args = (keys, one, one, one, one, one, 1 << 30, None)
    assert lib.hopgnn_sample_layerwise(None, one, 4, 4, ok, 2, *args) == 1
    assert lib.hopgnn_sample_layerwise(c.byref(g), one, 4, 0, ok, 2, *args) == 1          # seeds_per_key < 1
    assert lib.hopgnn_sample_layerwise(c.byref(g), one, -1, 4, ok, 2, *args) == 1
    assert lib.hopgnn_sample_layerwise(c.byref(g), one, 0, 4, ok, 2, *args) == 0          # no seeds
    assert lib.hopgnn_sample_layerwise(c.byref(g), one, 4, 4, (c.c_int32 * 2)(300, 300), 2, *args) == 3
    assert lib.hopgnn_sample_layerwise(c.byref(g), one, 4, 4, ok, 2, None, one, one, one, one, one, 1 << 30, None) == 1
    assert lib.hopgnn_sample_layerwise(c.byref(g), one, 4, 4, ok, 2, keys, one, one, one, one, one, 16, None) == 2
    assert lib.hopgnn_sample_layerwise(c.byref(g), one, 4, 4, ok, 2, keys, one, one, one, one, c.c_void_p(8), 1 << 30,
                                       None) == 1                                         # workspace not aligned
    assert lib.hopgnn_sample_layerwise(c.byref(g), one, 8000000, 4, ok, 2, *args) == 3    # 2^31 staging slots


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    from paper_2409_00657_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(binding.HopgnnError):
        binding.hopgnn_slots_per_seed([5, 5])
