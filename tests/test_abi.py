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
                             'offsetof(hopgnn_batch_plan,merge_layers));return 0;}\n')
        exe = os.path.join(d, "p")
        subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), src, "-o", exe], check=True)
        size, off_w, off_m = map(int, subprocess.run([exe], capture_output=True, text=True, check=True).stdout.split())
    assert c.sizeof(hb.BatchPlan) == size
    assert hb.BatchPlan.W_self.offset == off_w
    assert hb.BatchPlan.merge_layers.offset == off_m
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


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    from paper_2409_00657_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(binding.HopgnnError):
        binding.hopgnn_slots_per_seed([5, 5])
