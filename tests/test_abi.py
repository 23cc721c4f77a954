"""The C-ABI library builds for gfx950, loads, and exports every symbol include/cals.h declares
(no compute calls: there is no GPU here)."""
import os
import re

import paper_2010_04678_amd as P
from paper_2010_04678_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "cals.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(cals_[a-z_]+)\s*\(", src)))


def test_header_symbols_are_exported_and_bound():
    names = _declared()
    assert "cals_mttkrp" in names and "cals_iterate" in names and len(names) >= 11
    L = P.load_library()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names


def test_strerror_needs_no_device():
    L = P.load_library()
    assert L.cals_strerror(0) == b"ok"
    assert L.cals_strerror(-1) == b"invalid argument"
    assert b"unknown" in L.cals_strerror(-99)


def test_struct_layouts_match_header():
    import ctypes as C
    # sizes implied by the field lists in cals.h (natural alignment, 8-byte pointers)
    assert C.sizeof(binding._Options) == 32
    assert C.sizeof(binding._Result) == 40
    assert binding.MAX_MODES == 6      # CALS_MAX_MODES
    assert C.sizeof(binding._Stats) == 8 * 3 + 4 * 2 + 8 * 2 + 3 * 8 * binding.MAX_MODES + 8
    assert C.sizeof(binding._RoundRecord) == 32


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2010_04678_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in txt.lower() or f == "__never__", os.path.join(dirpath, f)


def test_suggested_buffer_width():
    # host logic only: plateau width, capped by the queue's total rank, never below the widest model
    assert P.suggest_max_total_rank([3, 4, 5]) == 12
    assert P.suggest_max_total_rank(list(range(1, 21)) * 10) == 256
    assert P.suggest_max_total_rank([20] * 3, plateau=16) == 20
    import pytest
    with pytest.raises(ValueError):
        P.suggest_max_total_rank([])
    # two-step sweeps: order 3, large enough to be past launch-bound rounds, intermediate within the budget
    assert P.suggest_two_step((1000, 1000, 1000), 420) and P.suggest_two_step((4000, 200, 50), 640)
    assert not P.suggest_two_step((32, 32, 32), 30) and P.suggest_two_step((180, 180, 180, 180), 420)
    assert not P.suggest_two_step((180, 180, 180, 180), 2048)      # 96 GB intermediate: over the default budget
    assert not P.suggest_two_step((100, 40000, 40000), 64)
    # a short first mode: the intermediate (I2*I3 x width) is many times the tensor, its passes cost more than they save
    assert not P.suggest_two_step((50, 200, 4000), 640) and P.suggest_two_step((200, 50, 4000), 64)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_launch_plan_invariants_on_the_host(tmp_path):
    # host logic of the fused MTTKRP: tile shape, column blocks and split of the contraction range for ~2 300 000
    # shapes (grid of boundary values plus pseudo-random ones); compiled against the built library, no GPU touched
    import shutil
    import subprocess
    import pytest
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not available")
    exe = str(tmp_path / "plan_check")
    src = os.path.join(ROOT, "tests", "host", "plan_check.cpp")
    libdir = os.path.dirname(binding.library_path())
    r = subprocess.run(["hipcc", "-O1", "-o", exe, src, "-L" + libdir, "-lcals_hip", "-Wl,-rpath," + libdir],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.startswith("ok "), r.stdout[-500:]
