"""The C-ABI library loads and exports every symbol that include/mj.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mj.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mj_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = declared_functions()
    for must in ("mj_init", "mj_step", "mj_legal_mask", "mj_observe", "mj_reward", "mj_reset_done",
                 "mj_sample_random", "mj_step_random", "mj_export", "mj_import", "mj_eval_hands", "mj_destroy"):
        assert must in names


def test_library_exports_every_declared_symbol():
    so = os.path.join(ROOT, "paper_2605_20577_amd", "libmj.so")
    if not os.path.exists(so):
        from paper_2605_20577_amd import build
        build.build()
    lib = ctypes.CDLL(so)
    for name in declared_functions():
        assert hasattr(lib, name), name
    import paper_2605_20577_amd.binding as b
    assert sorted(b.EXPORTS) == declared_functions()
    lib.mj_strerror.restype = ctypes.c_char_p
    assert lib.mj_strerror(-1) == b"bad argument"
    r = b.MjRules(12, 0, 25000, -1.0, 2)
    assert b.mj_state_bytes(65536, r) == 65536 * 1156 and b.mj_state_bytes(0, r) == 0
    assert 0 < b.mj_scratch_bytes(1, r) < 32 << 20          # tables only (8 MB of shanten block tables, 8 MB of pattern neighbours), independent of B


def test_binding_refuses_to_run_without_the_library(monkeypatch):
    import paper_2605_20577_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_SO", os.path.join(ROOT, "no_such_dir", "libmj.so"))
    with pytest.raises(RuntimeError):
        b.lib()


def test_binding_constants_mirror_the_header():
    import re
    import paper_2605_20577_amd as mj
    text = open(os.path.join(os.path.dirname(__file__), "..", "include", "mj.h")).read()
    assert int(re.search(r"#define\s+MJ_ROLLOUT_CHUNK\s+(\d+)", text).group(1)) == mj.ROLLOUT_CHUNK


def test_bench_refuses_more_than_one_gpu():
    """this build runs on one GPU: bench.py --gpus N with N > 1 says so and exits without touching a device"""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
