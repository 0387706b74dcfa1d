"""The C ABI library loads and exports every function include/pc.h declares;
the host-side argument checks reject bad calls without touching a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "pc.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(pc_[a-z_]+)\s*\(", src)))


def test_header_declares_the_six_calls():
    names = _declared()
    for n in ("pc_prefill_shared", "pc_decode_step", "pc_sample", "pc_group_stats", "pc_select_commit",
              "pc_advantages"):
        assert n in names


def test_library_exports_every_declared_symbol():
    from paper_2605_26606_amd import binding
    lib = binding.library()
    for n in _declared():
        assert hasattr(lib, n), n
    assert isinstance(lib.pc_last_error(), bytes)


def test_host_side_argument_checks_need_no_gpu():
    from paper_2605_26606_amd import binding
    lib = binding.library()
    # negative counts and null pointers are rejected before any HIP call
    assert lib.pc_group_stats(None, None, -1, None, None, None, None, None) == -1
    assert b"negative" in lib.pc_last_error()
    assert lib.pc_group_stats(None, None, 0, None, None, None, None, None) == 0
    assert lib.pc_group_stats(None, None, 3, None, None, None, None, None) == -1
    assert lib.pc_advantages(None, None, 2, 1e-6, None, None, None, None) == -1
    assert lib.pc_select_commit(None, 4, 0.125, 0.75, 1.0, 0, None, None, None, None, None, None) == -1
    one = np.zeros(4, np.int32)
    assert lib.pc_select_commit(one.ctypes.data, 4, 0.8, 0.75, 1.0, 0, None, None, one.ctypes.data, None,
                                one.ctypes.data, None) == -1      # p_lower > p_upper
    assert lib.pc_sample(None, None, 1, 16, 1.0, 1.0, 0, None, None, 0, -1, 0.0, None, None, None, None, None, None,
                         None) == -1
    assert lib.pc_sample(one.ctypes.data, None, 1, 16, 0.0, 1.0, 0, one.ctypes.data, None, 0, -1, 0.0,
                         one.ctypes.data, None, None, None, None, None, None) == -1   # temperature must be positive
    for bad_top_p in (0.0, 1.5, float("nan")):
        assert lib.pc_sample(one.ctypes.data, None, 1, 16, 1.0, bad_top_p, 0, one.ctypes.data, None, 0, -1, 0.0,
                             one.ctypes.data, None, None, None, None, None, None) == -1
        assert b"top_p" in lib.pc_last_error()
    assert lib.pc_saturation_count(None, None, 0) == -1
    assert lib.pc_create(None, None, None, None) == -1
    assert lib.pc_decode_step(None, None, None, 0, None, None) == -1
    assert lib.pc_destroy(None) == 0


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    from paper_2605_26606_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(ImportError):
        binding.library()
