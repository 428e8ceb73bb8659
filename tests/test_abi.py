"""The C-ABI library loads without a GPU and exports every function include/tlt.h declares."""
import ctypes
import os
import re

import pytest

from paper_2511_16665_amd import binding


def _declared_functions(header_text):
    text = re.sub(r"/\*.*?\*/", "", header_text, flags=re.S)
    return sorted(set(re.findall(r"\b(tlt_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(repo_root):
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_16665_amd import build
        build.build(verbose=False)
    header = open(os.path.join(repo_root, "include", "tlt.h")).read()
    names = _declared_functions(header)
    assert {"tlt_draft_expand", "tlt_verify_forward", "tlt_accept", "tlt_kv_commit"} <= set(names)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in names:
        assert hasattr(lib, name), f"{name} declared in tlt.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_host_side_validation_needs_no_gpu():
    lib = binding.load()
    assert lib.tlt_strerror(0) == b"ok"
    assert b"block table" in lib.tlt_strerror(-3)
    cfg = binding.ModelCfgC(2, 256, 4, 2, 64, 768, 1024, 1e-6, 1e6, 0, 16)
    assert lib.tlt_workspace_bytes(ctypes.byref(cfg), 2, 4, 4, 1, 256) > 0
    assert lib.tlt_workspace_bytes(ctypes.byref(cfg), 2, 65, 4, 1, 256) == 0      # tree larger than 64 nodes
    bad = binding.ModelCfgC(2, 256, 4, 3, 64, 768, 1024, 1e-6, 1e6, 0, 16)         # 4 q heads over 3 kv heads
    assert lib.tlt_workspace_bytes(ctypes.byref(bad), 2, 4, 4, 1, 256) == 0
    out = ctypes.c_void_p()
    assert lib.tlt_create(ctypes.byref(out), ctypes.byref(cfg), None, None, 2, 4, 4, 1, 256, None, 0) == -1
    assert lib.tlt_destroy(None) == -1
    assert lib.tlt_gemm(None, 0, 0, 4, 4, 4, None, None, None) == -1


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="not found"):
        binding.load()
