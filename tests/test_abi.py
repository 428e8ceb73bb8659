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


def test_draft_expand_rejects_more_provisional_rows_than_a_mask_holds():
    """(depth-1)*topk provisional drafter rows are one bit each of a 128-bit visibility mask: a
    depth/topk pair inside the published per-argument limits (16 each) but beyond 128 rows must
    be refused on the host, before anything is enqueued (no GPU is touched here)."""
    lib = binding.load()
    cfg = binding.ModelCfgC(1, 256, 4, 2, 64, 768, 1024, 1e-6, 1e6, 0, 16)
    fake = 0x10000      # never dereferenced: validation returns first
    layers = (binding.LayerWeightsC * 1)()
    for k, _ in binding.LayerWeightsC._fields_:
        setattr(layers[0], k, fake)
    tw = binding.WeightsC(fake, fake, fake, layers, None)
    dw = binding.WeightsC(fake, fake, fake, layers, fake)
    nbytes = lib.tlt_workspace_bytes(ctypes.byref(cfg), 2, 64, 16, 16, 4096)
    assert nbytes > 0
    h = ctypes.c_void_p()
    assert lib.tlt_create(ctypes.byref(h), ctypes.byref(cfg), ctypes.byref(tw), ctypes.byref(dw), 2, 64, 16, 16, 4096,
                          ctypes.c_void_p(fake), nbytes) == 0
    kv = binding.KVC(fake, fake, 1024, fake, fake, 300, 100)
    tree = binding.TreeC(fake, fake, fake, fake, fake, 64)
    call = lambda depth, topk: lib.tlt_draft_expand(h, None, 2, depth, topk, 64, 0, None, None, None, 0, None, 0,
                                                    ctypes.c_void_p(fake), ctypes.byref(kv), ctypes.byref(tree))
    assert call(10, 16) == -2            # 144 rows
    assert call(16, 16) == -2
    assert call(9, 17) == -2             # topk beyond the context's limit
    # the graph pool's bucket list is checked on the host as well, before a stream is created
    pool = ctypes.c_void_p()
    mk = lambda *b: lib.tlt_graph_pool_create(h, (ctypes.c_int32 * len(b))(*b), len(b), 1000, ctypes.byref(pool))
    assert mk() == -1                    # no bucket
    assert mk(1, 1) == -1                # not increasing
    assert mk(1, 4) == -1                # beyond the context's batch of 2
    assert lib.tlt_graph_pool_step(None, None, 1, 1, 1, 2, None) == -1
    assert lib.tlt_graph_pool_destroy(None) == 0
    assert lib.tlt_destroy(h) == 0
