"""Thin ctypes binding of libtlt.so: same names as the C ABI, argument marshalling only.

torch is used for device memory and streams; every step of the path runs in the library's HIP
kernels.  There is no CPU fallback: loading fails loudly when the library has not been built
(`python -m paper_2511_16665_amd.build`).
"""
from __future__ import annotations

import ctypes as C
import dataclasses
import os
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtlt.so")

TLT_F32, TLT_BF16 = 0, 1
ERRORS = {0: "TLT_OK", -1: "TLT_EINVAL", -2: "TLT_ESHAPE", -3: "TLT_ENOPAGES", -4: "TLT_EHIP", -5: "TLT_ENOTIMPL",
          -6: "TLT_ESYNC"}

EXPORTS = [
    "tlt_strerror", "tlt_last_hip_error", "tlt_workspace_bytes", "tlt_create", "tlt_destroy", "tlt_draft_expand",
    "tlt_tree_finalize", "tlt_verify_forward", "tlt_accept", "tlt_kv_commit", "tlt_gemm", "tlt_set_attention_impl",
    "tlt_profile_begin", "tlt_profile_read", "tlt_mab_create", "tlt_mab_destroy", "tlt_mab_select", "tlt_mab_record",
    "tlt_mab_median_reward", "tlt_ngram_create", "tlt_ngram_destroy", "tlt_ngram_insert", "tlt_ngram_propose",
    "tlt_template_build", "tlt_draft_sample", "tlt_gemm_argmax", "tlt_gemm_glu", "tlt_draft_pool", "tlt_set_oproj_rounding", "tlt_device_status", "tlt_accept_sample_static", "tlt_attention", "tlt_attention_workspace_bytes",
    "tlt_graph_pool_create", "tlt_graph_pool_destroy", "tlt_graph_pool_step", "tlt_graph_pool_count", "tlt_mfma_stream",
]


class TltError(RuntimeError):
    def __init__(self, code, where, hip=0):
        self.code = code
        super().__init__(f"{where}: {ERRORS.get(code, code)}" + (f" (hipError {hip})" if hip else ""))


class ModelCfgC(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "mlp", "vocab")] + \
        [("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32), ("page_size", C.c_int32)]


class LayerWeightsC(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("attn_norm", "wqkv", "wo", "mlp_norm", "wg", "wu", "wd", "bqkv")]


class WeightsC(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("layers", C.POINTER(LayerWeightsC)), ("fc", C.c_void_p)]


class StrategyC(C.Structure):
    _fields_ = [("draft_depth", C.c_int32), ("topk", C.c_int32), ("tokens_to_verify", C.c_int32)]


class KVC(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("n_pages", C.c_int64), ("block_table", C.c_void_p),
                ("seq_len", C.c_void_p), ("max_pages", C.c_int32), ("seq_len_bound", C.c_int32)]


class TreeC(C.Structure):
    _fields_ = [("token", C.c_void_p), ("parent", C.c_void_p), ("depth", C.c_void_p), ("anc_mask", C.c_void_p),
                ("score", C.c_void_p), ("n", C.c_int32)]


class StepArgsC(C.Structure):
    _fields_ = [("new_tokens", C.c_void_p), ("new_src", C.c_void_p), ("n_new", C.c_void_p), ("new_stride", C.c_int32),
                ("hidden", C.c_void_p), ("hidden_n", C.c_int32), ("draft_kv", C.POINTER(KVC)), ("tree", C.POINTER(TreeC)),
                ("kv", C.POINTER(KVC)), ("argmax", C.c_void_p), ("hidden_out", C.c_void_p), ("stride", C.c_int32),
                ("accept_len", C.c_void_p), ("path_idx", C.c_void_p), ("out_tokens", C.c_void_p), ("n_out", C.c_void_p)]


_lib = None


def load() -> C.CDLL:
    """Loads libtlt.so; raises if it is missing (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2511_16665_amd.build`")
    lib = C.CDLL(LIB_PATH)
    lib.tlt_strerror.restype = C.c_char_p
    lib.tlt_workspace_bytes.restype = C.c_size_t
    lib.tlt_workspace_bytes.argtypes = [C.POINTER(ModelCfgC)] + [C.c_int] * 5
    lib.tlt_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(ModelCfgC), C.POINTER(WeightsC), C.POINTER(WeightsC)] + \
        [C.c_int] * 5 + [C.c_void_p, C.c_size_t]
    lib.tlt_destroy.argtypes = [C.c_void_p]
    lib.tlt_last_hip_error.argtypes = [C.c_void_p]
    lib.tlt_draft_expand.argtypes = [C.c_void_p, C.c_void_p] + [C.c_int] * 5 + [C.c_void_p] * 3 + [C.c_int, C.c_void_p, C.c_int,
                                                                                         C.c_void_p, C.POINTER(KVC),
                                                                                         C.POINTER(TreeC)]
    lib.tlt_draft_pool.argtypes = [C.c_void_p, C.c_void_p] + [C.c_int] * 3 + [C.c_void_p] * 3
    lib.tlt_template_build.argtypes = [C.c_int] * 3 + [C.POINTER(C.c_int32)] * 4
    lib.tlt_draft_sample.argtypes = [C.c_void_p, C.c_void_p] + [C.c_int] * 4 + [C.c_float] + [C.c_void_p] * 3 + \
        [C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.POINTER(KVC), C.c_void_p, C.POINTER(TreeC), C.c_void_p]
    lib.tlt_tree_finalize.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.POINTER(TreeC)]
    lib.tlt_graph_pool_create.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int, C.c_int, C.POINTER(C.c_void_p)]
    lib.tlt_graph_pool_destroy.argtypes = [C.c_void_p]
    lib.tlt_graph_pool_step.argtypes = [C.c_void_p, C.c_void_p] + [C.c_int] * 4 + [C.POINTER(StepArgsC)]
    lib.tlt_graph_pool_count.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.tlt_verify_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.POINTER(TreeC), C.POINTER(KVC)] + [C.c_void_p] * 4
    lib.tlt_accept.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_float, C.POINTER(TreeC)] + [C.c_void_p] * 5 + \
        [C.c_int] + [C.c_void_p] * 4
    lib.tlt_accept_sample_static.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_float, C.POINTER(TreeC)] + [C.c_void_p] * 4 + \
        [C.c_int] + [C.c_void_p] * 5
    lib.tlt_kv_commit.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.POINTER(KVC), C.c_void_p, C.c_void_p, C.c_int]
    lib.tlt_gemm.argtypes = [C.c_void_p] + [C.c_int] * 5 + [C.c_void_p] * 3
    lib.tlt_gemm_glu.argtypes = [C.c_void_p] + [C.c_int] * 3 + [C.c_void_p] * 4
    lib.tlt_gemm_argmax.argtypes = [C.c_void_p] + [C.c_int] * 3 + [C.c_void_p] * 3 + [C.c_size_t, C.c_void_p]
    lib.tlt_mfma_stream.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
    lib.tlt_set_attention_impl.argtypes = [C.c_void_p, C.c_int]
    lib.tlt_attention_workspace_bytes.restype = C.c_size_t
    lib.tlt_attention_workspace_bytes.argtypes = [C.c_int] * 6
    lib.tlt_attention.argtypes = [C.c_void_p] + [C.c_int] * 7 + [C.c_void_p, C.c_void_p, C.POINTER(KVC), C.c_void_p, C.c_void_p,
                                                               C.c_size_t, C.c_int]
    lib.tlt_set_oproj_rounding.argtypes = [C.c_void_p, C.c_int]
    lib.tlt_device_status.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_uint32)]
    lib.tlt_profile_begin.argtypes = [C.c_void_p, C.c_int]
    lib.tlt_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_double),
                                     C.POINTER(C.c_double)]
    lib.tlt_mab_create.argtypes = [C.POINTER(StrategyC), C.c_int, C.POINTER(C.c_int32), C.c_int, C.c_double, C.c_int, C.c_int,
                                   C.POINTER(C.c_void_p)]
    lib.tlt_mab_destroy.argtypes = [C.c_void_p]
    lib.tlt_mab_destroy.restype = None
    lib.tlt_mab_select.argtypes = [C.c_void_p, C.c_int, C.c_uint32, C.c_uint32, C.POINTER(C.c_int32)]
    lib.tlt_mab_record.argtypes = [C.c_void_p, C.c_int, C.c_double, C.POINTER(C.c_int32), C.c_int, C.POINTER(C.c_double),
                                   C.POINTER(C.c_double)]
    lib.tlt_mab_median_reward.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int32)]
    lib.tlt_ngram_create.argtypes = [C.c_int, C.POINTER(C.c_void_p)]
    lib.tlt_ngram_destroy.argtypes = [C.c_void_p]
    lib.tlt_ngram_destroy.restype = None
    lib.tlt_ngram_insert.argtypes = [C.c_void_p, C.c_int64, C.POINTER(C.c_int32), C.c_int]
    lib.tlt_ngram_propose.argtypes = [C.c_void_p, C.c_int64, C.POINTER(C.c_int32), C.c_int, C.c_int, C.c_int, C.c_int,
                                      C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_float)]
    _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA/HIP tensors"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def torch_dtype(dtype_code: int):
    return torch.float32 if dtype_code == TLT_F32 else torch.bfloat16


@dataclasses.dataclass
class KV:
    """Paged KV cache of one model: pools [L, n_pages, Hkv, page, d], block_table [B, max_pages] int32,
    seq_len [B] int32 (device), seq_len_bound = host-known upper bound of seq_len."""
    k_pool: torch.Tensor
    v_pool: torch.Tensor
    block_table: torch.Tensor
    seq_len: torch.Tensor
    seq_len_bound: int

    def c(self) -> KVC:
        assert self.block_table.dtype == torch.int32 and self.seq_len.dtype == torch.int32
        return KVC(_ptr(self.k_pool), _ptr(self.v_pool), self.k_pool.shape[1], _ptr(self.block_table), _ptr(self.seq_len),
                   self.block_table.shape[1], int(self.seq_len_bound))


@dataclasses.dataclass
class Tree:
    """Token tree, device tensors [B, n]: token/parent/depth int32, anc_mask int64 (bit pattern), score fp32."""
    token: torch.Tensor
    parent: torch.Tensor
    depth: torch.Tensor
    anc_mask: torch.Tensor
    score: torch.Tensor

    @staticmethod
    def empty(B: int, n: int, device="cuda") -> "Tree":
        i32 = lambda: torch.zeros((B, n), dtype=torch.int32, device=device)
        return Tree(i32(), i32(), i32(), torch.zeros((B, n), dtype=torch.int64, device=device),
                    torch.zeros((B, n), dtype=torch.float32, device=device))

    @property
    def n(self) -> int:
        return self.token.shape[1]

    def c(self) -> TreeC:
        return TreeC(_ptr(self.token), _ptr(self.parent), _ptr(self.depth), _ptr(self.anc_mask), _ptr(self.score), self.n)


def _weights_c(w: dict, n_layers: int, fc=None, keep=None):
    layers = (LayerWeightsC * n_layers)()
    src = w["layers"] if "layers" in w else [w["layer"]]
    for i in range(n_layers):
        for k, _ in LayerWeightsC._fields_:
            if k in src[i]:                 # (bqkv is optional: a missing entry stays NULL)
                setattr(layers[i], k, src[i][k].data_ptr())
    keep.append(layers)
    return layers


class Context:
    """tlt_create / tlt_destroy plus the step's calls as methods with the C names."""

    def __init__(self, cfg, dtype_code: int, target: dict, draft: Optional[dict], max_batch: int, max_n: int,
                 max_depth: int, max_topk: int, max_ctx: int):
        lib = load()
        self.lib = lib
        self.cfg = cfg
        self.dtype_code = dtype_code
        self.ccfg = ModelCfgC(cfg.n_layers, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.mlp, cfg.vocab,
                              cfg.rms_eps, cfg.rope_theta, dtype_code, cfg.page_size)
        nbytes = lib.tlt_workspace_bytes(C.byref(self.ccfg), max_batch, max_n, max_depth, max_topk, max_ctx)
        if nbytes == 0:
            raise TltError(-1, "tlt_workspace_bytes")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self._keep = [target, draft]
        tl = _weights_c(target, cfg.n_layers, keep=self._keep)
        tw = WeightsC(target["embed"].data_ptr(), target["lm_head"].data_ptr(), target["final_norm"].data_ptr(), tl, None)
        dw_ref = None
        if draft is not None:
            dl = _weights_c(draft, 1, keep=self._keep)
            dw = WeightsC(target["embed"].data_ptr(), target["lm_head"].data_ptr(), target["final_norm"].data_ptr(), dl,
                          draft["fc"].data_ptr())
            dw_ref = C.byref(dw)
        self.handle = C.c_void_p()
        rc = lib.tlt_create(C.byref(self.handle), C.byref(self.ccfg), C.byref(tw), dw_ref, max_batch, max_n, max_depth,
                            max_topk, max_ctx, _ptr(self.workspace), nbytes)
        if rc:
            raise TltError(rc, "tlt_create")

    def close(self):
        if self.handle:
            torch.cuda.synchronize()
            self.lib.tlt_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc, where):
        if rc:
            raise TltError(rc, where, self.lib.tlt_last_hip_error(self.handle))

    def draft_expand(self, B, depth, topk, n_verify, new_tokens, new_src, n_new, hidden, root_tokens, draft_kv: KV,
                     out_tree: Optional[Tree], mode=0):
        new_stride = 0 if new_tokens is None else new_tokens.shape[1]
        hidden_n = 0 if hidden is None else hidden.shape[1]
        kvc = draft_kv.c()
        tree_ref = None
        if out_tree is not None:
            tc = out_tree.c()
            tree_ref = C.byref(tc)
        self._check(self.lib.tlt_draft_expand(self.handle, _stream(), B, depth, topk, n_verify, mode, _ptr(new_tokens),
                                              _ptr(new_src), _ptr(n_new), new_stride, _ptr(hidden), hidden_n,
                                              _ptr(root_tokens), C.byref(kvc), tree_ref), "tlt_draft_expand")

    def draft_pool(self, B, depth, topk):
        """(token, parent, score) device tensors [B, topk + (depth-1)*topk^2] of the last expansion's pool."""
        n = topk + (depth - 1) * topk * topk
        token, parent = (torch.empty((B, n), dtype=torch.int32, device="cuda") for _ in range(2))
        score = torch.empty((B, n), dtype=torch.float32, device="cuda")
        self._check(self.lib.tlt_draft_pool(self.handle, _stream(), B, depth, topk, _ptr(token), _ptr(parent), _ptr(score)),
                    "tlt_draft_pool")
        return token, parent, score

    def draft_sample(self, B, depth, topk, n_verify, temperature, new_tokens, new_src, n_new, hidden, root_tokens,
                     draft_kv: KV, u_draw, out_tree: Tree, out_draft_q):
        new_stride = 0 if new_tokens is None else new_tokens.shape[1]
        hidden_n = 0 if hidden is None else hidden.shape[1]
        kvc, tc = draft_kv.c(), out_tree.c()
        self._check(self.lib.tlt_draft_sample(self.handle, _stream(), B, depth, topk, n_verify, temperature,
                                              _ptr(new_tokens), _ptr(new_src), _ptr(n_new), new_stride, _ptr(hidden),
                                              hidden_n, _ptr(root_tokens), C.byref(kvc), _ptr(u_draw), C.byref(tc),
                                              _ptr(out_draft_q)), "tlt_draft_sample")

    def tree_finalize(self, B, tree: Tree):
        tc = tree.c()
        self._check(self.lib.tlt_tree_finalize(self.handle, _stream(), B, C.byref(tc)), "tlt_tree_finalize")

    def verify_forward(self, B, tree: Tree, kv: KV, out_logits=None, out_argmax=None, out_hidden=None, out_lse=None):
        tc, kvc = tree.c(), kv.c()
        self._check(self.lib.tlt_verify_forward(self.handle, _stream(), B, C.byref(tc), C.byref(kvc), _ptr(out_logits),
                                                _ptr(out_argmax), _ptr(out_lse), _ptr(out_hidden)), "tlt_verify_forward")

    def accept(self, B, mode, temperature, tree: Tree, target_logits, target_argmax, draft_q, u_accept, u_final, stride,
               accept_len, path_idx, out_tokens, n_out):
        tc = tree.c()
        self._check(self.lib.tlt_accept(self.handle, _stream(), B, mode, temperature, C.byref(tc), _ptr(target_logits),
                                        _ptr(target_argmax), _ptr(draft_q), _ptr(u_accept), _ptr(u_final), stride,
                                        _ptr(accept_len), _ptr(path_idx), _ptr(out_tokens), _ptr(n_out)), "tlt_accept")

    def kv_commit(self, B, kv: KV, accept_len, path_idx, stride):
        kvc = kv.c()
        self._check(self.lib.tlt_kv_commit(self.handle, _stream(), B, C.byref(kvc), _ptr(accept_len), _ptr(path_idx), stride),
                    "tlt_kv_commit")

    def set_attention_impl(self, impl: int):
        self._check(self.lib.tlt_set_attention_impl(self.handle, impl), "tlt_set_attention_impl")

    def device_status(self, check=True):
        """Synchronises the current stream and returns the device-side status bits (cleared by the call);
        with check=True a raised bit becomes a TltError (TLT_ESHAPE / TLT_ESYNC)."""
        flags = C.c_uint32()
        rc = self.lib.tlt_device_status(self.handle, _stream(), C.byref(flags))
        if check:
            self._check(rc, "tlt_device_status")
        return flags.value

    def set_oproj_rounding(self, round_to_model_dtype: bool):
        self._check(self.lib.tlt_set_oproj_rounding(self.handle, int(round_to_model_dtype)), "tlt_set_oproj_rounding")

    def profile_begin(self, enable=True):
        """enable: True/1 = start afresh, 2 = resume without dropping records, False/0 = pause."""
        self._check(self.lib.tlt_profile_begin(self.handle, int(enable)), "tlt_profile_begin")

    def profile_read(self):
        ms, n, fl, by = (C.c_double * 6)(), (C.c_int64 * 6)(), (C.c_double * 6)(), (C.c_double * 6)()
        self._check(self.lib.tlt_profile_read(self.handle, ms, n, fl, by), "tlt_profile_read")
        names = ("gemm", "attention", "kv_commit", "other", "gemm_draft", "attention_draft")
        return {k: {"ms": ms[i], "launches": n[i], "flops": fl[i], "bytes": by[i]} for i, k in enumerate(names)}


def accept_sample_static(B, vocab, temperature, tree: Tree, target_logits, draft_q, u_accept, u_final, stride, accept_len,
                         path_idx, out_tokens, n_out, status=None):
    """tlt_accept_sample_static: sampling acceptance on the library's static scratch; returns the library's code."""
    tc = tree.c()
    return load().tlt_accept_sample_static(_stream(), B, vocab, temperature, C.byref(tc), _ptr(target_logits), _ptr(draft_q),
                                           _ptr(u_accept), _ptr(u_final), stride, _ptr(accept_len), _ptr(path_idx),
                                           _ptr(out_tokens), _ptr(n_out), _ptr(status))


def template_build(topk: int, depth: int, n_verify: int):
    """Static tree template of sampled drafting: (parent, rank, depth) int32 arrays (host side)."""
    lib = load()
    par, rank, dep = (np.zeros(n_verify, dtype=np.int32) for _ in range(3))
    n = C.c_int32(0)
    p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    rc = lib.tlt_template_build(topk, depth, n_verify, p(par), p(rank), p(dep), C.byref(n))
    if rc:
        raise TltError(rc, "tlt_template_build")
    return par[: n.value].copy(), rank[: n.value].copy(), dep[: n.value].copy()


class Mab:
    """tlt_mab_*: the strategy selector (host only).  strategies: (Draft_Depth, topK, Tokens_to_Verify) tuples."""

    def __init__(self, strategies, thresholds, epsilon, window, sd_threshold=32):
        arr = (StrategyC * len(strategies))(*[StrategyC(*map(int, s)) for s in strategies])
        thr = (C.c_int32 * len(thresholds))(*map(int, thresholds))
        self.h = C.c_void_p()
        rc = load().tlt_mab_create(arr, len(strategies), thr, len(thresholds), float(epsilon), int(window),
                                   int(sd_threshold), C.byref(self.h))
        if rc:
            raise TltError(rc, "tlt_mab_create")

    def select(self, batch_size, u1, u2):
        """Strategy index, or None while speculation is switched off for this batch size."""
        out = C.c_int32()
        rc = load().tlt_mab_select(self.h, int(batch_size), int(u1), int(u2), C.byref(out))
        if rc:
            raise TltError(rc, "tlt_mab_select")
        return None if out.value < 0 else out.value

    def record(self, strategy, elapsed_time, accept_lens, batch_size):
        a, r = C.c_double(), C.c_double()
        lens = (C.c_int32 * len(accept_lens))(*map(int, accept_lens))
        rc = load().tlt_mab_record(self.h, int(strategy), float(elapsed_time), lens, int(batch_size), C.byref(a), C.byref(r))
        if rc:
            raise TltError(rc, "tlt_mab_record")
        return a.value, r.value

    def median_reward(self, strategy):
        m, n = C.c_double(), C.c_int32()
        rc = load().tlt_mab_median_reward(self.h, int(strategy), C.byref(m), C.byref(n))
        if rc:
            raise TltError(rc, "tlt_mab_median_reward")
        return m.value, n.value

    def close(self):
        if self.h:
            load().tlt_mab_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class NGram:
    """tlt_ngram_*: the model-free drafter (host only)."""

    def __init__(self, order):
        self.h = C.c_void_p()
        rc = load().tlt_ngram_create(int(order), C.byref(self.h))
        if rc:
            raise TltError(rc, "tlt_ngram_create")

    def insert(self, prompt_id, tokens):
        arr = np.ascontiguousarray(tokens, dtype=np.int32)
        rc = load().tlt_ngram_insert(self.h, int(prompt_id), arr.ctypes.data_as(C.POINTER(C.c_int32)), len(arr))
        if rc:
            raise TltError(rc, "tlt_ngram_insert")

    def propose(self, prompt_id, context, depth, topk, n_nodes):
        """(token [n], parent [n], score [n]) numpy arrays of the proposed tree."""
        ctx = np.ascontiguousarray(context, dtype=np.int32)
        token, parent = np.empty(n_nodes, np.int32), np.empty(n_nodes, np.int32)
        score = np.empty(n_nodes, np.float32)
        rc = load().tlt_ngram_propose(self.h, int(prompt_id), ctx.ctypes.data_as(C.POINTER(C.c_int32)), len(ctx), int(depth),
                                      int(topk), int(n_nodes), token.ctypes.data_as(C.POINTER(C.c_int32)),
                                      parent.ctypes.data_as(C.POINTER(C.c_int32)), score.ctypes.data_as(C.POINTER(C.c_float)))
        if rc:
            raise TltError(rc, "tlt_ngram_propose")
        return token, parent, score

    def close(self):
        if self.h:
            load().tlt_ngram_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def gemm(dtype_code, out_mode, A, W, Cout):
    """tlt_gemm: Cout[M, N] (op)= A[M, K] . W[N, K]^T on device tensors."""
    M, K = A.shape
    N = W.shape[0]
    rc = load().tlt_gemm(_stream(), dtype_code, out_mode, M, N, K, _ptr(A), _ptr(W), _ptr(Cout))
    if rc:
        raise TltError(rc, "tlt_gemm")


def attention_workspace(B, n, n_q_heads, n_kv_heads, head_dim, max_ctx) -> torch.Tensor:
    nbytes = load().tlt_attention_workspace_bytes(B, n, n_q_heads, n_kv_heads, head_dim, max_ctx)
    if nbytes == 0:
        raise TltError(-1, "tlt_attention_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device="cuda")


def attention(dtype_code, n_q_heads, page_size, qkv, anc_mask, kv: KV, out, ws, impl=-1):
    """tlt_attention on one layer's pools [n_pages, Hkv, page, d]; qkv [B, n, (Hq+2Hkv)*d]; returns the code."""
    B, n = qkv.shape[0], qkv.shape[1]
    n_kv, d = kv.k_pool.shape[-3], kv.k_pool.shape[-1]
    kvc = KVC(_ptr(kv.k_pool), _ptr(kv.v_pool), kv.k_pool.shape[-4], _ptr(kv.block_table), _ptr(kv.seq_len),
              kv.block_table.shape[1], int(kv.seq_len_bound))
    return load().tlt_attention(_stream(), dtype_code, B, n, n_q_heads, n_kv, d, page_size, _ptr(qkv), _ptr(anc_mask),
                                C.byref(kvc), _ptr(out), _ptr(ws), ws.numel(), impl)


def gemm_argmax(A, W, ws, out):
    """out[m] = argmax_n (A W^T)[m, n] for bf16 device tensors A [M, K], W [N, K]; returns the library's code."""
    M, K = A.shape
    N = W.shape[0]
    return load().tlt_gemm_argmax(_stream(), M, N, K, _ptr(A), _ptr(W), _ptr(ws), ws.numel() * ws.element_size(), _ptr(out))


def gemm_glu(A, Wg, Wu, act):
    """act = silu(A Wg^T) * (A Wu^T) for bf16 device tensors A [M, K], Wg/Wu [N, K], act [M, N]; returns the code."""
    M, K = A.shape
    return load().tlt_gemm_glu(_stream(), M, Wg.shape[0], K, _ptr(A), _ptr(Wg), _ptr(Wu), _ptr(act))


def mfma_stream(frags, out, iters):
    """tlt_mfma_stream: `iters` rounds of a wave tile's 64 MFMAs on the register fragments read from `frags` (bf16
    device tensor of 16384 values), every lane's accumulator sum to `out` (fp32 device tensor of 65536); returns the code."""
    assert frags.numel() * frags.element_size() == 32768 and out.numel() == 65536 and out.element_size() == 4
    return load().tlt_mfma_stream(_stream(), _ptr(frags), _ptr(out), int(iters))


class GraphPool:
    """tlt_graph_pool_*: the library's HIP-graph pool (greedy step per batch bucket, drafter and target graphs
    apart).  The caller's tensors must stay alive and in place for as long as their graphs are replayed."""

    def __init__(self, ctx: "Context", buckets, seq_len_bound: int):
        self.ctx = ctx
        self.lib = ctx.lib
        arr = (C.c_int32 * len(buckets))(*buckets)
        self.handle = C.c_void_p()
        rc = self.lib.tlt_graph_pool_create(ctx.handle, arr, len(buckets), int(seq_len_bound), C.byref(self.handle))
        if rc:
            raise TltError(rc, "tlt_graph_pool_create", self.lib.tlt_last_hip_error(ctx.handle))

    def step(self, B, depth, topk, n_verify, new_tokens, new_src, n_new, hidden, draft_kv: "KV", tree: "Tree", kv: "KV",
             argmax, hidden_out, stride, accept_len, path_idx, out_tokens, n_out):
        dkv_c, kv_c, tree_c = draft_kv.c(), kv.c(), tree.c()
        a = StepArgsC(_ptr(new_tokens), _ptr(new_src), _ptr(n_new), new_tokens.shape[1], _ptr(hidden), hidden.shape[1],
                      C.pointer(dkv_c), C.pointer(tree_c), C.pointer(kv_c), _ptr(argmax), _ptr(hidden_out), stride,
                      _ptr(accept_len), _ptr(path_idx), _ptr(out_tokens), _ptr(n_out))
        rc = self.lib.tlt_graph_pool_step(self.handle, _stream(), B, depth, topk, n_verify, C.byref(a))
        if rc:
            raise TltError(rc, "tlt_graph_pool_step", self.lib.tlt_last_hip_error(self.ctx.handle))

    def count(self):
        nd, nt = C.c_int32(), C.c_int32()
        rc = self.lib.tlt_graph_pool_count(self.handle, C.byref(nd), C.byref(nt))
        if rc:
            raise TltError(rc, "tlt_graph_pool_count")
        return nd.value, nt.value

    def close(self):
        if self.handle:
            torch.cuda.synchronize()
            self.lib.tlt_graph_pool_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
