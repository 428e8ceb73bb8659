"""ctypes wrapper over accept.c (the oracle's acceptance rules) plus the without-replacement draw
of sibling tokens that the sampling rule presupposes.

Test infrastructure only (see the package docstring).  The C file is compiled with gcc on first
use (and by the repository's build step); nothing here touches the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "accept.c")
_LIB = os.path.join(_HERE, "liboracle_accept.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-Wall", "-shared", "-fPIC",
                               _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a, t):
    return a.ctypes.data_as(ctypes.POINTER(t))


def _outputs(B, stride):
    return (np.zeros(B, np.int32), np.zeros((B, stride), np.int32), np.zeros((B, stride), np.int32),
            np.zeros(B, np.int32))


def accept_greedy(token, parent, logits, stride):
    """token, parent [B, n] int32; logits [B, n, V] float32.
    Returns accept_len [B], path_idx [B, stride], out_tokens [B, stride], n_out [B]; unused = -1."""
    token = np.ascontiguousarray(token, np.int32)
    parent = np.ascontiguousarray(parent, np.int32)
    logits = np.ascontiguousarray(logits, np.float32)
    B, n, V = logits.shape
    al, path, out, n_out = _outputs(B, stride)
    _load().oracle_accept_greedy(B, n, V, stride, _p(token, ctypes.c_int32), _p(parent, ctypes.c_int32),
                                 _p(logits, ctypes.c_float), _p(al, ctypes.c_int32), _p(path, ctypes.c_int32),
                                 _p(out, ctypes.c_int32), _p(n_out, ctypes.c_int32))
    return al, path, out, n_out


def accept_sample(token, parent, logits, draft_q, u_accept, u_final, temperature, stride, with_near=False):
    """with_near: also return near [B] int32, 1 where some decision of the sequence was within 8 units of
    2^-32 of going the other way (see accept.c): the only place a platform's last-bit `exp` can show."""
    token = np.ascontiguousarray(token, np.int32)
    parent = np.ascontiguousarray(parent, np.int32)
    logits = np.ascontiguousarray(logits, np.float32)
    draft_q = np.ascontiguousarray(draft_q, np.float32)
    u_accept = np.ascontiguousarray(u_accept, np.uint32)
    u_final = np.ascontiguousarray(u_final, np.uint32)
    B, n, V = logits.shape
    assert draft_q.shape == logits.shape and u_accept.shape == (B, n) and u_final.shape == (B,)
    al, path, out, n_out = _outputs(B, stride)
    near = np.zeros(B, np.int32)
    _load().oracle_accept_sample_near(B, n, V, stride, ctypes.c_float(temperature), _p(token, ctypes.c_int32),
                                      _p(parent, ctypes.c_int32), _p(logits, ctypes.c_float),
                                      _p(draft_q, ctypes.c_float), _p(u_accept, ctypes.c_uint32),
                                      _p(u_final, ctypes.c_uint32), _p(al, ctypes.c_int32),
                                      _p(path, ctypes.c_int32), _p(out, ctypes.c_int32), _p(n_out, ctypes.c_int32),
                                      _p(near, ctypes.c_int32))
    return (al, path, out, n_out, near) if with_near else (al, path, out, n_out)


def accept_target_only(token, parent, logits, u_accept, u_final, temperature, stride, with_near=False):
    """The rule for trees whose shape depends on the drafter's values (deterministic top-K trees).
    with_near: as in accept_sample."""
    token = np.ascontiguousarray(token, np.int32)
    parent = np.ascontiguousarray(parent, np.int32)
    logits = np.ascontiguousarray(logits, np.float32)
    u_accept = np.ascontiguousarray(u_accept, np.uint32)
    u_final = np.ascontiguousarray(u_final, np.uint32)
    B, n, V = logits.shape
    assert u_accept.shape == (B, n) and u_final.shape == (B,)
    al, path, out, n_out = _outputs(B, stride)
    near = np.zeros(B, np.int32)
    _load().oracle_accept_target_only_near(B, n, V, stride, ctypes.c_float(temperature), _p(token, ctypes.c_int32),
                                           _p(parent, ctypes.c_int32), _p(logits, ctypes.c_float),
                                           _p(u_accept, ctypes.c_uint32), _p(u_final, ctypes.c_uint32),
                                           _p(al, ctypes.c_int32), _p(path, ctypes.c_int32), _p(out, ctypes.c_int32),
                                           _p(n_out, ctypes.c_int32), _p(near, ctypes.c_int32))
    return (al, path, out, n_out, near) if with_near else (al, path, out, n_out)


def assert_equal_unless_near(got, want, near, what=""):
    """got/want: the four output arrays of an acceptance call.  Sequences whose oracle decisions were all
    clear of their thresholds must agree exactly; a flagged sequence may differ and is reported."""
    bad = []
    for b in range(len(near)):
        same = all(np.array_equal(np.asarray(g)[b], np.asarray(w)[b]) for g, w in zip(got, want))
        if not same:
            assert near[b], f"{what}: sequence {b} differs from the oracle although no decision was near a threshold"
            bad.append(b)
    return bad


def draw_without_replacement(q, k, rng):
    """k distinct tokens per row of q [..., V]: the first from q, the next from q with the first
    removed and renormalised, and so on (done with the Gumbel-top-k identity).  Sibling lists of a
    sampled tree must be drawn this way for the sampling acceptance rule to be lossless."""
    g = rng.gumbel(size=q.shape)
    with np.errstate(divide="ignore"):
        key = np.log(q) + g
    return np.argsort(-key, axis=-1)[..., :k]
