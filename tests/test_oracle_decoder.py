"""Pins of the oracle's decoder pieces against library routines, closed forms and invariants."""
import dataclasses
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import decoder as dec
from synth import TINY, make_decoder_weights

SMALL = dataclasses.replace(TINY, name="small", hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16, mlp=96,
                            vocab=50, n_layers=2)


def test_rmsnorm_matches_torch_library():
    rng = np.random.default_rng(0)
    x = rng.normal(size=(5, 64))
    g = rng.normal(size=64)
    want = F.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), eps=1e-6).numpy()
    np.testing.assert_allclose(dec.rmsnorm(x, g, 1e-6), want, rtol=1e-12, atol=1e-12)


def test_gated_mlp_matches_torch_library():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(3, 64))
    w = {"wg": rng.normal(size=(96, 64)), "wu": rng.normal(size=(96, 64)), "wd": rng.normal(size=(64, 96))}
    tx = torch.from_numpy(x)
    want = F.linear(F.silu(F.linear(tx, torch.from_numpy(w["wg"]))) * F.linear(tx, torch.from_numpy(w["wu"])),
                    torch.from_numpy(w["wd"])).numpy()
    np.testing.assert_allclose(dec.mlp(SMALL, w, x), want, rtol=1e-11, atol=1e-11)


def test_causal_gqa_attention_matches_torch_sdpa():
    rng = np.random.default_rng(2)
    T, Hq, Hkv, d = 9, 6, 2, 16
    q, k, v = rng.normal(size=(T, Hq, d)), rng.normal(size=(T, Hkv, d)), rng.normal(size=(T, Hkv, d))
    causal = np.tril(np.ones((T, T), dtype=bool))
    got = dec.attention(q, k, v, causal)
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (q, k, v))
    want = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True, enable_gqa=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)


def test_attention_arbitrary_mask_matches_torch_sdpa():
    rng = np.random.default_rng(3)
    n, T, Hq, Hkv, d = 5, 11, 4, 2, 8
    q, k, v = rng.normal(size=(n, Hq, d)), rng.normal(size=(T, Hkv, d)), rng.normal(size=(T, Hkv, d))
    vis = rng.random((n, T)) < 0.5
    vis[:, 0] = True
    got = dec.attention(q, k, v, vis)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (k, v))
    want = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=torch.from_numpy(vis), enable_gqa=True)[0]
    np.testing.assert_allclose(got, want.permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)


def test_rope_closed_form_d2_and_d4():
    # d = 2: a single pair turning by pos * theta^0 = pos radians.
    x = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    got = dec.rope(x, np.array([3, 3]), 10000.0)
    np.testing.assert_allclose(got[0, 0], [math.cos(3), math.sin(3)], atol=1e-15)
    np.testing.assert_allclose(got[1, 0], [-math.sin(3), math.cos(3)], atol=1e-15)
    # d = 4, theta = 10000: pairs (0,2) at 1 rad/position and (1,3) at 0.01 rad/position.
    y = dec.rope(np.array([[[1.0, 2.0, 3.0, 4.0]]]), np.array([5]), 10000.0)[0, 0]
    a, b = 5.0, 0.05
    want = [1 * math.cos(a) - 3 * math.sin(a), 2 * math.cos(b) - 4 * math.sin(b),
            3 * math.cos(a) + 1 * math.sin(a), 4 * math.cos(b) + 2 * math.sin(b)]
    np.testing.assert_allclose(y, want, atol=1e-14)


def test_rope_invariants():
    rng = np.random.default_rng(4)
    q, k = rng.normal(size=(1, 1, 32)), rng.normal(size=(1, 1, 32))
    np.testing.assert_allclose(dec.rope(q, np.array([0]), 1e6), q, atol=0)
    np.testing.assert_allclose(np.linalg.norm(dec.rope(q, np.array([777]), 1e6)), np.linalg.norm(q), rtol=1e-12)
    dots = [float(np.sum(dec.rope(q, np.array([m]), 1e6) * dec.rope(k, np.array([m - 5]), 1e6))) for m in (5, 90, 4000)]
    np.testing.assert_allclose(dots, dots[0], rtol=1e-9)


def _torch_reference_forward(cfg, w, tokens):
    """The same decoder assembled from torch library routines (complex-number rotary)."""
    t = lambda a: torch.from_numpy(np.asarray(a))
    T = len(tokens)
    x = F.embedding(torch.tensor(tokens), t(w["embed"]))
    half = cfg.head_dim // 2
    inv = torch.pow(torch.tensor(cfg.rope_theta, dtype=torch.float64), -torch.arange(half, dtype=torch.float64) / half)
    rot = torch.polar(torch.ones(T, half, dtype=torch.float64), torch.arange(T, dtype=torch.float64)[:, None] * inv)

    def rotary(z):  # z [T, H, d]
        zc = torch.complex(z[..., :half], z[..., half:]) * rot[:, None, :]
        return torch.cat([zc.real, zc.imag], dim=-1)

    for lw in w["layers"]:
        xn = F.rms_norm(x, (cfg.hidden,), t(lw["attn_norm"]), eps=cfg.rms_eps)
        qkv = F.linear(xn, t(lw["wqkv"]), t(lw["bqkv"]) if "bqkv" in lw else None)
        q, k, v = torch.split(qkv, [cfg.q_dim, cfg.kv_dim, cfg.kv_dim], dim=-1)
        q = rotary(q.reshape(T, cfg.n_q_heads, cfg.head_dim)).permute(1, 0, 2)[None]
        k = rotary(k.reshape(T, cfg.n_kv_heads, cfg.head_dim)).permute(1, 0, 2)[None]
        v = v.reshape(T, cfg.n_kv_heads, cfg.head_dim).permute(1, 0, 2)[None]
        a = F.scaled_dot_product_attention(q, k, v, is_causal=True, enable_gqa=True)[0].permute(1, 0, 2).reshape(T, -1)
        x = x + F.linear(a, t(lw["wo"]))
        xn = F.rms_norm(x, (cfg.hidden,), t(lw["mlp_norm"]), eps=cfg.rms_eps)
        x = x + F.linear(F.silu(F.linear(xn, t(lw["wg"]))) * F.linear(xn, t(lw["wu"])), t(lw["wd"]))
    return F.linear(F.rms_norm(x, (cfg.hidden,), t(w["final_norm"]), eps=cfg.rms_eps), t(w["lm_head"])).numpy(), x.numpy()


@pytest.mark.parametrize("std,bias", [(0.02, False), (0.3, False), (0.1, True)])
def test_dense_forward_matches_torch_assembly(std, bias):
    w = dec.weights_to_f64(make_decoder_weights(SMALL, seed=5, std=std, qkv_bias=bias))
    assert ("bqkv" in w["layers"][0]) == bias
    tokens = list(np.random.default_rng(6).integers(0, SMALL.vocab, size=12))
    logits, hidden, ks, vs = dec.dense_forward(SMALL, w, tokens)
    want_logits, want_hidden = _torch_reference_forward(SMALL, w, tokens)
    np.testing.assert_allclose(hidden, want_hidden, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(logits, want_logits, rtol=1e-9, atol=1e-11)
    assert ks.shape == (SMALL.n_layers, 12, SMALL.n_kv_heads, SMALL.head_dim)


def test_round_to_bf16_matches_torch():
    x = np.random.default_rng(7).normal(size=1000) * 3
    want = torch.from_numpy(x).float().to(torch.bfloat16).double().numpy()
    np.testing.assert_array_equal(dec.round_to_bf16(x), want)
