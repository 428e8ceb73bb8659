"""Oracle decoder: a pre-norm transformer decoder written out in float64 numpy.

Test infrastructure only (see the package docstring).  The paper names the model family
(Qwen2.5, Section 6.1 "Models") and the drafter's shape (one decoder block that reuses the
target's embedding and LM head, Section 4.1 "Model Architecture") but prints no equations for
the block, so the block below is the textbook definition of that family's decoder layer:

    x <- x + Wo . Attn(RoPE(Wq n1(x)), RoPE(Wk n1(x)), Wv n1(x))
    x <- x + Wd . (SiLU(Wg n2(x)) * Wu n2(x))
    logits = Wlm . nf(x),   n(x) = x / sqrt(mean(x^2) + eps) * gamma

with grouped-query attention (query head j reads kv head j // G), scores scaled by 1/sqrt(d),
rotary embedding in the rotate-half convention (element i pairs with i + d/2), no biases.

Pins (tests/test_oracle_decoder.py): rmsnorm, SiLU-gated MLP and causal GQA attention against
torch's library routines; RoPE against its closed form for d = 2, norm preservation and the
relative-position property; `dense_forward` (cache-free) against a torch assembly of library
routines; the cached/tree path `forward_rows` against `dense_forward` on every root-to-node path.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------- containers
def weights_to_f64(w):
    """Recursively turn a dict/list of torch tensors (any dtype/device) into float64 numpy."""
    if isinstance(w, dict):
        return {k: weights_to_f64(v) for k, v in w.items()}
    if isinstance(w, (list, tuple)):
        return [weights_to_f64(v) for v in w]
    if isinstance(w, np.ndarray):
        return w.astype(np.float64)
    return w.detach().to("cpu").double().numpy()


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bfloat16 (ties to even), returned as float64.

    The cache is model state held in the model's storage type, so in bf16 mode the oracle rounds
    what it stores there; activations stay float64."""
    f = np.ascontiguousarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(x.shape)


def identity(x):
    return x


# ----------------------------------------------------------------------------- pieces
def rmsnorm(x, gamma, eps):
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * gamma


def silu(x):
    return x / (1.0 + np.exp(-x))


def rope(x, pos, theta):
    """x [n, H, d], pos [n] -> rotated copy.  Pair (i, i + d/2) turns by pos * theta^(-2i/d)."""
    d = x.shape[-1]
    half = d // 2
    inv_freq = theta ** (-(2.0 * np.arange(half, dtype=np.float64)) / d)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def attention(q, K, V, visible):
    """q [n, Hq, d]; K, V [T, Hkv, d]; visible [n, T] bool.  Returns [n, Hq, d].

    Row i is a softmax over exactly the keys with visible[i] set."""
    n, Hq, d = q.shape
    G = Hq // K.shape[1]
    out = np.zeros_like(q)
    for j in range(Hq):
        kh = j // G
        s = (q[:, j, :] @ K[:, kh, :].T) / np.sqrt(float(d))
        s = np.where(visible, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, j, :] = p @ V[:, kh, :]
    return out


def mlp(cfg, w, x):
    return (silu(x @ w["wg"].T) * (x @ w["wu"].T)) @ w["wd"].T


# ----------------------------------------------------------------------------- cache-free definition
def qkv_projection(lw, xn):
    """Query/key/value projection; `bqkv` (optional) is the additive bias that the Qwen2.5 family of
    Section 6.1's target models carries on exactly these three projections."""
    qkv = xn @ lw["wqkv"].T
    return qkv + lw["bqkv"] if "bqkv" in lw else qkv


def dense_forward(cfg, w, tokens, n_layers=None):
    """Textbook causal forward of the whole token sequence with no cache.

    Returns (logits [T, V], hidden [T, h] = last block's output before the final norm,
    keys [L, T, Hkv, d], values [L, T, Hkv, d])."""
    tokens = np.asarray(tokens, dtype=np.int64)
    T = len(tokens)
    pos = np.arange(T)
    causal = pos[None, :] <= pos[:, None]
    x = w["embed"][tokens]
    ks, vs = [], []
    layers = w["layers"] if n_layers is None else w["layers"][:n_layers]
    for lw in layers:
        xn = rmsnorm(x, lw["attn_norm"], cfg.rms_eps)
        qkv = qkv_projection(lw, xn)
        q = qkv[:, : cfg.q_dim].reshape(T, cfg.n_q_heads, cfg.head_dim)
        k = qkv[:, cfg.q_dim : cfg.q_dim + cfg.kv_dim].reshape(T, cfg.n_kv_heads, cfg.head_dim)
        v = qkv[:, cfg.q_dim + cfg.kv_dim :].reshape(T, cfg.n_kv_heads, cfg.head_dim)
        q = rope(q, pos, cfg.rope_theta)
        k = rope(k, pos, cfg.rope_theta)
        ks.append(k)
        vs.append(v)
        a = attention(q, k, v, causal).reshape(T, cfg.q_dim)
        x = x + a @ lw["wo"].T
        x = x + mlp(cfg, lw, rmsnorm(x, lw["mlp_norm"], cfg.rms_eps))
    logits = rmsnorm(x, w["final_norm"], cfg.rms_eps) @ w["lm_head"].T
    return logits, x, np.stack(ks), np.stack(vs)


# ----------------------------------------------------------------------------- cached / tree path
class LayerCache:
    """Keys and values of one sequence in one layer, dense: row s = token slot s."""

    def __init__(self, cfg, capacity):
        self.k = np.zeros((capacity, cfg.n_kv_heads, cfg.head_dim))
        self.v = np.zeros((capacity, cfg.n_kv_heads, cfg.head_dim))


def block_rows(cfg, lw, x, pos, slots, visible, cache: LayerCache, store=identity):
    """One decoder block over n new rows of one sequence.

    x [n, h]; pos [n] rotary positions; slots [n] cache rows the new keys/values are written to;
    visible [n, T] says which cache rows 0..T-1 (T > max slot) each new row may attend to."""
    n = x.shape[0]
    xn = rmsnorm(x, lw["attn_norm"], cfg.rms_eps)
    qkv = qkv_projection(lw, xn)
    q = qkv[:, : cfg.q_dim].reshape(n, cfg.n_q_heads, cfg.head_dim)
    k = qkv[:, cfg.q_dim : cfg.q_dim + cfg.kv_dim].reshape(n, cfg.n_kv_heads, cfg.head_dim)
    v = qkv[:, cfg.q_dim + cfg.kv_dim :].reshape(n, cfg.n_kv_heads, cfg.head_dim)
    q = rope(q, pos, cfg.rope_theta)
    k = rope(k, pos, cfg.rope_theta)
    cache.k[slots] = store(k)
    cache.v[slots] = store(v)
    T = visible.shape[1]
    a = attention(q, cache.k[:T], cache.v[:T], visible).reshape(n, cfg.q_dim)
    x = x + a @ lw["wo"].T
    x = x + mlp(cfg, lw, rmsnorm(x, lw["mlp_norm"], cfg.rms_eps))
    return x


def lm_logits(cfg, w, x):
    return rmsnorm(x, w["final_norm"], cfg.rms_eps) @ w["lm_head"].T


def log_softmax(z):
    z = z - z.max(axis=-1, keepdims=True)
    return z - np.log(np.exp(z).sum(axis=-1, keepdims=True))
