"""Seeded generators for every synthetic input of the speculative-decoding step.

Nothing here computes any part of the method (no norm, attention, softmax, sampling rule):
only shapes, seeds and draws.  Tensors are torch tensors on the requested device so that the
7B-sized inputs can be drawn directly in HBM; callers that feed the CPU oracle copy them to
host memory and widen them to float64 themselves.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class ModelCfg:
    name: str
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    mlp: int
    vocab: int
    rms_eps: float = 1e-6
    rope_theta: float = 1e6
    page_size: int = 16

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def qkv_dim(self) -> int:
        return self.q_dim + 2 * self.kv_dim

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def gemm_params(self) -> int:
        per_layer = self.hidden * self.qkv_dim + self.q_dim * self.hidden + 3 * self.hidden * self.mlp
        return per_layer * self.n_layers + self.hidden * self.vocab

    def kv_bytes_per_token(self, elt_bytes: int) -> int:
        return 2 * self.n_layers * self.kv_dim * elt_bytes


# Shapes of the five workloads: a tiny fp32 decoder, a mid-sized decoder that spans several GEMM
# and attention tiles while staying cheap for the CPU oracle, and the 7B / 32B Qwen2.5 shapes.
TINY = ModelCfg("tiny", 2, 256, 4, 2, 64, 768, 1024)
MID = ModelCfg("mid", 3, 512, 8, 2, 128, 1280, 4096)
QWEN7B = ModelCfg("qwen2.5-7b-shape", 28, 3584, 28, 4, 128, 18944, 152064)
QWEN32B = ModelCfg("qwen2.5-32b-shape", 64, 5120, 40, 8, 128, 27648, 152064)
LLAMA70B = ModelCfg("llama-3.3-70b-shape", 80, 8192, 64, 8, 128, 28672, 128256)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _normal(shape, std, seed, device, dtype):
    g = _gen(device, seed)
    t = torch.empty(shape, device=device, dtype=torch.float32)
    t.normal_(0.0, std, generator=g)
    return t.to(dtype)


def _gain(n, seed, device, dtype, jitter):
    g = _gen(device, seed)
    t = torch.empty((n,), device=device, dtype=torch.float32)
    t.normal_(0.0, jitter, generator=g)
    return (1.0 + t).to(dtype)


def _layer(cfg: ModelCfg, seed: int, device, dtype, std, jitter, qkv_bias=False):
    h, F = cfg.hidden, cfg.mlp
    bias = {"bqkv": _normal((cfg.qkv_dim,), 10 * std, seed + 8, device, dtype)} if qkv_bias else {}
    return {
        **bias,
        "attn_norm": _gain(h, seed + 1, device, dtype, jitter),
        "wqkv": _normal((cfg.qkv_dim, h), std, seed + 2, device, dtype),
        "wo": _normal((h, cfg.q_dim), std, seed + 3, device, dtype),
        "mlp_norm": _gain(h, seed + 4, device, dtype, jitter),
        "wg": _normal((F, h), std, seed + 5, device, dtype),
        "wu": _normal((F, h), std, seed + 6, device, dtype),
        "wd": _normal((h, F), std, seed + 7, device, dtype),
    }


def make_decoder_weights(cfg: ModelCfg, seed: int, device="cpu", dtype=torch.float32, std=0.02,
                         norm_jitter=0.1, n_layers=None, qkv_bias=False):
    """Random-init decoder: every matrix iid N(0, std^2), norm gains 1 + N(0, norm_jitter^2);
    qkv_bias adds a bias N(0, (10 std)^2) on the query/key/value projections.

    Matrices are stored [out_features, in_features] row-major.  `wqkv` stacks the q heads, then
    the k heads, then the v heads along the output dimension.  One seed per tensor, derived from
    (seed, layer, tensor), so any layer can be regenerated on its own.
    """
    L = cfg.n_layers if n_layers is None else n_layers
    base = seed * 100003
    return {
        "embed": _normal((cfg.vocab, cfg.hidden), std, base + 11, device, dtype),
        "lm_head": _normal((cfg.vocab, cfg.hidden), std, base + 12, device, dtype),
        "final_norm": _gain(cfg.hidden, base + 13, device, dtype, norm_jitter),
        "layers": [_layer(cfg, base + 1000 * (l + 1), device, dtype, std, norm_jitter, qkv_bias) for l in range(L)],
    }


def make_drafter_weights(cfg: ModelCfg, seed: int, device="cpu", dtype=torch.float32, std=0.02,
                         norm_jitter=0.1):
    """Single-decoder-layer drafter of the target's width plus the 2h->h input projection `fc`
    (columns 0..h-1 multiply the token embedding, columns h..2h-1 the hidden state)."""
    base = seed * 100003 + 500000
    return {
        "fc": _normal((cfg.hidden, 2 * cfg.hidden), std, base + 21, device, dtype),
        "layer": _layer(cfg, base + 1000, device, dtype, std, norm_jitter),
    }


def lognormal_contexts(batch: int, median: float, sigma: float, cap: int, floor: int, seed: int) -> np.ndarray:
    """Long-tailed context lengths: exp(N(ln median, sigma^2)) rounded, clipped to [floor, cap]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = np.exp(rng.normal(math.log(median), sigma, size=batch))
    return np.clip(np.rint(x), floor, cap).astype(np.int32)


def uniform_contexts(batch: int, lo: int, hi: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(lo, hi + 1, size=batch).astype(np.int32)


def pages_needed(lengths, page_size: int) -> np.ndarray:
    return (np.asarray(lengths, dtype=np.int64) + page_size - 1) // page_size


def random_block_table(capacities, page_size: int, seed: int, extra_pages: int = 0):
    """Assign every sequence enough pages for `capacities[b]` tokens, as a random permutation of
    the pool's page ids (so consecutive logical pages are scattered in memory).

    Returns (block_table [B, max_pages] int32 with -1 padding, n_pages_total)."""
    need = pages_needed(capacities, page_size)
    total = int(need.sum()) + int(extra_pages)
    rng = np.random.Generator(np.random.PCG64(seed))
    perm = rng.permutation(total).astype(np.int32)
    B, mp = len(need), int(need.max())
    table = np.full((B, mp), -1, dtype=np.int32)
    o = 0
    for b in range(B):
        table[b, : need[b]] = perm[o : o + need[b]]
        o += int(need[b])
    return table, total


def fill_kv_pool(n_layers: int, n_pages: int, n_kv_heads: int, page_size: int, head_dim: int, seed: int,
                 device="cpu", dtype=torch.float32, std=1.0):
    """K and V pools [n_layers, n_pages, n_kv_heads, page_size, head_dim] filled with N(0, std^2)."""
    shape = (n_layers, n_pages, n_kv_heads, page_size, head_dim)
    k = torch.empty(shape, device=device, dtype=dtype)
    v = torch.empty(shape, device=device, dtype=dtype)
    gk, gv = _gen(device, seed * 7 + 1), _gen(device, seed * 7 + 2)
    for l in range(n_layers):  # per layer, to bound the fp32 staging buffer
        k[l] = torch.empty(shape[1:], device=device, dtype=torch.float32).normal_(0.0, std, generator=gk).to(dtype)
        v[l] = torch.empty(shape[1:], device=device, dtype=torch.float32).normal_(0.0, std, generator=gv).to(dtype)
    return k, v


def prompts(batch: int, length: int, vocab: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, vocab, size=(batch, length)).astype(np.int32)


def uniforms_u32(shape, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, 2**32, size=shape, dtype=np.uint64).astype(np.uint32)


def synthetic_logits(shape, seed: int, std: float = 1.5) -> np.ndarray:
    """fp32 logits ~ N(0, std^2), used where the acceptance rule is tested apart from the model."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return (rng.standard_normal(size=shape, dtype=np.float32) * np.float32(std)).astype(np.float32)
