"""Verification forward at the shapes of the other workloads (two decoder blocks each, reduced
vocabulary: the full-vocabulary LM head is covered by test_gpu_fullsize.py), sampled sequences
against the oracle:

* long-tail phase: 7B block shape (28 query / 4 kv heads, 7 query heads per kv head), 4 sequences at
  24k-32k context, trees of 64 nodes with depth <= 8 and at most 10 children per node
  (448 query rows per kv head: two row groups of three row tiles per wave, 6-7 work items per sequence);
* 32B block shape (40 query / 8 kv heads, 5 per kv head, hidden 5120, MLP 27648), 16 sequences with
  lognormal contexts (median 8k, cap 32k), trees of 32 nodes (160 rows per kv head: two row tiles per wave);
* 70B block shape of the paper's largest target (64 query / 8 kv heads, 8 per kv head, hidden 8192,
  MLP 28672), with a bias on the q/k/v projections switched on to cover that path at width, 8
  sequences, trees of 32 nodes (256 rows per kv head).
"""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import decoder as dec
from oracle import sd
from paper_2511_16665_amd import binding as tlt
from paper_2511_16665_amd import engine as eng
from synth import (LLAMA70B, QWEN7B, QWEN32B, fill_kv_pool, lognormal_contexts, make_decoder_weights, random_block_table)

from gpu_util import EmbedRows, LazyLayers, dense_cache, rel_err

pytestmark = pytest.mark.gpu

TOL = 2e-2


def _bounded_tree(rng, n, vocab, max_depth, max_children):
    parent, depth, kids = [-1], [0], [0]
    for i in range(1, n):
        while True:
            p = int(rng.integers(max(0, i - 12), i))
            if depth[p] < max_depth and kids[p] < max_children:
                break
        parent.append(p)
        depth.append(depth[p] + 1)
        kids[p] += 1
        kids.append(0)
    return sd.Tree(rng.integers(0, vocab, size=n), np.array(parent), np.array(depth), np.zeros(n))


def _run(cfg, ctx, n, max_depth, max_children, sample, seed, qkv_bias=False, std=0.02):
    B = len(ctx)
    rng = np.random.default_rng(seed)
    table, n_pages = random_block_table(ctx + n + 16, cfg.page_size, seed=seed, extra_pages=8)
    dt = torch.bfloat16
    tw = make_decoder_weights(cfg, 77, device="cuda", dtype=dt, qkv_bias=qkv_bias, std=std)
    k, v = fill_kv_pool(cfg.n_layers, n_pages, cfg.n_kv_heads, cfg.page_size, cfg.head_dim, seed + 1, "cuda", dt)
    k0, v0 = k.clone(), v.clone()
    kv = eng.alloc_kv(cfg, tlt.TLT_BF16, cfg.n_layers, table, n_pages, ctx, fill=(k, v))
    c = tlt.Context(cfg, tlt.TLT_BF16, tw, None, B, n, 8, 10, int(ctx.max()) + n + 64)
    trees = [_bounded_tree(rng, n, cfg.vocab, max_depth, max_children) for _ in range(B)]
    t = tlt.Tree.empty(B, n)
    t.token.copy_(torch.tensor(np.stack([tr.token for tr in trees]), dtype=torch.int32))
    t.parent.copy_(torch.tensor(np.stack([tr.parent for tr in trees]), dtype=torch.int32))
    c.tree_finalize(B, t)
    hidden = torch.zeros((B, n, cfg.hidden), dtype=torch.float32, device="cuda")
    logits = torch.zeros((B, n, cfg.vocab), dtype=torch.float32, device="cuda")
    print(f"verify {cfg.name} B={B} n={n} contexts {int(ctx.min())}..{int(ctx.max())}", flush=True)
    c.verify_forward(B, t, kv, logits, None, hidden)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(t.depth.cpu().numpy(), np.stack([tr.depth for tr in trees]))
    tw64 = {"embed": EmbedRows(tw["embed"]), "lm_head": dec.weights_to_f64(tw["lm_head"]),
            "final_norm": dec.weights_to_f64(tw["final_norm"]), "layers": LazyLayers(tw["layers"])}
    for b in sample:
        cb = int(ctx[b])
        print(f" oracle on sequence {b} (context {cb})", flush=True)
        st = sd.SeqState(cfg, cb + n, dec.round_to_bf16)
        for l in range(cfg.n_layers):
            st.target[l].k[:cb] = dense_cache(k0[l:l + 1], table, b, cb, cfg.page_size)[0]
            st.target[l].v[:cb] = dense_cache(v0[l:l + 1], table, b, cb, cfg.page_size)[0]
        st.ctx = cb
        want_logits, want_hidden = sd.verify(cfg, tw64, st, trees[b])
        e_h, e_l = rel_err(hidden[b].cpu().numpy(), want_hidden), rel_err(logits[b].cpu().numpy(), want_logits)
        print(f"  rel err hidden {e_h:.3e} logits {e_l:.3e}", flush=True)
        assert e_h <= TOL and e_l <= TOL
        for l in range(cfg.n_layers):
            kn = dense_cache(kv.k_pool[l:l + 1], table, b, cb + n, cfg.page_size)[0]
            vn = dense_cache(kv.v_pool[l:l + 1], table, b, cb + n, cfg.page_size)[0]
            assert rel_err(kn[cb:], st.target[l].k[cb:cb + n]) <= TOL and rel_err(vn[cb:], st.target[l].v[cb:cb + n]) <= TOL
            np.testing.assert_array_equal(kn[:cb], st.target[l].k[:cb])          # committed rows untouched
    c.close()


def test_long_tail_shape_7b_blocks_24k_to_32k_context_tree_64():
    cfg = dataclasses.replace(QWEN7B, name="7b-blocks-x2", n_layers=2, vocab=4096)
    ctx = np.array([24576, 32000, 27001, 30719], dtype=np.int32)
    _run(cfg, ctx, 64, 8, 10, sample=[1, 2], seed=11)


def test_32b_block_shape_lognormal_contexts_tree_32():
    cfg = dataclasses.replace(QWEN32B, name="32b-blocks-x2", n_layers=2, vocab=4096)
    ctx = lognormal_contexts(16, 8192, 0.8, 32768, 256, seed=3)
    order = np.argsort(ctx)
    _run(cfg, ctx, 32, 6, 8, sample=[int(order[0]), int(order[len(order) // 2])], seed=13)


def test_70b_block_shape_with_qkv_bias_tree_32():
    cfg = dataclasses.replace(LLAMA70B, name="70b-blocks-x2", n_layers=2, vocab=4096)
    ctx = lognormal_contexts(8, 4096, 0.8, 16384, 256, seed=5)
    order = np.argsort(ctx)
    # weights N(0, 0.013^2): the 7B shape's 0.02 scaled by sqrt(3584 / 8192), so that queries and keys
    # (and with them the sharpness of the attention, which sets how much a bf16 rounding of q or k
    # moves the output) have the size they have there
    _run(cfg, ctx, 32, 6, 8, sample=[int(order[0]), int(order[len(order) // 2])], seed=17, qkv_bias=True, std=0.013)
