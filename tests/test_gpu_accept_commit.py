"""tlt_accept and tlt_kv_commit against the oracle, bit-exact on identical inputs."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import accept as oa
from oracle import sd
from paper_2511_16665_amd import binding as tlt
from synth import TINY, make_decoder_weights, random_block_table, synthetic_logits, uniforms_u32

pytestmark = pytest.mark.gpu


def _ctx(vocab, B, n, dtype=tlt.TLT_F32, cfg=TINY):
    cfg = dataclasses.replace(cfg, vocab=vocab, n_layers=1)
    dt = tlt.torch_dtype(dtype)
    w = make_decoder_weights(cfg, 1, device="cuda", dtype=dt)
    return cfg, tlt.Context(cfg, dtype, w, None, B, n, 8, 4, 4096)


def _random_trees(rng, B, n, V, branching=3, dup=False):
    token = rng.integers(0, V, size=(B, n)).astype(np.int32)
    parent = np.full((B, n), -1, dtype=np.int32)
    for b in range(B):
        for i in range(1, n):
            parent[b, i] = rng.integers(max(0, i - branching), i)
    return token, parent


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _tree_dev(token, parent):
    B, n = token.shape
    t = tlt.Tree.empty(B, n)
    t.token.copy_(_dev(token))
    t.parent.copy_(_dev(parent))
    return t


def _run_accept(ctx, B, n, stride, mode, tree, **kw):
    outs = [torch.full(s, -7, dtype=torch.int32, device="cuda") for s in ((B,), (B, stride), (B, stride), (B,))]
    ctx.accept(B, mode, kw.get("temperature", 1.0), tree, kw.get("logits"), kw.get("argmax"), kw.get("draft_q"),
               kw.get("u_accept"), kw.get("u_final"), stride, *outs)
    torch.cuda.synchronize()
    return [o.cpu().numpy() for o in outs]


@pytest.mark.parametrize("B,n,V,stride", [(64, 12, 5, 12), (3, 64, 1024, 9), (1, 1, 17, 1), (32, 48, 4099, 7)])
def test_greedy_accept_bit_exact(B, n, V, stride):
    rng = np.random.default_rng(B * 1000 + n)
    cfg, ctx = _ctx(V, B, n)
    token, parent = _random_trees(rng, B, n, V)
    logits = synthetic_logits((B, n, V), seed=n)
    if V == 5:
        logits = np.round(logits)                     # many exact ties: lowest index must win
    want = oa.accept_greedy(token, parent, logits, stride)
    print(f"greedy accept B={B} n={n} V={V}", flush=True)
    tree = _tree_dev(token, parent)
    got = _run_accept(ctx, B, n, stride, 0, tree, logits=_dev(logits))
    for g, w in zip(got, want):
        np.testing.assert_array_equal(g, w)
    # same through the argmax fast path
    am = torch.from_numpy(np.argmax(logits, axis=2).astype(np.int32)).cuda()
    got2 = _run_accept(ctx, B, n, stride, 0, tree, argmax=am)
    for g, w in zip(got2, want):
        np.testing.assert_array_equal(g, w)
    ctx.close()


@pytest.mark.parametrize("B,n,V,tau,k", [(256, 4, 16, 1.0, 2), (16, 21, 1000, 0.9, 4), (4, 64, 152064, 1.0, 3)])
def test_sampling_accept_bit_exact(B, n, V, tau, k):
    """Trees whose sibling lists are drawn without replacement from a noisy copy of the target
    distribution (sigma = 1 on the logits): the long-tail workload's drafter."""
    rng = np.random.default_rng(V + n)
    cfg, ctx = _ctx(V, B, n)
    logits = synthetic_logits((B, n, V), seed=7)
    ql = logits + rng.standard_normal(size=logits.shape).astype(np.float32)
    q = np.exp(ql - ql.max(axis=-1, keepdims=True))
    q = (q / q.sum(axis=-1, keepdims=True)).astype(np.float32)
    token = np.zeros((B, n), dtype=np.int32)
    parent = np.full((B, n), -1, dtype=np.int32)
    for b in range(B):                                 # breadth-first k-ary template
        nxt = 1
        for p in range(n):
            if nxt >= n:
                break
            kids = oa.draw_without_replacement(q[b, p], k, rng)
            for t in kids:
                if nxt < n:
                    token[b, nxt], parent[b, nxt] = t, p
                    nxt += 1
    u_acc, u_fin = uniforms_u32((B, n), 11), uniforms_u32((B,), 12)
    stride = 6
    *want, near = oa.accept_sample(token, parent, logits, q, u_acc, u_fin, tau, stride, with_near=True)
    assert want[0].max() >= 1
    print(f"sampling accept B={B} n={n} V={V}", flush=True)
    got = _run_accept(ctx, B, n, stride, 1, _tree_dev(token, parent), logits=_dev(logits), draft_q=_dev(q),
                      u_accept=_dev(u_acc), u_final=_dev(u_fin), temperature=tau)
    assert ctx.device_status() == 0
    # bit for bit, except where the oracle itself says a decision sat within 8 units of 2^-32 of its
    # threshold (a platform's last-bit `exp` can move a weight by one unit): those are reported
    differ = oa.assert_equal_unless_near(got, want, near, "sampling accept")
    print(f"  near-threshold sequences {int(near.sum())} of {B}, of which differing {len(differ)}", flush=True)
    assert near.sum() <= max(1, B // 8)
    ctx.close()


@pytest.mark.parametrize("mode", [1, 2])
def test_sampling_accept_root_only_tree_is_a_plain_draw(mode):
    """N = 1 (no speculation): both sampling rules reduce to one inverse-CDF draw from the target."""
    B, n, V, tau = 5, 1, 1031, 0.8
    cfg, ctx = _ctx(V, B, n)
    logits = synthetic_logits((B, n, V), seed=3)
    q = np.full((B, n, V), 1.0 / V, dtype=np.float32)
    token = np.zeros((B, n), dtype=np.int32)
    parent = np.full((B, n), -1, dtype=np.int32)
    u_acc, u_fin = uniforms_u32((B, n), 1), uniforms_u32((B,), 2)
    u_fin[0], u_fin[1] = 0, 2**32 - 1
    if mode == 1:
        want = oa.accept_sample(token, parent, logits, q, u_acc, u_fin, tau, 1)
    else:
        want = oa.accept_target_only(token, parent, logits, u_acc, u_fin, tau, 1)
    got = _run_accept(ctx, B, n, 1, mode, _tree_dev(token, parent), logits=_dev(logits), draft_q=_dev(q),
                      u_accept=_dev(u_acc), u_final=_dev(u_fin), temperature=tau)
    for g, w in zip(got, want):
        np.testing.assert_array_equal(g, w)
    assert (got[0] == 0).all() and (got[3] == 1).all()
    ctx.close()


@pytest.mark.parametrize("B,n,V,tau,k", [(256, 4, 16, 1.0, 2), (16, 21, 1000, 0.9, 4), (4, 64, 152064, 0.9, 3), (8, 64, 97, 0.7, 63)])
def test_target_only_sampling_accept_bit_exact(B, n, V, tau, k):
    """Deterministic top-k trees of a noisy copy of the target (the trees the target-only rule is
    for); the last case hangs 63 children (with repeated tokens) under the root."""
    rng = np.random.default_rng(V + n + 1)
    cfg, ctx = _ctx(V, B, n)
    logits = synthetic_logits((B, n, V), seed=8)
    if V == 16:
        logits = logits * 3                             # peaked targets: accepts happen often
    ql = logits + rng.standard_normal(size=logits.shape).astype(np.float32)
    token = np.zeros((B, n), dtype=np.int32)
    parent = np.full((B, n), -1, dtype=np.int32)
    for b in range(B):                                 # breadth-first k-ary tree of the k most likely tokens
        nxt = 1
        for p in range(n):
            if nxt >= n:
                break
            kids = np.argsort(-ql[b, p])[:k] if k <= V else rng.integers(0, V, size=k)
            if k == 63:
                kids = rng.integers(0, V, size=k)       # arbitrary tokens, some repeated
            for t in kids:
                if nxt < n:
                    token[b, nxt], parent[b, nxt] = t, p
                    nxt += 1
    u_acc, u_fin = uniforms_u32((B, n), 21), uniforms_u32((B,), 22)
    stride = 6
    *want, near = oa.accept_target_only(token, parent, logits, u_acc, u_fin, tau, stride, with_near=True)
    print(f"target-only accept B={B} n={n} V={V}: accept lengths up to {want[0].max()}", flush=True)
    got = _run_accept(ctx, B, n, stride, 2, _tree_dev(token, parent), logits=_dev(logits), u_accept=_dev(u_acc),
                      u_final=_dev(u_fin), temperature=tau)
    differ = oa.assert_equal_unless_near(got, want, near, "target-only accept")
    print(f"  near-threshold sequences {int(near.sum())} of {B}, of which differing {len(differ)}", flush=True)
    assert near.sum() <= max(1, B // 8)
    ctx.close()


@pytest.mark.parametrize("mode", [1, 2])
def test_sampling_accept_skips_children_whose_token_is_outside_the_vocabulary(mode):
    """Caller-made trees may carry -1 or tokens >= V: both rules skip such a child (never accepted,
    nothing else changes) instead of reading weights outside the row."""
    B, n, V, tau, stride = 6, 9, 517, 0.9, 5
    rng = np.random.default_rng(5)
    cfg, ctx = _ctx(V, B, n)
    logits = synthetic_logits((B, n, V), seed=4) * 2
    q = np.exp(logits - logits.max(axis=-1, keepdims=True))
    q = (q / q.sum(axis=-1, keepdims=True)).astype(np.float32)        # q = p: every in-range child is accepted
    token = rng.integers(0, V, size=(B, n)).astype(np.int32)
    parent = np.full((B, n), -1, dtype=np.int32)
    parent[:, 1:] = (np.arange(1, n) - 1) // 2                         # binary tree
    token[:, 1] = -1                                                   # the root's first child
    token[:, 3] = V                                                    # node 1's first child
    token[:, 5] = V + 1000
    token[0, 2] = 2**31 - 1
    u_acc, u_fin = uniforms_u32((B, n), 31), uniforms_u32((B,), 32)
    if mode == 1:
        want = oa.accept_sample(token, parent, logits, q, u_acc, u_fin, tau, stride)
    else:
        want = oa.accept_target_only(token, parent, logits, u_acc, u_fin, tau, stride)
    got = _run_accept(ctx, B, n, stride, mode, _tree_dev(token, parent), logits=_dev(logits), draft_q=_dev(q),
                      u_accept=_dev(u_acc), u_final=_dev(u_fin), temperature=tau)
    for g, w in zip(got, want):
        np.testing.assert_array_equal(g, w)
    for b in range(B):
        assert 1 not in got[1][b] and 3 not in got[1][b] and 5 not in got[1][b]
    ctx.close()


@pytest.mark.parametrize("dtype", [tlt.TLT_F32, tlt.TLT_BF16])
def test_kv_commit_bit_exact_and_touches_nothing_else(dtype):
    cfg = dataclasses.replace(TINY, n_layers=3)
    B, n, stride = 5, 24, 9
    rng = np.random.default_rng(0)
    ctxlen = np.array([0, 5, 16, 37, 100], dtype=np.int32)
    table, n_pages = random_block_table(ctxlen + n, cfg.page_size, seed=4, extra_pages=4)
    dt = tlt.torch_dtype(dtype)
    w = make_decoder_weights(cfg, 1, device="cuda", dtype=dt)
    ctx = tlt.Context(cfg, dtype, w, None, B, n, 8, 4, 4096)
    shape = (cfg.n_layers, n_pages, cfg.n_kv_heads, cfg.page_size, cfg.head_dim)
    k = torch.randn(shape, generator=torch.Generator().manual_seed(1)).to(dt)
    v = torch.randn(shape, generator=torch.Generator().manual_seed(2)).to(dt)
    # paths: strictly increasing node indices starting at the root, including the hazard 0,2,5 -> 0,1,2
    accept_len = np.array([0, 2, 8, 3, 5], dtype=np.int32)
    path = np.full((B, stride), -1, dtype=np.int32)
    path[:, 0] = 0
    path[1, :3] = [0, 2, 5]
    path[2, :9] = [0, 1, 2, 3, 4, 5, 6, 7, 8]          # identity: nothing moves
    path[3, :4] = [0, 3, 4, 23]
    path[4, :6] = [0, 1, 3, 7, 8, 16]                   # crosses a page boundary
    kv = tlt.KV(k.cuda(), v.cuda(), _dev(table), _dev(ctxlen), int(ctxlen.max()))
    print(f"kv_commit dtype={dtype}", flush=True)
    ctx.kv_commit(B, kv, _dev(accept_len), _dev(path), stride)
    torch.cuda.synchronize()
    # bf16 -> float64 is exact, so equality of the float64 images is bit equality
    k_want, v_want = k.double().numpy().copy(), v.double().numpy().copy()
    for b in range(B):
        slots = np.arange(ctxlen[b] + n)
        pg, off = table[b, slots // cfg.page_size], slots % cfg.page_size
        for l in range(cfg.n_layers):
            kd, vd = k_want[l][pg, :, off], v_want[l][pg, :, off]          # dense view [slots, Hkv, d] (copies)
            new_len = sd.commit_rows(kd, vd, int(ctxlen[b]), [int(p) for p in path[b, : accept_len[b] + 1]])
            assert new_len == ctxlen[b] + accept_len[b] + 1
            k_want[l][pg, :, off] = kd
            v_want[l][pg, :, off] = vd
    np.testing.assert_array_equal(kv.k_pool.double().cpu().numpy(), k_want)
    np.testing.assert_array_equal(kv.v_pool.double().cpu().numpy(), v_want)
    assert not np.array_equal(k_want, k.double().numpy())               # the case moved something
    np.testing.assert_array_equal(kv.seq_len.cpu().numpy(), ctxlen + accept_len + 1)
    ctx.close()
