"""tlt_verify_forward against the oracle on random trees over random paged caches."""
import numpy as np
import pytest
import torch

from oracle import decoder as dec
from oracle import sd
from paper_2511_16665_amd import binding as tlt
import dataclasses

from synth import MID, TINY, fill_kv_pool

MID7 = dataclasses.replace(MID, name="mid-g7", n_q_heads=14, n_layers=2)   # 7 query heads per kv head, as in the 7B shape

from gpu_util import dense_cache, make_engine, make_models, rel_err

pytestmark = pytest.mark.gpu


def _random_tree(rng, n, vocab):
    parent = np.array([-1] + [int(rng.integers(max(0, i - 4), i)) for i in range(1, n)])
    depth = np.zeros(n, dtype=np.int64)
    for i in range(1, n):
        depth[i] = depth[parent[i]] + 1
    return sd.Tree(rng.integers(0, vocab, size=n), parent, depth, np.zeros(n))


@pytest.mark.parametrize("cfg,dtype,tol,n,ctxs,std,impl", [
    (TINY, "fp32", 1e-4, 13, [0, 37, 150], 0.02, -1),
    (TINY, "fp32", 1e-4, 13, [0, 37, 150], 0.02, -2),     # with a bias on the q/k/v projections (impl -2 = automatic + bias)
    (MID7, "bf16", 2e-2, 48, [700, 90], 0.02, -2),
    (TINY, "fp32", 1e-4, 64, [1, 200], 0.1, -1),
    (TINY, "fp32", 1e-4, 1, [5, 64], 0.02, -1),           # N = 1: plain decode
    (MID, "bf16", 2e-2, 13, [0, 37, 150], 0.02, 0),       # wave-per-row attention in bf16
    (MID, "bf16", 2e-2, 13, [0, 37, 150], 0.02, 1),       # MFMA attention, 1 row tile per wave
    (MID, "bf16", 2e-2, 48, [300, 1100, 17], 0.02, 1),    # several key chunks / GEMM tiles, ragged
    (MID, "bf16", 2e-2, 1, [63, 64, 65, 1000], 0.02, 1),  # N = 1 on page and tile boundaries
    (MID7, "bf16", 2e-2, 48, [700, 90], 0.02, 1),         # 336 query rows per kv head: 3 row tiles per wave
    (MID7, "bf16", 2e-2, 64, [2100, 5], 0.05, 1),         # 448 rows: two row groups
])
def test_verify_forward_matches_oracle(cfg, dtype, tol, n, ctxs, std, impl):
    rng = np.random.default_rng(n)
    B = len(ctxs)
    ctxs = np.array(ctxs, dtype=np.int32)
    qkv_bias = impl == -2
    impl = max(impl, -1)
    tw_dev, dw_dev, tw, dw = make_models(cfg, 3, dtype, std=std, qkv_bias=qkv_bias)
    assert ("bqkv" in tw["layers"][0]) == qkv_bias
    cap = int(ctxs.max()) + n + 16
    e, table, _ = make_engine(cfg, dtype, tw_dev, dw_dev, B, n, 4, 2, cap, seed=5, seq_len=ctxs)
    dt = tlt.torch_dtype(e.ctx.dtype_code)
    k, v = fill_kv_pool(cfg.n_layers, e.kv.k_pool.shape[1], cfg.n_kv_heads, cfg.page_size, cfg.head_dim, seed=9, dtype=dt)
    e.kv.k_pool.copy_(k)
    e.kv.v_pool.copy_(v)
    trees = [_random_tree(rng, n, cfg.vocab) for _ in range(B)]
    t = e.tree(n)
    t.token.copy_(torch.tensor(np.stack([tr.token for tr in trees]), dtype=torch.int32))
    t.parent.copy_(torch.tensor(np.stack([tr.parent for tr in trees]), dtype=torch.int32))
    print(f"verify {cfg.name} {dtype} n={n} ctx={list(ctxs)}", flush=True)
    e.ctx.tree_finalize(B, t)
    e.ctx.set_attention_impl(impl)
    logits = torch.zeros((B, n, cfg.vocab), dtype=torch.float32, device="cuda")
    hidden = torch.zeros((B, n, cfg.hidden), dtype=torch.float32, device="cuda")
    argmax = torch.zeros((B, n), dtype=torch.int32, device="cuda")
    lse = torch.zeros((B, n, 2), dtype=torch.float32, device="cuda")
    e.ctx.verify_forward(B, t, e.kv, logits, argmax, hidden, out_lse=lse)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(t.depth.cpu().numpy(), np.stack([tr.depth for tr in trees]))
    np.testing.assert_array_equal(e.kv.seq_len.cpu().numpy(), ctxs)           # verify does not commit
    store = dec.identity if dtype == "fp32" else dec.round_to_bf16
    got_logits = logits.cpu().numpy()
    np.testing.assert_array_equal(argmax.cpu().numpy(), got_logits.argmax(axis=2))
    k_after, v_after = e.kv.k_pool, e.kv.v_pool
    for b in range(B):
        c = int(ctxs[b])
        st = sd.SeqState(cfg, c + n, store)
        kd, vd = dense_cache(k, table, b, c, cfg.page_size), dense_cache(v, table, b, c, cfg.page_size)
        for l in range(cfg.n_layers):
            st.target[l].k[:c], st.target[l].v[:c] = kd[l], vd[l]
        st.ctx = c
        want_logits, want_hidden = sd.verify(cfg, tw, st, trees[b])
        assert rel_err(got_logits[b], want_logits) <= tol, ("logits", b)
        # (largest logit, log-sum-exp) of every row against the plain definition on the oracle's logits
        want_max = want_logits.max(axis=1)
        want_lse = want_max + np.log(np.exp(want_logits - want_max[:, None]).sum(axis=1))
        got_lse = lse[b].cpu().numpy().astype(np.float64)
        scale = np.abs(want_logits).max()
        assert np.abs(got_lse[:, 0] - want_max).max() <= tol * scale and np.abs(got_lse[:, 1] - want_lse).max() <= tol * scale, ("lse", b)
        assert rel_err(hidden[b].cpu().numpy(), want_hidden) <= tol, ("hidden", b)
        kn, vn = dense_cache(k_after, table, b, c + n, cfg.page_size), dense_cache(v_after, table, b, c + n, cfg.page_size)
        for l in range(cfg.n_layers):
            assert rel_err(kn[l, c:], st.target[l].k[c:c + n]) <= tol, ("k rows", b, l)
            assert rel_err(vn[l, c:], st.target[l].v[c:c + n]) <= tol, ("v rows", b, l)
            np.testing.assert_array_equal(kn[l, :c], kd[l])                  # committed rows untouched
    e.ctx.close()


def test_verify_rejects_a_block_table_that_is_too_short():
    cfg = TINY
    tw_dev, dw_dev, tw, dw = make_models(cfg, 3, "fp32")
    e, table, _ = make_engine(cfg, "fp32", tw_dev, dw_dev, 1, 8, 4, 2, 64, seq_len=np.array([60], np.int32))
    t = e.tree(8)
    with pytest.raises(tlt.TltError, match="TLT_ENOPAGES"):
        e.ctx.verify_forward(1, t, e.kv, None, None, None)
    e.ctx.close()


def test_a_length_bound_below_the_device_side_lengths_is_reported():
    """seq_len lives on the device and the caller passes an upper bound that sizes the attention's work
    list: a bound below the real lengths cannot be seen on the host, would drop context rows, and is
    reported by tlt_device_status as TLT_ESHAPE (once; the word is cleared by the read)."""
    cfg = MID
    ctxs = np.array([700, 90], dtype=np.int32)
    tw_dev, dw_dev, tw, dw = make_models(cfg, 3, "bf16")
    e, table, _ = make_engine(cfg, "bf16", tw_dev, dw_dev, 2, 8, 4, 2, 900, seed=5, seq_len=ctxs)
    t = e.tree(8)
    t.token.fill_(1)
    t.parent.copy_(torch.arange(-1, 7, dtype=torch.int32, device="cuda").expand(2, 8))
    e.ctx.tree_finalize(2, t)
    print("verify with an honest bound", flush=True)
    e.ctx.verify_forward(2, t, e.kv, None, None, None)
    assert e.ctx.device_status() == 0
    print("verify with a bound of 500 for a sequence of 700", flush=True)
    e.kv.seq_len_bound = 500
    e.ctx.verify_forward(2, t, e.kv, None, None, None)
    with pytest.raises(tlt.TltError, match="TLT_ESHAPE"):
        e.ctx.device_status()
    assert e.ctx.device_status() == 0          # cleared
    e.kv.seq_len_bound = 700
    e.ctx.verify_forward(2, t, e.kv, None, None, None)
    assert e.ctx.device_status() == 0
    e.ctx.close()
