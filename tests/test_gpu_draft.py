"""tlt_draft_expand in bf16 on the long-tail workload's tree shape (depth 8, top-k 10, 64 verify
tokens: 70 provisional drafter rows, i.e. two mask words) against the oracle's drafter."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import decoder as dec
from oracle import sd
from paper_2511_16665_amd import binding as tlt
from synth import MID, fill_kv_pool

from gpu_util import check_draft_tree_against_forced_oracle, dense_cache, make_engine, make_models

pytestmark = pytest.mark.gpu

MID7 = dataclasses.replace(MID, name="mid-g7", n_q_heads=14, n_layers=1)


@pytest.mark.parametrize("K,D,N,impl", [(10, 8, 64, 1), (10, 8, 64, 0), (8, 6, 48, 1), (2, 4, 8, 1)])
def test_draft_expand_bf16_matches_oracle(K, D, N, impl):
    cfg = MID7
    B = 3
    ctxs = np.array([40, 300, 1000], dtype=np.int32)
    n_new = np.array([1, 3, 2], dtype=np.int32)
    hidden_n, stride = 5, 4
    tw_dev, dw_dev, tw, dw = make_models(cfg, 5, "bf16", std=0.05)
    cap = int(ctxs.max()) + 160
    e, _, dtable = make_engine(cfg, "bf16", tw_dev, dw_dev, B, N, D, K, cap, seed=3, seq_len=ctxs)
    dk, dv = fill_kv_pool(1, e.dkv.k_pool.shape[1], cfg.n_kv_heads, cfg.page_size, cfg.head_dim, 6, dtype=torch.bfloat16)
    e.dkv.k_pool.copy_(dk)
    e.dkv.v_pool.copy_(dv)
    rng = np.random.default_rng(1)
    new_tok = rng.integers(0, cfg.vocab, size=(B, stride)).astype(np.int32)
    new_src = rng.integers(0, hidden_n, size=(B, stride)).astype(np.int32)
    hidden = rng.normal(size=(B, hidden_n, cfg.hidden)).astype(np.float32)
    tree = e.tree(N)
    e.ctx.set_attention_impl(impl)
    print(f"draft_expand bf16 K={K} D={D} N={N} impl={impl}", flush=True)
    dev = lambda a: torch.from_numpy(a).cuda()
    e.ctx.draft_expand(B, D, K, N, dev(new_tok), dev(new_src), dev(n_new), dev(hidden), None, e.dkv, tree)
    pool_dev = e.ctx.draft_pool(B, D, K)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(e.dkv.seq_len.cpu().numpy(), ctxs + n_new)
    g_tok, g_par, g_dep, g_sc = (x.cpu().numpy() for x in (tree.token, tree.parent, tree.depth, tree.score))
    g_mask = tree.anc_mask.cpu().numpy().astype(np.uint64)
    n_same = 0
    for b in range(B):
        c = int(ctxs[b])
        st = sd.SeqState(cfg, cap, dec.round_to_bf16)
        st.draft.k[:c] = dense_cache(dk, dtable, b, c, cfg.page_size)[0]
        st.draft.v[:c] = dense_cache(dv, dtable, b, c, cfg.page_size)[0]
        st.draft_len = c
        toks = [int(t) for t in new_tok[b, : n_new[b]]]
        sd.draft_extend(cfg, tw, dw, st, toks, hidden[b][new_src[b, : n_new[b]]].astype(np.float64))
        # structural invariants hold whatever the rounding did
        assert g_tok[b, 0] == toks[-1] and g_par[b, 0] == -1 and g_dep[b, 0] == 0
        for i in range(1, N):
            p = g_par[b, i]
            assert 0 <= p < i and g_dep[b, i] == g_dep[b, p] + 1 and g_sc[b, i] <= g_sc[b, p] + 1e-6
            assert g_mask[b, i] == (g_mask[b, p] | np.uint64(1 << i))
        # the GPU's choices replayed through the oracle's drafter: scores within tolerance, every choice
        # optimal within twice the tolerance, tree = pruning of that pool, identical when no choice differs
        g_pool = tuple(x[b].cpu().numpy() for x in pool_dev)
        seen = check_draft_tree_against_forced_oracle(sd, cfg, tw, dw, st, toks[-1], K, D, N, g_pool,
                                                      (g_tok[b], g_par[b], g_dep[b], g_sc[b]), 2e-2)
        print(f"  sequence {b}: {seen}", flush=True)
        n_same += int(seen["identical"])
    print("identical trees:", n_same, "of", B, flush=True)
    e.ctx.close()
