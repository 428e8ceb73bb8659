"""tlt_draft_sample (sampled drafting on the static template) against the oracle, and the sampled SD
step end to end (draft_sample -> verify -> rejection-sampling acceptance -> commit -> extend).

What is compared.  The tree's shape is the template: exact.  A child draw is exact integer
arithmetic GIVEN the fp32 distribution q, so every drawn token must equal the oracle's draw from
the GPU's own q row with the same uniform.  q itself comes out of the bf16 (or fp32) drafter and is
compared with the oracle's drafter run on the GPU's tokens.  Its tolerance follows from the
forward's: logits are held to TOL * max|l| (2e-2 in bf16, 1e-4 in fp32), and q_j = exp(l_j / tau) / Z
turns an absolute logit error d into a relative error of at most 2 d / tau (numerator and
normaliser), so max|dq| / max q <= 2 TOL max|l| / tau.  max|l| is at least half the spread of the
logits, and spread / tau is the spread of log q, so the bar used is TOL * (max log q - min log q)
of the oracle's row: never looser than the derived bound.
"""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import accept as oacc
from oracle import decoder as dec
from oracle import sample_draft as osd
from oracle import sd
from paper_2511_16665_amd import binding as tlt
from synth import MID, TINY, fill_kv_pool, prompts

from gpu_util import dense_cache, make_engine, make_models, rel_err

pytestmark = pytest.mark.gpu

MID7 = dataclasses.replace(MID, name="mid-g7", n_q_heads=14, n_layers=1)


def _u32(rng, *shape):
    return rng.integers(0, 2**32, size=shape, dtype=np.uint64).astype(np.uint32)


def _dev_u32(a):
    return torch.from_numpy(a.view(np.int32)).cuda()


@pytest.mark.parametrize("cfg,dtype,K,D,N,tau,tol", [(MID7, "bf16", 10, 8, 64, 0.9, 2e-2), (MID7, "bf16", 8, 6, 48, 1.0, 2e-2),
                                                   (MID7, "bf16", 1, 4, 5, 0.9, 2e-2), (TINY, "fp32", 3, 4, 12, 0.9, 1e-4),
                                                   (TINY, "fp32", 2, 2, 4, 0.5, 1e-4),
                                                   (TINY, "fp32", 4, 1, 5, 0.9, 1e-4),      # depth 1: a star, no drafter pass
                                                   (TINY, "fp32", 3, 3, 1, 0.9, 1e-4)])     # one node: the root alone
def test_draft_sample_matches_oracle(cfg, dtype, K, D, N, tau, tol):
    cfg = dataclasses.replace(cfg, n_layers=1)
    B = 3
    ctxs = np.array([40, 300, 1000], dtype=np.int32)
    n_new = np.array([1, 3, 2], dtype=np.int32)
    hidden_n, stride = 5, 4
    tw_dev, dw_dev, tw, dw = make_models(cfg, 5, dtype, std=0.05)
    cap = int(ctxs.max()) + 160
    e, _, dtable = make_engine(cfg, dtype, tw_dev, dw_dev, B, max(N, stride), D, K, cap, seed=3, seq_len=ctxs)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    dk, dv = fill_kv_pool(1, e.dkv.k_pool.shape[1], cfg.n_kv_heads, cfg.page_size, cfg.head_dim, 6, dtype=tdt)
    e.dkv.k_pool.copy_(dk)
    e.dkv.v_pool.copy_(dv)
    rng = np.random.default_rng(1)
    new_tok = rng.integers(0, cfg.vocab, size=(B, stride)).astype(np.int32)
    new_src = rng.integers(0, hidden_n, size=(B, stride)).astype(np.int32)
    hidden = rng.normal(size=(B, hidden_n, cfg.hidden)).astype(np.float32)
    parent, rank, depth = osd.static_template(K, D, N)
    n = len(parent)
    u = _u32(rng, B, n)
    if n > 1:
        u[0, 1:3] = [0, 2**32 - 1][: min(2, n - 1)]              # the extreme uniforms
    tree = e.tree(n)
    q = torch.full((B, n, cfg.vocab), -1.0, dtype=torch.float32, device="cuda")
    dev = lambda a: torch.from_numpy(a).cuda()
    print(f"draft_sample {cfg.name} {dtype} K={K} D={D} N={N} n={n}", flush=True)
    e.ctx.draft_sample(B, D, K, N, tau, dev(new_tok), dev(new_src), dev(n_new), dev(hidden), None, e.dkv, _dev_u32(u), tree, q)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(e.dkv.seq_len.cpu().numpy(), ctxs + n_new)
    g_tok, g_par, g_dep, g_sc = (x.cpu().numpy() for x in (tree.token, tree.parent, tree.depth, tree.score))
    g_mask = tree.anc_mask.cpu().numpy().astype(np.uint64)
    g_q = q.cpu().numpy()
    store = dec.round_to_bf16 if dtype == "bf16" else dec.identity
    worst, same = 0.0, 0
    for b in range(B):
        np.testing.assert_array_equal(g_par[b], parent)
        np.testing.assert_array_equal(g_dep[b], depth)
        assert not g_sc[b].any()
        assert g_tok[b, 0] == new_tok[b, n_new[b] - 1] and g_mask[b, 0] == 1
        for i in range(1, n):
            assert g_mask[b, i] == (g_mask[b, parent[i]] | np.uint64(1 << i))
        # oracle drafter on the GPU's tokens
        c = int(ctxs[b])
        st = sd.SeqState(cfg, cap, store)
        st.draft.k[:c] = dense_cache(dk, dtable, b, c, cfg.page_size)[0]
        st.draft.v[:c] = dense_cache(dv, dtable, b, c, cfg.page_size)[0]
        st.draft_len = c
        toks = [int(t) for t in new_tok[b, : n_new[b]]]
        sd.draft_extend(cfg, tw, dw, st, toks, hidden[b][new_src[b, : n_new[b]]].astype(np.float64))
        _, o_q = osd.draft_sample(cfg, tw, dw, st, toks[-1], K, D, N, tau, u[b], forced_tokens=g_tok[b])
        o_tree, _ = osd.draft_sample(cfg, tw, dw, st, toks[-1], K, D, N, tau, u[b])
        same += int(np.array_equal(o_tree.token, g_tok[b]))
        for i in range(n):
            kids = [k for k in range(n) if parent[k] == i]
            if not kids:
                assert (g_q[b, i] == -1.0).all()               # rows of childless nodes are not written
                continue
            assert abs(float(g_q[b, i].astype(np.float64).sum()) - 1.0) < 1e-4
            lq = np.log(o_q[i][o_q[i] > 0].astype(np.float64))
            worst = max(worst, rel_err(g_q[b, i], o_q[i]) / (lq.max() - lq.min()))
            # the draws: exact, given the GPU's own distribution
            assert [int(g_tok[b, k]) for k in kids] == osd.draw_children(g_q[b, i], [u[b, k] for k in kids]), (b, i)
            assert len(set(int(g_tok[b, k]) for k in kids)) == len(kids)
    print(f"  worst rel err of q / spread of log q {worst:.3e}; trees identical to the oracle's own draws: {same} of {B}", flush=True)
    assert worst <= tol
    if dtype == "fp32":
        assert same == B          # fp32: a draw flips only if a threshold falls within ~1e-6 of a boundary
    e.ctx.close()


def test_sampled_sd_steps_end_to_end_decisions_match_the_oracle_rule():
    """Six sampled steps on the tiny fp32 model: every step's acceptance must be the oracle's rule
    applied to the GPU's own tree, logits and distributions (bit-exact), the caches must advance by
    accept_len + 1, and the next step must pick up the emitted bonus token as its root."""
    cfg = TINY
    B, K, D, N, tau = 4, 3, 4, 12, 0.9
    tw_dev, dw_dev, tw, dw = make_models(cfg, 7, "fp32", std=0.08)
    P = 24
    e, table, dtable = make_engine(cfg, "fp32", tw_dev, dw_dev, B, max(N, P), D, K, P + 6 * (D + 1) + N + 32, seed=2)
    pr = np.stack(prompts(B, P, cfg.vocab, seed=4)).astype(np.int32)
    e.prefill(pr)
    n = len(osd.static_template(K, D, N)[0])
    rng = np.random.default_rng(9)
    lens = np.full(B, P - 1)
    root = pr[:, -1].copy()
    total = 0
    for step in range(6):
        u_d, u_a, u_f = _u32(rng, B, n), _u32(rng, B, n), _u32(rng, B)
        print(f"sampled step {step}", flush=True)
        al, out = e.step_sampled(K, D, N, tau, _dev_u32(u_d), _dev_u32(u_a), _dev_u32(u_f))
        tree = e.tree(n)
        g_tok, g_par = tree.token.cpu().numpy(), tree.parent.cpu().numpy()
        np.testing.assert_array_equal(g_tok[:, 0], root)
        o_al, o_path, o_out, o_nout = oacc.accept_sample(g_tok, g_par, e.logits(n).cpu().numpy(), e.draft_q(n).cpu().numpy(),
                                                         u_a, u_f, tau, e.stride)
        np.testing.assert_array_equal(al, o_al)
        np.testing.assert_array_equal(out, o_out)
        np.testing.assert_array_equal(e.path_idx.cpu().numpy(), o_path)
        lens = lens + al + 1
        np.testing.assert_array_equal(e.kv.seq_len.cpu().numpy(), lens)
        root = np.array([out[b, al[b]] for b in range(B)])
        total += int(al.sum())
    print("accepted drafts over 6 steps:", total, flush=True)
    assert total > 0
    e.ctx.close()


def test_topk_tree_steps_with_target_only_sampling_acceptance_match_the_oracle_rule():
    """The drafter's deterministic top-k trees with the target-only sampling rule (the variant for
    trees whose shape depends on the drafter): six steps, every decision equal to the oracle's rule on
    the GPU's own tree and logits, lengths and roots carried from step to step.  (A child is accepted
    with the target's own probability of its token, which is tiny for a random model's flat
    distribution at temperature 0.9; a low temperature makes the targets peaked so that accepts occur.)"""
    cfg = TINY
    B, K, D, N, tau = 4, 3, 4, 12, 0.02
    tw_dev, dw_dev, tw, dw = make_models(cfg, 7, "fp32", std=0.08)
    P = 24
    e, table, dtable = make_engine(cfg, "fp32", tw_dev, dw_dev, B, max(N, P), D, K, P + 6 * (D + 1) + N + 32, seed=2)
    pr = np.stack(prompts(B, P, cfg.vocab, seed=4)).astype(np.int32)
    e.prefill(pr)
    rng = np.random.default_rng(19)
    lens = np.full(B, P - 1)
    root = pr[:, -1].copy()
    total = 0
    for step in range(6):
        u_a, u_f = _u32(rng, B, N), _u32(rng, B)
        print(f"target-only step {step}", flush=True)
        al, out = e.step(K, D, N, sample=(tau, _dev_u32(u_a), _dev_u32(u_f)))
        tree = e.tree(N)
        g_tok, g_par = tree.token.cpu().numpy(), tree.parent.cpu().numpy()
        np.testing.assert_array_equal(g_tok[:, 0], root)
        o_al, o_path, o_out, o_nout = oacc.accept_target_only(g_tok, g_par, e.logits(N).cpu().numpy(), u_a, u_f, tau, e.stride)
        np.testing.assert_array_equal(al, o_al)
        np.testing.assert_array_equal(out, o_out)
        np.testing.assert_array_equal(e.path_idx.cpu().numpy(), o_path)
        lens = lens + al + 1
        np.testing.assert_array_equal(e.kv.seq_len.cpu().numpy(), lens)
        root = np.array([out[b, al[b]] for b in range(B)])
        total += int(al.sum())
    print("accepted drafts over 6 steps:", total, flush=True)
    assert total > 0
    e.ctx.close()
