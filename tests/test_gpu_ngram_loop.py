"""Greedy decoding driven by the model-free drafter's trees (Section 5.3) through the GPU path:
whatever the n-gram database proposes, the output must be the plain autoregressive greedy
continuation (Section 2.2: verification is lossless), and with sibling rollouts that resemble the
sequence being generated several tokens per step must be accepted."""
import numpy as np
import pytest

from paper_2511_16665_amd import binding as tlt
from synth import TINY, prompts

from gpu_util import make_engine, make_models

pytestmark = pytest.mark.gpu


def test_ngram_trees_give_the_autoregressive_output_and_accept_planted_repeats():
    cfg = TINY
    B, P, T = 3, 24, 48
    tw_dev, dw_dev, _, _ = make_models(cfg, 31, "fp32", std=0.08)
    pr = prompts(B, P, cfg.vocab, seed=9)
    depth, topk, n_nodes = 4, 2, 8
    ref_e, _, _ = make_engine(cfg, "fp32", tw_dev, dw_dev, B, n_nodes, depth, topk, P + T + 64, seed=3)
    sd_e, _, _ = make_engine(cfg, "fp32", tw_dev, dw_dev, B, n_nodes, depth, topk, P + T + 64, seed=3)
    ref_e.prefill(pr)
    sd_e.prefill(pr)
    # plain decoding: one-node trees
    ref = [[] for _ in range(B)]
    root = pr[:, -1].copy()
    for _ in range(T):
        al, out = ref_e.step_trees(root.reshape(B, 1), np.full((B, 1), -1, np.int32))
        assert (al == 0).all()
        root = out[:, 0].copy()
        for b in range(B):
            ref[b].append(int(root[b]))
    # sibling rollouts: the same continuation with every 9th token changed
    rng = np.random.default_rng(0)
    db = tlt.NGram(4)
    for b in range(B):
        sib = list(pr[b]) + ref[b]
        for i in range(P + 3, len(sib), 9):
            sib[i] = int(rng.integers(cfg.vocab))
        db.insert(b, sib)
    gen = [[] for _ in range(B)]
    seqs = [list(pr[b]) for b in range(B)]
    accepted, steps = 0, 0
    while min(len(g) for g in gen) < T - depth - 1:
        tok = np.zeros((B, n_nodes), np.int32)
        par = np.zeros((B, n_nodes), np.int32)
        for b in range(B):
            tok[b], par[b], _ = db.propose(b, seqs[b][-8:], depth, topk, n_nodes)
        al, out = sd_e.step_trees(tok, par)
        for b in range(B):
            new = [int(x) for x in out[b, : al[b] + 1]]
            gen[b] += new
            seqs[b] += new
        accepted += int(al.sum())
        steps += 1
    for b in range(B):
        m = min(len(gen[b]), T)
        assert gen[b][:m] == ref[b][:m], f"sequence {b} diverged from plain greedy decoding"
    mean_accept = accepted / (steps * B)
    print(f"{steps} steps, mean accepted drafts per step {mean_accept:.2f}", flush=True)
    assert mean_accept > 1.0
    for e in (ref_e, sd_e):
        e.ctx.close()


def test_switching_between_the_model_free_and_the_learned_drafter_keeps_the_drafter_cache_in_step():
    """Steps alternate between n-gram trees (the learned drafter's cache following along) and the
    learned drafter.  The output must stay the plain greedy continuation, and every tree the learned
    drafter builds after a model-free phase must be the oracle's, whose drafter state is advanced
    over the same accepted tokens: a stale or misaligned drafter cache would change those trees."""
    from oracle import decoder as dec
    from oracle import sd

    cfg = TINY
    B, P, depth, topk, n_nodes = 2, 24, 4, 2, 8
    tw_dev, dw_dev, tw, dw = make_models(cfg, 31, "fp32", std=0.08)
    pr = prompts(B, P, cfg.vocab, seed=9)
    e, _, _ = make_engine(cfg, "fp32", tw_dev, dw_dev, B, n_nodes, depth, topk, P + 160, seed=3)
    e.prefill(pr)
    states, roots = [], []
    for b in range(B):
        st = sd.SeqState(cfg, P + 160)
        roots.append(sd.prefill(cfg, tw, dw, st, [int(t) for t in pr[b]]))
        states.append(st)
    db = tlt.NGram(3)
    for b in range(B):
        db.insert(b, [int(t) for t in pr[b]])
    seqs = [[int(t) for t in pr[b]] for b in range(B)]
    plan = ["ngram", "ngram", "learned", "ngram", "learned", "learned", "ngram", "ngram", "ngram", "learned"]
    same_trees = 0
    for step, kind in enumerate(plan):
        print(f"step {step}: {kind}", flush=True)
        if kind == "ngram":
            tok = np.zeros((B, n_nodes), np.int32)
            par = np.zeros((B, n_nodes), np.int32)
            for b in range(B):
                tok[b], par[b], _ = db.propose(b, seqs[b][-8:], depth, topk, n_nodes)
            al, out = e.step_trees(tok, par, keep_drafter=True)
        else:
            al, out = e.step(topk, depth, n_nodes)
            g_tree = e.tree(n_nodes)
            g_tok, g_par = g_tree.token.cpu().numpy(), g_tree.parent.cpu().numpy()
        for b in range(B):
            st = states[b]
            if kind == "ngram":
                depth_b = np.zeros(n_nodes, np.int64)
                for i in range(1, n_nodes):
                    depth_b[i] = depth_b[par[b, i]] + 1
                fixed = sd.Tree(tok[b].astype(np.int64), par[b].astype(np.int64), depth_b, np.zeros(n_nodes))
                o_out, o_a, *_ = sd.sd_step(cfg, tw, dw, st, roots[b], topk, depth, n_nodes, tree_fn=lambda s_, r_: fixed)
            else:
                o_out, o_a, o_tree, *_ = sd.sd_step(cfg, tw, dw, st, roots[b], topk, depth, n_nodes)
                if np.array_equal(o_tree.token, g_tok[b]) and np.array_equal(o_tree.parent, g_par[b]):
                    same_trees += 1
                else:
                    # only a near-tie between path scores may reorder the tree in fp32
                    sc = np.sort(o_tree.score[1:])
                    assert np.min(np.diff(sc)) < 1e-4, (step, b, "learned drafter's tree differs from the oracle's")
            assert o_a == al[b] and o_out == [int(x) for x in out[b, : al[b] + 1]], (step, b)
            roots[b] = o_out[-1]
            seqs[b] += o_out
            db.insert(b, seqs[b])
    print("learned-drafter trees identical to the oracle's:", same_trees, "of", B * plan.count("learned"), flush=True)
    assert same_trees >= B * plan.count("learned") - 1
    for b in range(B):   # and the whole output is the plain greedy continuation
        gen = seqs[b][P:]
        assert gen == sd.ar_greedy(cfg, tw, [int(t) for t in pr[b]], len(gen))
    e.ctx.close()


def test_activating_the_drafter_in_the_middle_of_a_rollout():
    """Sequences of different lengths are decoded for a while without the learned drafter (its cache
    empty), then it is switched on: after Engine.activate_drafter the trees it builds must be the
    oracle's, whose drafter has seen every token from the start, and decoding stays plain greedy."""
    import torch

    from oracle import sd

    cfg = TINY
    B, depth, topk, n_nodes = 3, 4, 2, 8
    tw_dev, dw_dev, tw, dw = make_models(cfg, 31, "fp32", std=0.08)
    P = 20
    pr = prompts(B, P, cfg.vocab, seed=12)
    e, _, _ = make_engine(cfg, "fp32", tw_dev, dw_dev, B, 16, depth, topk, P + 200, seed=3)
    e.prefill(pr)
    # no drafter so far: forget what prefill put into its cache
    e.dkv.k_pool.zero_()
    e.dkv.v_pool.zero_()
    e.dkv.seq_len.zero_()
    e.dkv.seq_len_bound = 0
    seqs = [[int(t) for t in pr[b]] for b in range(B)]
    ref = [sd.ar_greedy(cfg, tw, seqs[b], 40) for b in range(B)]
    rng = np.random.default_rng(1)
    for step in range(9):     # decoding with guessed chains: sequence 0 is guessed right twice per step,
        tok = np.zeros((B, 3), np.int32)   # sequence 1 once, sequence 2 never, so the lengths drift apart
        par = np.tile(np.array([-1, 0, 1], np.int32), (B, 1))
        for b in range(B):
            done = len(seqs[b]) - P
            guess = [ref[b][done + j] if j < 2 - b else int(rng.integers(cfg.vocab)) for j in range(2)]
            tok[b] = [seqs[b][-1]] + guess
        al, out = e.step_trees(tok, par)
        for b in range(B):
            seqs[b] += [int(x) for x in out[b, : al[b] + 1]]
    lens = np.array([len(s) - 1 for s in seqs], dtype=np.int32)
    assert len(set(lens)) == B          # ragged: the 5-position chunks end at different places
    width = int(lens.max()) + 1
    tokens = np.zeros((B, width), np.int32)
    for b in range(B):
        tokens[b, : len(seqs[b])] = seqs[b]
    print("activating the drafter at lengths", lens, flush=True)
    e.activate_drafter(tokens, lens, chunk=5)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(e.dkv.seq_len.cpu().numpy(), lens)
    np.testing.assert_array_equal(e.kv.seq_len.cpu().numpy(), lens)
    # oracle: the same sequences with the drafter following from the start
    states, roots = [], []
    for b in range(B):
        st = sd.SeqState(cfg, P + 200)
        roots.append(sd.prefill(cfg, tw, dw, st, seqs[b], chunk=7))
        states.append(st)
    same = 0
    for step in range(3):
        al, out = e.step(topk, depth, n_nodes)
        g_tree = e.tree(n_nodes)
        g_tok, g_par = g_tree.token.cpu().numpy(), g_tree.parent.cpu().numpy()
        for b in range(B):
            o_out, o_a, o_tree, *_ = sd.sd_step(cfg, tw, dw, states[b], roots[b], topk, depth, n_nodes)
            if np.array_equal(o_tree.token, g_tok[b]) and np.array_equal(o_tree.parent, g_par[b]):
                same += 1
            else:
                sc = np.sort(o_tree.score[1:])
                assert np.min(np.diff(sc)) < 1e-4, (step, b, "tree differs from the oracle's after activation")
            assert o_a == al[b] and o_out == [int(x) for x in out[b, : al[b] + 1]], (step, b)
            roots[b] = o_out[-1]
            seqs[b] += o_out
    print("trees identical to the oracle's after activation:", same, "of", 3 * B, flush=True)
    assert same >= 3 * B - 1
    for b in range(B):
        gen = seqs[b][P:]
        assert gen == sd.ar_greedy(cfg, tw, [int(t) for t in pr[b]], len(gen))
    e.ctx.close()
