"""Pins of the oracle's speculative-decoding step against what the paper and mathematics fix."""
import dataclasses
import itertools

import numpy as np
import pytest

from oracle import decoder as dec
from oracle import sd
from synth import TINY, make_decoder_weights, make_drafter_weights, prompts

SMALLV = dataclasses.replace(TINY, name="tiny-v8", vocab=8)   # small vocab: the random drafter is right often
MICRO = dataclasses.replace(TINY, name="micro", hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16, mlp=96,
                            vocab=40, n_layers=2)


def _models(cfg, seed, std=0.02, qkv_bias=False):
    tw = dec.weights_to_f64(make_decoder_weights(cfg, seed, std=std, qkv_bias=qkv_bias))
    dw = dec.weights_to_f64(make_drafter_weights(cfg, seed, std=std))
    return tw, dw


# ---------------------------------------------------------------- P1: greedy SD == autoregressive greedy
def test_config1_chain_greedy_sd_equals_autoregressive():
    """Tiny decoder, chain depth 4 / top-1 / 4 verify tokens, context 128, 32 steps (workload 1)."""
    tw, dw = _models(TINY, 1234)
    for b, prompt in enumerate(prompts(2, 129, TINY.vocab, seed=1)):
        emitted, accept_lens, st = sd.sd_generate(TINY, tw, dw, prompt, n_steps=32, K=1, D=4, N=4)
        assert len(emitted) == 32 + sum(accept_lens)
        assert emitted == sd.ar_greedy(TINY, tw, prompt, len(emitted))
        assert st.ctx == 128 + len(emitted)


@pytest.mark.parametrize("K,D,N", [(1, 4, 4), (3, 3, 8), (4, 5, 16)])
def test_tree_greedy_sd_equals_autoregressive_with_accepts(K, D, N):
    """Small vocabulary so that the random drafter is often right: accepted paths, cache moves and
    drafter catch-up with several tokens are all exercised."""
    tw, dw = _models(SMALLV, 8, std=0.05)
    total_accepts = 0
    for prompt in prompts(2, 21, SMALLV.vocab, seed=3):
        emitted, accept_lens, _ = sd.sd_generate(SMALLV, tw, dw, prompt, n_steps=12, K=K, D=D, N=N)
        assert emitted == sd.ar_greedy(SMALLV, tw, prompt, len(emitted))
        total_accepts += sum(accept_lens)
    assert total_accepts > 0


def test_greedy_sd_lossless_for_a_strong_proposer():
    """Trees proposed from the target's own next-token distribution plus noise: long accepts."""
    cfg = MICRO
    tw, dw = _models(cfg, 11, std=0.3)
    rng = np.random.default_rng(0)
    prompt = prompts(1, 9, cfg.vocab, seed=5)[0]
    history = []

    def tree_fn(st, root):
        prefix = [int(t) for t in prompt[:-1]] + history + [root]

        def level_fn(level, frontier, pool):
            rows = []
            for pi in frontier:
                toks, a = [], pi
                while a >= 0:
                    toks.append(pool[a].token)
                    a = pool[a].parent
                logits, *_ = dec.dense_forward(cfg, tw, prefix + toks[::-1])
                rows.append(dec.log_softmax(logits[-1] + rng.normal(0, 0.5, cfg.vocab)))
            return np.stack(rows)

        logits, *_ = dec.dense_forward(cfg, tw, prefix)
        pool = sd.expand_tree(dec.log_softmax(logits[-1] + rng.normal(0, 0.5, cfg.vocab)), level_fn, 3, 4)
        return sd.prune_tree(pool, root, 10)

    st = sd.SeqState(cfg, 200)
    root = sd.prefill(cfg, tw, dw, st, prompt)
    emitted, accepts = [], []
    for _ in range(8):
        history[:] = [int(prompt[-1])] + emitted[:-1] if emitted else []
        out, a, *_ = sd.sd_step(cfg, tw, dw, st, root, 3, 4, 10, tree_fn)
        emitted.extend(out)
        accepts.append(a)
        root = out[-1]
    assert emitted == sd.ar_greedy(cfg, tw, prompt, len(emitted))
    assert max(accepts) >= 2 and sum(accepts) >= 6


# ---------------------------------------------------------------- P4 / P5: tree attention, chain, N = 1
def _random_tree(rng, n, vocab):
    parent = np.array([-1] + [int(rng.integers(0, i)) for i in range(1, n)])
    depth = np.zeros(n, dtype=np.int64)
    for i in range(1, n):
        depth[i] = depth[parent[i]] + 1
    return sd.Tree(rng.integers(0, vocab, size=n), parent, depth, np.zeros(n))


@pytest.mark.parametrize("ctx,bias", [(0, False), (7, False), (7, True)])
def test_tree_verification_equals_per_path_causal_forward(ctx, bias):
    cfg = MICRO
    tw, dw = _models(cfg, 21, std=0.3, qkv_bias=bias)
    rng = np.random.default_rng(ctx)
    context = [int(t) for t in rng.integers(0, cfg.vocab, size=ctx)]
    st = sd.SeqState(cfg, 64)
    if ctx:
        sd.verify(cfg, tw, st, sd.chain_tree(context))
        sd.commit(st, list(range(ctx)))
    tree = _random_tree(rng, 9, cfg.vocab)
    logits, hidden = sd.verify(cfg, tw, st, tree)
    for i in range(tree.n):
        path_tokens = [int(tree.token[a]) for a in tree.ancestors_or_self(i)]
        want_logits, want_hidden, *_ = dec.dense_forward(cfg, tw, context + path_tokens)
        np.testing.assert_allclose(logits[i], want_logits[-1], rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(hidden[i], want_hidden[-1], rtol=1e-9, atol=1e-11)


def test_chain_tree_from_empty_cache_is_dense_causal_forward_and_n1_is_plain_decode():
    cfg = MICRO
    tw, dw = _models(cfg, 22, std=0.3)
    toks = [int(t) for t in np.random.default_rng(1).integers(0, cfg.vocab, size=13)]
    st = sd.SeqState(cfg, 32)
    logits, hidden = sd.verify(cfg, tw, st, sd.chain_tree(toks[:12]))
    want_logits, want_hidden, ks, vs = dec.dense_forward(cfg, tw, toks[:12])
    np.testing.assert_allclose(logits, want_logits, rtol=1e-9, atol=1e-11)
    sd.commit(st, list(range(12)))
    for l in range(cfg.n_layers):
        np.testing.assert_allclose(st.target[l].k[:12], ks[l], rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(st.target[l].v[:12], vs[l], rtol=1e-9, atol=1e-12)
    # N = 1: a tree that is only the root is one plain decode step on the cache.
    one, _ = sd.verify(cfg, tw, st, sd.chain_tree(toks[12:13]))
    full, *_ = dec.dense_forward(cfg, tw, toks)
    np.testing.assert_allclose(one[0], full[-1], rtol=1e-9, atol=1e-11)


# ---------------------------------------------------------------- P6: commit invariant
def test_committed_cache_equals_dense_forward_cache():
    cfg = SMALLV
    tw, dw = _models(cfg, 8, std=0.05)
    prompt = prompts(1, 17, cfg.vocab, seed=9)[0]
    emitted, accept_lens, st = sd.sd_generate(cfg, tw, dw, prompt, n_steps=10, K=3, D=3, N=8)
    assert sum(accept_lens) > 0
    seq = [int(t) for t in prompt] + emitted
    assert st.ctx == len(seq) - 1          # everything but the pending root is cached
    _, _, ks, vs = dec.dense_forward(cfg, tw, seq[: st.ctx])
    for l in range(cfg.n_layers):
        np.testing.assert_allclose(st.target[l].k[: st.ctx], ks[l], rtol=1e-8, atol=1e-11)
        np.testing.assert_allclose(st.target[l].v[: st.ctx], vs[l], rtol=1e-8, atol=1e-11)
    assert st.draft_len == st.ctx


def test_commit_rows_moves_exactly_the_path_and_nothing_else():
    rng = np.random.default_rng(0)
    k, v = rng.normal(size=(20, 2, 4)), rng.normal(size=(20, 2, 4))
    k0, v0 = k.copy(), v.copy()
    new_len = sd.commit_rows(k, v, 5, [0, 2, 5])     # destination of j=2 is the source of j=1
    assert new_len == 8
    np.testing.assert_array_equal(k[5:8], k0[[5, 7, 10]])
    np.testing.assert_array_equal(v[5:8], v0[[5, 7, 10]])
    np.testing.assert_array_equal(k[:5], k0[:5])
    np.testing.assert_array_equal(k[8:], k0[8:])


# ---------------------------------------------------------------- P7: tree building
def _markov_level_fn(table):
    def level_fn(level, frontier, pool):
        return np.stack([table[pool[pi].token] for pi in frontier])
    return level_fn


def test_pool_size_of_the_papers_shape_example():
    """Tree-decoding figure: topK = 2, Draft_Depth = 4, Tokens_to_Verify = 8."""
    rng = np.random.default_rng(0)
    table = dec.log_softmax(rng.normal(size=(12, 12)))
    pool = sd.expand_tree(table[0], _markov_level_fn(table), K=2, D=4)
    assert len(pool) == 2 + 3 * 4
    tree = sd.prune_tree(pool, 0, 8)
    assert tree.n == 8 and tree.depth.max() <= 4


@pytest.mark.parametrize("K,D,N,V,seed", [(2, 4, 8, 12, 0), (3, 3, 10, 7, 1), (1, 5, 4, 9, 2), (4, 2, 40, 6, 3)])
def test_tree_invariants_and_brute_force(K, D, N, V, seed):
    rng = np.random.default_rng(seed)
    table = dec.log_softmax(rng.normal(size=(V, V)) * 2)
    root_logp = dec.log_softmax(rng.normal(size=V) * 2)
    pool = sd.expand_tree(root_logp, _markov_level_fn(table), K, D)
    tree = sd.prune_tree(pool, 5, N)
    assert len(pool) == K + (D - 1) * K * K
    assert tree.n == 1 + min(N - 1, len(pool))
    assert tree.parent[0] == -1 and tree.depth[0] == 0
    for i in range(1, tree.n):
        assert 0 <= tree.parent[i] < i
        assert tree.depth[i] == tree.depth[tree.parent[i]] + 1
        assert tree.score[i] <= tree.score[tree.parent[i]] + 1e-15
    if K == 1:
        np.testing.assert_array_equal(tree.parent, np.arange(-1, tree.n - 1))
    # siblings carry distinct tokens
    for p in range(tree.n):
        sib = [int(tree.token[c]) for c in range(tree.n) if tree.parent[c] == p]
        assert len(sib) == len(set(sib))

    # Brute force: score every token path of the full V-ary tree, then re-derive frontier and pool
    # from sorted sets of paths rather than level by level bookkeeping.
    def path_score(path):
        s, prev = root_logp[path[0]], path[0]
        for t in path[1:]:
            s, prev = s + table[prev][t], t
        return s

    def best_children(prefix):   # K most likely continuations of a path, by local probability
        row = root_logp if not prefix else table[prefix[-1]]
        order = sorted(range(V), key=lambda t: (-row[t], t))[:K]
        return [prefix + (t,) for t in order]

    frontier, pool_paths = [()], []
    for level in range(D):
        cands = list(itertools.chain.from_iterable(best_children(p) for p in frontier))
        pool_paths.extend(cands)
        frontier = sorted(cands, key=lambda p: -path_score(p))[:K] if level else cands
    assert len(pool_paths) == len(pool)
    keep = sorted(pool_paths, key=lambda p: -path_score(p))[: N - 1]
    got_paths = set()
    for i in range(1, tree.n):
        got_paths.add(tuple(int(tree.token[a]) for a in tree.ancestors_or_self(i)[1:]))
    assert got_paths == set(keep)
    for i in range(1, tree.n):
        p = tuple(int(tree.token[a]) for a in tree.ancestors_or_self(i)[1:])
        assert abs(tree.score[i] - path_score(p)) < 1e-12


def test_topk_tie_break_prefers_lower_index():
    assert sd.topk_desc([1.0, 3.0, 3.0, 2.0, 3.0], 3) == [1, 2, 4]


# ---------------------------------------------------------------- P8: Algorithm 1 bookkeeping
def test_record_reward_arithmetic():
    a_bar, r = sd.record_reward(0.5, [3, 0, 5, 2], 4)
    assert a_bar == 3.5 and r == 28.0
    # no speculation: every accept length 0 -> one token per sequence per step
    assert sd.record_reward(2.0, [0] * 8, 8) == (1.0, 4.0)


# ---------------------------------------------------------------- the real drafter's expansion, cache-free
_plain_block_rows = dec.block_rows     # the unpatched routine (the mutation tests below swap sd's copy)


def _pool_against_cache_free_drafter(K, D, N, seed=21):
    """Every candidate of `sd.draft_expand`'s pool against a drafter run WITHOUT a cache (Section 4.1:
    the drafter drafts autoregressively from its own output; Section 5.1: topK options per step):
    the log-probability row behind a frontier node == one dense causal drafter pass over (committed
    entries ++ the node's root-to-node path, each path entry built from its token and its parent's
    output); its children == that row's K best tokens; every candidate's score == the sum of those
    row entries along its path; each next frontier == the K best of the level.  Pins the provisional
    rows' cache slots, rotary positions and visibility sets.  Returns the number of rows checked."""
    cfg = MICRO
    tw, dw = _models(cfg, seed, std=0.3)
    prompt = [int(t) for t in prompts(1, 12, cfg.vocab, seed=9)[0]]
    st = sd.SeqState(cfg, 96)
    root = sd.prefill(cfg, tw, dw, st, prompt)
    tree, pool = sd.draft_expand(cfg, tw, dw, st, root, K, D, N)
    assert len(pool) == K + (D - 1) * K * K

    _, hidden, _, _ = dec.dense_forward(cfg, tw, prompt[:-1])
    x_committed = sd.drafter_input(cfg, tw, dw, prompt[1:], hidden)    # entry s = (token s+1, hidden s)
    assert len(x_committed) == st.draft_len

    def dense_drafter(x):
        T = len(x)
        pos = np.arange(T)
        return _plain_block_rows(cfg, dw["layer"], x, pos, pos, pos[None, :] <= pos[:, None], dec.LayerCache(cfg, T))

    def path_of(ci):
        out = []
        while ci >= 0:
            out.append(ci)
            ci = pool[ci].parent
        return out[::-1]

    rows = {}

    def row_after(ci):   # log-probabilities of the token following candidate ci (-1: the root)
        if ci not in rows:
            x = x_committed
            out = dense_drafter(x)
            for node in ([] if ci < 0 else path_of(ci)):
                x = np.concatenate([x, sd.drafter_input(cfg, tw, dw, [pool[node].token], out[-1:])])
                out = dense_drafter(x)
            rows[ci] = dec.log_softmax(dec.lm_logits(cfg, tw, out[-1]))
        return rows[ci]

    # level by level: children of each expanded node, their scores, the next frontier
    frontier = [-1]
    at = 0
    for level in range(D):
        level_cands = []
        for parent_ci in frontier:
            row = row_after(parent_ci)
            best = sorted(range(cfg.vocab), key=lambda t: (-row[t], t))[:K]
            for t in best:
                c = pool[at]
                assert (c.token, c.parent, c.depth) == (t, parent_ci, level + 1), (at, c)
                want = (0.0 if parent_ci < 0 else pool[parent_ci].score) + row[t]
                assert abs(c.score - want) < 1e-9, (at, c.score, want)
                level_cands.append(at)
                at += 1
        frontier = sorted(level_cands, key=lambda ci: (-pool[ci].score, ci))[:K]
    assert at == len(pool)
    # the kept nodes: the N-1 best of the pool
    keep = sorted(sorted(range(len(pool)), key=lambda ci: (-pool[ci].score, ci))[: N - 1])
    assert [int(t) for t in tree.token[1:]] == [pool[ci].token for ci in keep]
    return len(rows)


@pytest.mark.parametrize("K,D,N", [(3, 4, 12), (2, 5, 9), (4, 3, 40)])
def test_draft_expand_pool_equals_cache_free_drafter_forward_of_every_path(K, D, N):
    assert _pool_against_cache_free_drafter(K, D, N) >= 1 + (D - 1) * K - K


@pytest.mark.parametrize("mutation", ["position", "sibling_visible", "ancestors_hidden", "slot"])
def test_the_cache_free_pin_catches_planted_mistakes_in_the_provisional_rows(mutation, monkeypatch):
    """The pin above must fail when the oracle's provisional drafter rows are wrong: a rotary position
    off by one, siblings of a level seeing each other, a node not seeing its ancestors, two nodes
    sharing a cache row.  The mistake is planted in the oracle (CPU), in the routine draft_expand calls."""
    in_expand = {"on": False}
    real_expand = sd.draft_expand

    def block_rows(cfg, lw, x, pos, slots, visible, cache, store=dec.identity):
        if in_expand["on"]:
            base = int(np.min(slots))
            if mutation == "position":
                pos = pos + 1
            elif mutation == "sibling_visible":
                visible = visible.copy()
                visible[:, slots] = True
            elif mutation == "ancestors_hidden":
                keep_self = np.zeros_like(visible)
                keep_self[np.arange(len(slots)), slots] = True
                visible = visible.copy()
                visible[:, cache_len["n"]:] = False      # no provisional row but its own
                visible |= keep_self
            elif mutation == "slot":
                slots = np.full_like(slots, base)
        return _plain_block_rows(cfg, lw, x, pos, slots, visible, cache, store)

    cache_len = {"n": 0}

    def expand(cfg, tw, dw, st, *a, **k):
        in_expand["on"] = True
        cache_len["n"] = st.draft_len
        try:
            return real_expand(cfg, tw, dw, st, *a, **k)
        finally:
            in_expand["on"] = False

    monkeypatch.setattr(sd.dec, "block_rows", block_rows)
    monkeypatch.setattr(sd, "draft_expand", expand)
    with pytest.raises(AssertionError):
        _pool_against_cache_free_drafter(3, 4, 12)


def test_forced_choices_replay_the_same_pool_and_report_the_ranked_values():
    """`pick`: with the default every decision is the K best; a function that returns other indices is
    followed (scores stay sums of the rows' entries) and sees the values it chose among."""
    rng = np.random.default_rng(4)
    table = dec.log_softmax(rng.normal(size=(9, 9)) * 2)
    seen = []

    def second_best_first(where, values, k):
        seen.append((where, len(values)))
        best = sd.topk_desc(values, k + 1)
        return best[1:] if where[0] == "children" and len(values) > k else best[:k]

    pool = sd.expand_tree(table[0], _markov_level_fn(table), 2, 3, pick=second_best_first)
    assert [w for w, _ in seen] == [("root",), ("children", 1, 0), ("children", 1, 1), ("frontier", 1),
                                    ("children", 2, 0), ("children", 2, 1), ("frontier", 2)]
    for c in pool[2:]:
        assert abs(c.score - (pool[c.parent].score + table[pool[c.parent].token][c.token])) < 1e-12
    first = pool[0]
    kids = [c.token for c in pool[2:4]]
    order = sorted(range(9), key=lambda t: (-table[first.token][t], t))
    assert kids == order[1:3]
