"""Pins of the oracle's sampled drafting (oracle/sample_draft.py): the static template and the
without-replacement draw of sibling tokens."""
import itertools
import math

import numpy as np
import pytest
from scipy import stats

from oracle import accept as oa
from oracle import sample_draft as osd

from test_oracle_accept import V16, _tables


# ---------------------------------------------------------------- template
def _brute_force(K, D, N):
    nodes = [r for d in range(1, D + 1) for r in itertools.product(range(K), repeat=d)]
    w = {r: math.prod(0.6 * 0.4 ** x for x in r) for r in nodes}      # the prior weight itself, not its log
    order = sorted(nodes, key=lambda r: (-round(math.log(w[r]), 9), len(r), r))
    return set(order[: max(0, N - 1)])


@pytest.mark.parametrize("K,D,N", [(1, 4, 3), (2, 2, 4), (2, 4, 8), (3, 3, 10), (3, 4, 25), (2, 5, 20), (4, 2, 64), (3, 3, 1)])
def test_template_is_the_best_of_the_fully_enumerated_tree(K, D, N):
    parent, rank, depth = osd.static_template(K, D, N)
    n = len(parent)
    # rebuild each node's rank sequence from the arrays
    seq = {0: ()}
    for i in range(1, n):
        assert 0 <= parent[i] < i and depth[i] == depth[parent[i]] + 1 and 0 <= rank[i] < K
        seq[i] = seq[int(parent[i])] + (int(rank[i]),)
    assert set(seq.values()) - {()} == _brute_force(K, D, N)
    assert n == min(N, 1 + sum(K ** d for d in range(1, D + 1)))
    # numbering: by depth, then parent number, then rank
    keys = [(int(depth[i]), int(parent[i]), int(rank[i])) for i in range(1, n)]
    assert keys == sorted(keys)
    # closed under "parent of" (by construction of seq) and "earlier sibling of"
    have = set(seq.values())
    for s in have - {()}:
        assert s[:-1] in have and all(s[:-1] + (r,) in have for r in range(s[-1]))


def test_template_closed_forms_and_the_hand_worked_case():
    # topK = 1: a chain; depth 1: a star; root only
    p, r, d = osd.static_template(1, 5, 4)
    assert list(p) == [-1, 0, 1, 2] and list(r) == [-1, 0, 0, 0] and list(d) == [0, 1, 2, 3]
    p, r, d = osd.static_template(5, 1, 4)
    assert list(p) == [-1, 0, 0, 0] and list(r) == [-1, 0, 1, 2] and list(d) == [0, 1, 1, 1]
    p, r, d = osd.static_template(3, 3, 1)
    assert list(p) == [-1]
    # K=2, D=2, N=4.  Weights: (0) .6, (1) .24, (0,0) .36, (0,1) .144, (1,0) .144, (1,1) .0576
    # -> kept (0), (0,0), (1); numbered (0)=1, (1)=2, (0,0)=3
    p, r, d = osd.static_template(2, 2, 4)
    assert list(p) == [-1, 0, 0, 1] and list(r) == [-1, 0, 1, 0] and list(d) == [0, 1, 1, 2]
    # one more node: (0,1) and (1,0) tie at .144, same depth: the smaller rank sequence (0,1) wins
    p, r, d = osd.static_template(2, 2, 5)
    assert list(p) == [-1, 0, 0, 1, 1] and list(r) == [-1, 0, 1, 0, 1]
    # the benchmark's long-tail shape: depth 8, topK 10, 64 nodes -- bounded, closed, 63 drafted nodes
    p, r, d = osd.static_template(10, 8, 64)
    assert len(p) == 64 and d.max() <= 8 and r.max() < 10 and np.bincount(p[1:]).max() <= 10


# ---------------------------------------------------------------- the draw
def test_draw_hand_worked_thresholds():
    q = np.array([0.5, 0.25, 0.25], dtype=np.float32)       # exact in fp32: weights 2^31, 2^30, 2^30, sum 2^32
    # threshold (U * 2^32) >> 32 = U; first running sum above it
    assert osd.draw_children(q, [0]) == [0]
    assert osd.draw_children(q, [2**31 - 1]) == [0]
    assert osd.draw_children(q, [2**31]) == [1]              # running sum 2^31 is not above 2^31
    assert osd.draw_children(q, [2**31 + 2**30]) == [2]
    assert osd.draw_children(q, [2**32 - 1]) == [2]
    # second draw: token 0 removed, weights (0, 2^30, 2^30), sum 2^31, threshold U >> 1
    assert osd.draw_children(q, [0, 0]) == [0, 1]
    assert osd.draw_children(q, [0, 2**31 - 1]) == [0, 1]
    assert osd.draw_children(q, [0, 2**31]) == [0, 2]
    assert osd.draw_children(q, [2**32 - 1, 2**32 - 1, 0]) == [2, 1, 0]
    # zero-probability tokens are never drawn
    q = np.array([0.0, 1.0, 0.0], dtype=np.float32)
    assert osd.draw_children(q, [0]) == [1] and osd.draw_children(q, [2**32 - 1]) == [1]


def test_vectorised_draw_equals_the_plain_one():
    rng = np.random.default_rng(5)
    q = rng.dirichlet(np.full(37, 0.3), size=200).astype(np.float32)
    q[:, 5] = 0
    u = rng.integers(0, 2**32, size=(200, 6), dtype=np.uint64).astype(np.uint32)
    u[0] = 0
    u[1] = 2**32 - 1
    got = osd.draw_children_rows(q, u)
    for b in range(200):
        assert list(got[b]) == osd.draw_children(q[b], list(u[b]))
        assert len(set(got[b])) == 6 and 5 not in got[b]


def test_successive_draws_follow_sampling_without_replacement():
    # P(first = a, second = b) = q_a q_b / (1 - q_a)
    rng = np.random.default_rng(7)
    q = np.array([0.35, 0.05, 0.2, 0.1, 0.25, 0.05], dtype=np.float32)
    n = 400_000
    u = rng.integers(0, 2**32, size=(n, 2), dtype=np.uint64).astype(np.uint32)
    picks = osd.draw_children_rows(np.tile(q, (n, 1)), u)
    hist = np.zeros((6, 6))
    np.add.at(hist, (picks[:, 0], picks[:, 1]), 1)
    q64 = q.astype(np.float64) / q.astype(np.float64).sum()
    expected = q64[:, None] * q64[None, :] / (1 - q64[:, None]) * n
    np.fill_diagonal(expected, 0)
    assert np.trace(hist) == 0
    off = ~np.eye(6, dtype=bool)
    chi2 = ((hist[off] - expected[off]) ** 2 / expected[off]).sum()
    assert stats.chi2.sf(chi2, off.sum() - 1) > 1e-3


# ---------------------------------------------------------------- template + draw + acceptance rule together
def test_sampled_template_trees_keep_the_target_distribution_chi_square():
    """Two generated tokens against p(x1) p(x2|x1) on the 16-token toy model (target and drafter are
    bigram tables), every tree built from static_template(2, 2, 4) and draw_children_rows."""
    P, Q = _tables(0)
    parent, rank, depth = osd.static_template(2, 2, 4)
    assert list(parent) == [-1, 0, 0, 1]
    n_draws = 1_000_000
    rng = np.random.default_rng(321)

    def step(roots):
        B = len(roots)
        u = rng.integers(0, 2**32, size=(B, 4), dtype=np.uint64).astype(np.uint32)
        token = np.zeros((B, 4), dtype=np.int64)
        token[:, 0] = roots
        q_root = Q[roots].astype(np.float32)
        token[:, 1:3] = osd.draw_children_rows(q_root, u[:, 1:3])          # nodes 1, 2: children of the root
        q_1 = Q[token[:, 1]].astype(np.float32)
        token[:, 3] = osd.draw_children_rows(q_1, u[:, 3:4])[:, 0]         # node 3: child of node 1
        with np.errstate(divide="ignore"):
            logits = np.log(P[token]).astype(np.float32)
        draft_q = Q[token].astype(np.float32)
        u_acc = rng.integers(0, 2**32, size=(B, 4), dtype=np.uint64).astype(np.uint32)
        u_fin = rng.integers(0, 2**32, size=B, dtype=np.uint64).astype(np.uint32)
        return oa.accept_sample(token.astype(np.int32), np.tile(parent.astype(np.int32), (B, 1)), logits, draft_q,
                                u_acc, u_fin, 1.0, 4)

    x0 = 3
    al, _, out, n_out = step(np.full(n_draws, x0))
    x1, x2 = out[:, 0].copy(), out[:, 1].copy()
    need = n_out < 2
    _, _, out2, _ = step(x1[need])
    x2[need] = out2[:, 0]
    hist = np.zeros((V16, V16))
    np.add.at(hist, (x1, x2), 1)
    expected = (P[x0][:, None] * P) * n_draws
    assert al.max() == 2 and (al == 0).mean() > 0.05
    keep = expected > 5
    chi2 = ((hist[keep] - expected[keep]) ** 2 / expected[keep]).sum() + \
        (hist[~keep].sum() - expected[~keep].sum()) ** 2 / max(expected[~keep].sum(), 1e-9)
    assert stats.chi2.sf(chi2, keep.sum()) > 1e-3


# ---------------------------------------------------------------- the drafter forward behind the distributions
def test_drafted_distributions_equal_a_cache_free_drafter_forward_of_every_path():
    """q of every node with children == softmax(logits / tau) of the drafter run WITHOUT a cache over
    (committed entries ++ the node's root-to-node path), one dense causal pass per path: pins the
    slots, positions and visibility sets of the provisional drafter entries."""
    import dataclasses

    from oracle import decoder as dec
    from oracle import sd
    from synth import TINY, make_decoder_weights, make_drafter_weights, prompts

    cfg = dataclasses.replace(TINY, name="micro", hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16, mlp=96, vocab=40,
                              n_layers=2)
    tw = dec.weights_to_f64(make_decoder_weights(cfg, 21, std=0.3))
    dw = dec.weights_to_f64(make_drafter_weights(cfg, 21, std=0.3))
    prompt = [int(t) for t in prompts(1, 12, cfg.vocab, seed=9)[0]]
    st = sd.SeqState(cfg, 64)
    root = sd.prefill(cfg, tw, dw, st, prompt)
    K, D, N, tau = 3, 4, 12, 0.9
    u = np.random.default_rng(2).integers(0, 2**32, size=N, dtype=np.uint64).astype(np.uint32)
    tree, q = osd.draft_sample(cfg, tw, dw, st, root, K, D, N, tau, u)
    parent, rank, depth = osd.static_template(K, D, N)
    np.testing.assert_array_equal(tree.parent, parent)
    np.testing.assert_array_equal(tree.depth, depth)
    assert tree.token[0] == root

    # committed drafter inputs, rebuilt from a dense target forward: entry s = (token s+1, hidden s)
    _, hidden, _, _ = dec.dense_forward(cfg, tw, prompt[:-1])
    x_committed = sd.drafter_input(cfg, tw, dw, prompt[1:], hidden)
    T0 = len(x_committed)
    assert T0 == st.draft_len

    def dense_drafter(x):
        T = len(x)
        pos = np.arange(T)
        return dec.block_rows(cfg, dw["layer"], x, pos, pos, pos[None, :] <= pos[:, None], dec.LayerCache(cfg, T))

    checked = 0
    for i in range(tree.n):
        kids = [c for c in range(tree.n) if parent[c] == i]
        if not kids:
            assert not q[i].any()
            continue
        path = tree.ancestors_or_self(i)                  # root .. i
        x = x_committed
        out = dense_drafter(x)
        for node in path[1:]:                             # each path node: its token + its parent's output feature
            x = np.concatenate([x, sd.drafter_input(cfg, tw, dw, [int(tree.token[node])], out[-1:])])
            out = dense_drafter(x)
        want = osd.softmax_temperature(dec.lm_logits(cfg, tw, out[-1]), tau)
        np.testing.assert_allclose(q[i], want, rtol=1e-5, atol=1e-9)
        # the children are the draws from exactly this row
        assert [int(tree.token[c]) for c in kids] == osd.draw_children(q[i], [u[c] for c in kids])
        checked += 1
    assert checked >= 4
