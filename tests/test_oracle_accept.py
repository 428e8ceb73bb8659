"""Pins of the oracle's acceptance rules (oracle/accept.c)."""
import numpy as np
import pytest
from scipy import stats

from oracle import accept as oa
from oracle import sd


def _random_tree_arrays(rng, B, n, V, branching=3):
    token = rng.integers(0, V, size=(B, n)).astype(np.int32)
    parent = np.full((B, n), -1, dtype=np.int32)
    for b in range(B):
        for i in range(1, n):
            parent[b, i] = rng.integers(max(0, i - branching), i)
    return token, parent


# ---------------------------------------------------------------- greedy: brute force over all paths
def test_greedy_accept_is_the_longest_path_matching_the_targets_argmax():
    rng = np.random.default_rng(0)
    B, n, V, stride = 64, 12, 5, 12
    token, parent = _random_tree_arrays(rng, B, n, V)
    logits = rng.normal(size=(B, n, V)).astype(np.float32)
    al, path, out, n_out = oa.accept_greedy(token, parent, logits, stride)
    assert al.max() >= 2          # the case is not trivial
    for b in range(B):
        best = np.argmax(logits[b], axis=1)
        # all root-to-node paths; a path is "correct" if every node's token is the argmax at its parent
        good = [[0]]
        for i in range(1, n):
            chain = [i]
            while parent[b, chain[-1]] >= 0:
                chain.append(parent[b, chain[-1]])
            chain = chain[::-1]
            if all(token[b, c] == best[parent[b, c]] for c in chain[1:]):
                good.append(chain)
        longest = max(len(g) for g in good)
        cands = [g for g in good if len(g) == longest]
        # several longest correct paths can exist only through duplicate sibling tokens: the rule
        # takes the lowest node index at every level
        want = min(cands)
        assert al[b] == longest - 1 and n_out[b] == longest
        assert list(path[b, :longest]) == want
        assert list(out[b, : longest - 1]) == [token[b, c] for c in want[1:]]
        assert out[b, longest - 1] == best[want[-1]]
        assert (path[b, longest:] == -1).all() and (out[b, longest:] == -1).all()


def test_greedy_matches_the_float64_reference_form_and_ties_take_lowest_index():
    rng = np.random.default_rng(1)
    token, parent = _random_tree_arrays(rng, 8, 9, 4)
    logits = rng.integers(0, 3, size=(8, 9, 4)).astype(np.float32)      # many exact ties
    al, path, out, n_out = oa.accept_greedy(token, parent, logits, 9)
    for b in range(8):
        depth = np.zeros(9, dtype=np.int64)
        tree = sd.Tree(token[b].astype(np.int64), parent[b].astype(np.int64), depth, np.zeros(9))
        a, p, o = sd.accept_greedy(tree, logits[b].astype(np.float64))
        assert a == al[b] and p == list(path[b, : a + 1]) and o == list(out[b, : a + 1])


def test_greedy_respects_path_capacity():
    token = np.array([[7, 1, 1, 1]], dtype=np.int32)
    parent = np.array([[-1, 0, 1, 2]], dtype=np.int32)
    logits = np.zeros((1, 4, 3), dtype=np.float32)
    logits[:, :, 1] = 1.0
    al, path, out, n_out = oa.accept_greedy(token, parent, logits, 2)
    assert al[0] == 1 and list(path[0]) == [0, 1] and list(out[0]) == [1, 1]


# ---------------------------------------------------------------- sampling: distribution and closed form
V16 = 16


def _tables(seed):
    rng = np.random.default_rng(seed)
    P = rng.dirichlet(np.full(V16, 0.7), size=V16)        # target bigram table p(next | cur)
    Q = rng.dirichlet(np.full(V16, 0.7), size=V16)        # drafter bigram table
    Q = 0.5 * Q + 0.5 * P                                 # a drafter that is roughly right
    return P, Q


def _step(rng, P, Q, roots, children_fn):
    """One SD step for many sequences on the static tree root -> (c1 -> g, c2)."""
    B = len(roots)
    kids = children_fn(Q[roots], 2, rng)                  # [B, 2]
    g = children_fn(Q[kids[:, 0]], 1, rng)[:, 0]
    token = np.stack([roots, kids[:, 0], kids[:, 1], g], axis=1).astype(np.int32)
    parent = np.tile(np.array([-1, 0, 0, 1], dtype=np.int32), (B, 1))
    with np.errstate(divide="ignore"):
        logits = np.log(P[token]).astype(np.float32)      # [B, 4, V]
    draft_q = Q[token].astype(np.float32)
    u_acc = rng.integers(0, 2**32, size=(B, 4), dtype=np.uint64).astype(np.uint32)
    u_fin = rng.integers(0, 2**32, size=B, dtype=np.uint64).astype(np.uint32)
    return oa.accept_sample(token, parent, logits, draft_q, u_acc, u_fin, 1.0, 4)


def _two_token_histogram(children_fn, n_draws, seed):
    P, Q = _tables(seed)
    rng = np.random.default_rng(seed + 100)
    x0 = 3
    roots = np.full(n_draws, x0)
    al, path, out, n_out = _step(rng, P, Q, roots, children_fn)
    x1 = out[:, 0].copy()
    x2 = out[:, 1].copy()
    need = n_out < 2                                       # only one token emitted: run a second step
    al2, _, out2, _ = _step(rng, P, Q, x1[need], children_fn)
    x2[need] = out2[:, 0]
    hist = np.zeros((V16, V16))
    np.add.at(hist, (x1, x2), 1)
    expected = (P[x0][:, None] * P) * n_draws
    return hist, expected, al


def test_sampling_acceptance_reproduces_the_target_distribution_chi_square():
    n = 1_000_000
    hist, expected, al = _two_token_histogram(oa.draw_without_replacement, n, seed=0)
    assert al.max() == 2 and (al == 0).mean() > 0.05       # all branches of the rule are exercised
    keep = expected > 5
    chi2 = ((hist[keep] - expected[keep]) ** 2 / expected[keep]).sum() + \
        (hist[~keep].sum() - expected[~keep].sum()) ** 2 / max(expected[~keep].sum(), 1e-9)
    dof = keep.sum()
    p_value = stats.chi2.sf(chi2, dof)
    assert p_value > 1e-3, (chi2, dof, p_value)


def test_sampling_acceptance_negative_control_deterministic_topk_children_is_biased():
    def topk_children(q, k, rng):
        return np.argsort(-q, axis=-1)[..., :k]
    hist, expected, _ = _two_token_histogram(topk_children, 200_000, seed=0)
    keep = expected > 5
    chi2 = ((hist[keep] - expected[keep]) ** 2 / expected[keep]).sum()
    assert stats.chi2.sf(chi2, keep.sum()) < 1e-12


@pytest.mark.parametrize("tau", [1.0, 0.7])
def test_first_accept_probability_is_one_minus_total_variation(tau):
    rng = np.random.default_rng(5)
    B = 400_000
    logit = rng.normal(size=V16) * 1.5
    p = np.exp(logit / tau) / np.exp(logit / tau).sum()
    q = np.exp(logit + rng.normal(size=V16))
    q /= q.sum()
    child = oa.draw_without_replacement(np.tile(q, (B, 1)), 1, rng)[:, 0]
    token = np.stack([np.zeros(B, dtype=np.int64), child], axis=1).astype(np.int32)
    parent = np.tile(np.array([-1, 0], dtype=np.int32), (B, 1))
    logits = np.tile(logit.astype(np.float32), (B, 2, 1))
    dq = np.tile(q.astype(np.float32), (B, 2, 1))
    u_acc = rng.integers(0, 2**32, size=(B, 2), dtype=np.uint64).astype(np.uint32)
    u_fin = rng.integers(0, 2**32, size=B, dtype=np.uint64).astype(np.uint32)
    al, path, out, n_out = oa.accept_sample(token, parent, logits, dq, u_acc, u_fin, tau, 2)
    rate = (al >= 1).mean()
    want = np.minimum(p, q).sum()
    assert abs(rate - want) < 5 * np.sqrt(want * (1 - want) / B)
    # and the first emitted token is distributed as p
    hist = np.bincount(out[:, 0], minlength=V16)
    assert stats.chisquare(hist, p * B).pvalue > 1e-3


def test_sampling_with_no_children_is_a_plain_draw_by_inverse_cdf():
    """Closed form: with only the root, the emitted token is the first index whose cumulative
    weight exceeds u * total."""
    logit = np.log(np.array([0.5, 0.25, 0.125, 0.125])).astype(np.float32)
    e = 4096   # fp32 logs are not exact: stay a few thousand units clear of each boundary
    us = np.array([0, 2**31 - e, 2**31 + e, 2**31 + 2**30 - e, 2**31 + 2**30 + e, 2**32 - 2**29 - e, 2**32 - 2**29 + e,
                   2**32 - 1], dtype=np.uint64).astype(np.uint32)
    B = len(us)
    token = np.zeros((B, 1), dtype=np.int32)
    parent = np.full((B, 1), -1, dtype=np.int32)
    al, path, out, n_out = oa.accept_sample(token, parent, np.tile(logit, (B, 1, 1)), np.full((B, 1, 4), 0.25, np.float32),
                                            np.zeros((B, 1), np.uint32), us, 1.0, 1)
    assert list(out[:, 0]) == [0, 0, 1, 1, 2, 2, 3, 3] and (al == 0).all()


# ---------------------------------------------------------------- target-only rule (any tree)
def _step_target_only(rng, P, Q, roots):
    """One SD step on root -> (c1 -> g, c2) with DETERMINISTIC top-k children of the drafter table."""
    B = len(roots)
    top = np.argsort(-Q, axis=-1)
    kids = top[roots][:, :2]
    g = top[kids[:, 0]][:, 0]
    token = np.stack([roots, kids[:, 0], kids[:, 1], g], axis=1).astype(np.int32)
    parent = np.tile(np.array([-1, 0, 0, 1], dtype=np.int32), (B, 1))
    with np.errstate(divide="ignore"):
        logits = np.log(P[token]).astype(np.float32)
    u_acc = rng.integers(0, 2**32, size=(B, 4), dtype=np.uint64).astype(np.uint32)
    u_fin = rng.integers(0, 2**32, size=B, dtype=np.uint64).astype(np.uint32)
    return oa.accept_target_only(token, parent, logits, u_acc, u_fin, 1.0, 4)


def test_target_only_rule_is_lossless_on_deterministic_topk_trees_chi_square():
    """The trees of the negative control above (on which the p/q rule is biased): two generated
    tokens against p(x1) p(x2|x1) over 1e6 draws."""
    P, Q = _tables(0)
    n_draws = 1_000_000
    rng = np.random.default_rng(77)
    x0 = 3
    al, _, out, n_out = _step_target_only(rng, P, Q, np.full(n_draws, x0))
    x1, x2 = out[:, 0].copy(), out[:, 1].copy()
    need = n_out < 2
    _, _, out2, _ = _step_target_only(rng, P, Q, x1[need])
    x2[need] = out2[:, 0]
    hist = np.zeros((V16, V16))
    np.add.at(hist, (x1, x2), 1)
    expected = (P[x0][:, None] * P) * n_draws
    assert al.max() == 2 and (al == 0).mean() > 0.05
    keep = expected > 5
    chi2 = ((hist[keep] - expected[keep]) ** 2 / expected[keep]).sum() + \
        (hist[~keep].sum() - expected[~keep].sum()) ** 2 / max(expected[~keep].sum(), 1e-9)
    assert stats.chi2.sf(chi2, keep.sum()) > 1e-3


def test_target_only_accept_probabilities_closed_form_and_hand_worked_thresholds():
    # p = (.5, .25, .125, .125); children of the root: tokens 1 then 0
    logit = np.log(np.array([0.5, 0.25, 0.125, 0.125])).astype(np.float32)
    token = np.array([[9, 1, 0]], dtype=np.int32) % 4
    parent = np.array([[-1, 0, 0]], dtype=np.int32)
    e = 4096      # fp32 logs are not exact: stay a few thousand units clear of each boundary

    def run(u1, u2, uf):
        al, path, out, n_out = oa.accept_target_only(token, parent, np.tile(logit, (1, 3, 1)),
                                                     np.array([[0, u1, u2]], dtype=np.uint64).astype(np.uint32),
                                                     np.array([uf], dtype=np.uint64).astype(np.uint32), 1.0, 2)
        return int(al[0]), [int(x) for x in path[0]], [int(x) for x in out[0]]
    # child 1 (token 1, p = .25) is accepted iff U < .25
    assert run(2**30 - e, 0, 0)[:2] == (1, [0, 1])
    a, path, out = run(2**30 + e, 0, 0)
    # rejected: token 1 removed (remaining mass .75); child 2 (token 0) accepted iff U * .75 < .5
    assert (a, path) == (1, [0, 2]) and out[0] == 0
    assert run(2**30 + e, int(2**32 * 2 / 3) - e, 0)[1] == [0, 2]
    a, path, out = run(2**30 + e, int(2**32 * 2 / 3) + e, 0)
    # both rejected: the emitted token is drawn from (0, 0, .125, .125): halves of the final uniform
    assert (a, path) == (0, [0, -1]) and out[0] == 2
    assert run(2**30 + e, int(2**32 * 2 / 3) + e, 2**31 + e)[2][0] == 3
    # closed form over many draws: P(accept first child) = p(c), and the emitted token ~ p
    rng = np.random.default_rng(3)
    B = 400_000
    lg = rng.normal(size=V16) * 1.5
    p = np.exp(lg / 0.8) / np.exp(lg / 0.8).sum()
    tok = np.tile(np.array([0, 5, 11], dtype=np.int32), (B, 1))
    par = np.tile(np.array([-1, 0, 0], dtype=np.int32), (B, 1))
    al, path, out, n_out = oa.accept_target_only(tok, par, np.tile(lg.astype(np.float32), (B, 3, 1)),
                                                 rng.integers(0, 2**32, size=(B, 3), dtype=np.uint64).astype(np.uint32),
                                                 rng.integers(0, 2**32, size=B, dtype=np.uint64).astype(np.uint32), 0.8, 2)
    first = (path[:, 1] == 1).mean()
    assert abs(first - p[5]) < 5 * np.sqrt(p[5] * (1 - p[5]) / B)
    second = (path[:, 1] == 2).mean()
    assert abs(second - p[11]) < 5 * np.sqrt(p[11] * (1 - p[11]) / B)
    assert stats.chisquare(np.bincount(out[:, 0], minlength=V16), p * B).pvalue > 1e-3
