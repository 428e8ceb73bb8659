"""The check that judges a lower-precision drafter tree against the oracle (gpu_util.
check_draft_tree_against_forced_oracle) must be able to fail.  Here the "GPU" is the oracle itself
with its choices disturbed on the CPU: noise well inside the tolerance must pass (and a noise-free
run must be recognised as identical), a planted wrong choice or a wrong score must not."""
import dataclasses

import numpy as np
import pytest

from oracle import decoder as dec
from oracle import sd
from synth import TINY, make_decoder_weights, make_drafter_weights, prompts

from gpu_util import check_draft_tree_against_forced_oracle

MICRO = dataclasses.replace(TINY, name="micro", hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16, mlp=96,
                            vocab=40, n_layers=2)
K, D, N, TOL = 3, 4, 12, 2e-2


def _state():
    tw = dec.weights_to_f64(make_decoder_weights(MICRO, 21, std=0.3))
    dw = dec.weights_to_f64(make_drafter_weights(MICRO, 21, std=0.3))
    st = sd.SeqState(MICRO, 96)
    root = sd.prefill(MICRO, tw, dw, st, [int(t) for t in prompts(1, 12, MICRO.vocab, seed=9)[0]])
    return tw, dw, st, root


def _disturbed(tw, dw, st, root, pick, score_shift=None):
    """A tree and pool as a lower-precision implementation would return them: the oracle's algorithm
    run with `pick`, scores shifted by `score_shift(pool index)`."""
    tree, pool = sd.draft_expand(MICRO, tw, dw, st, root, K, D, N, pick=pick)
    shift = score_shift or (lambda j: 0.0)
    p_sc = np.array([c.score + shift(j) for j, c in enumerate(pool)], dtype=np.float32)
    keep = [j for j in range(len(pool)) if any(
        pool[j].token == tree.token[i] and pool[j].depth == tree.depth[i] and abs(pool[j].score - tree.score[i]) < 1e-12
        for i in range(1, tree.n))]
    t_sc = np.concatenate([[0.0], p_sc[keep]]).astype(np.float32)
    g_pool = (np.array([c.token for c in pool]), np.array([c.parent for c in pool]), p_sc)
    return g_pool, (tree.token, tree.parent, tree.depth, t_sc)


def _check(tw, dw, st, root, g_pool, g_tree, tol=TOL):
    return check_draft_tree_against_forced_oracle(sd, MICRO, tw, dw, st, root, K, D, N, g_pool, g_tree, tol)


def test_the_oracles_own_tree_passes_and_is_recognised_as_identical():
    tw, dw, st, root = _state()
    seen = _check(tw, dw, st, root, *_disturbed(tw, dw, st, root, sd.pick_best))
    assert seen["identical"] and seen["choices"] == 1 + (D - 1) * K + (D - 2) + 1


def test_noise_inside_the_tolerance_passes():
    tw, dw, st, root = _state()
    rng = np.random.default_rng(0)

    def noisy(where, values, k):
        v = np.asarray(values, dtype=np.float64)
        spread = np.ptp(v[np.isfinite(v)])
        return sd.topk_desc(v + rng.normal(0, 0.2 * TOL * spread, size=v.shape), k)

    seen = _check(tw, dw, st, root, *_disturbed(tw, dw, st, root, noisy, lambda j: 1e-3 * np.sin(j)))
    assert seen["worst_slack"] <= 0 and seen["worst_score_err"] < 1


@pytest.mark.parametrize("where", ["root", "children", "frontier", "keep"])
def test_a_clearly_worse_choice_fails(where):
    tw, dw, st, root = _state()

    def wrong(w, values, k):
        best = sd.topk_desc(values, len(values))
        if w[0] == where and (where != "children" or w[1:] == (2, 1)) and (where != "frontier" or w[1] == 1):
            return best[: k - 1] + [best[-1]]        # the worst candidate takes the last place
        return best[:k]

    # (this toy drafter's rows spread over ~10 nats, so a depth-4 path's tolerance at 2e-2 is 0.8 nats: the
    # kept set's worst-for-best swap, 1.5 nats apart, is judged at a quarter of it)
    with pytest.raises(AssertionError):
        _check(tw, dw, st, root, *_disturbed(tw, dw, st, root, wrong), tol=TOL / 4)


def test_a_wrong_score_fails():
    tw, dw, st, root = _state()
    with pytest.raises(AssertionError):
        _check(tw, dw, st, root, *_disturbed(tw, dw, st, root, sd.pick_best, lambda j: 0.5 if j == 7 else 0.0))


def test_a_tree_that_is_not_the_pruning_of_its_pool_fails():
    tw, dw, st, root = _state()
    g_pool, (tok, par, dep, sc) = _disturbed(tw, dw, st, root, sd.pick_best)
    par = par.copy()
    par[-1] = 0 if par[-1] != 0 else 1
    with pytest.raises(AssertionError):
        _check(tw, dw, st, root, g_pool, (tok, par, dep, sc))
