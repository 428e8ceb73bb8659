"""Pins for the model-free (n-gram) drafter's oracle: a worked example computed by hand, back-off,
the planted-repeat closed form, tie-breaking, padding and the tree invariants."""
import math

import numpy as np

from oracle.ngram import NGramDB


def test_worked_example_counts_and_tree():
    db = NGramDB(3)
    db.insert(7, [1, 2, 3, 1, 2, 4, 1, 2, 3])
    # windows: (1,2)->3 twice, (1,2)->4 once; (2,3)->1 once; (2,4)->1 once; (3,1)->2, (4,1)->2; (2)->3 x2, (2)->4 ...
    assert db.continuations(7, [9, 1, 2]) == [(3, math.log(2 / 3)), (4, math.log(1 / 3))]
    assert db.continuations(7, [2, 3]) == [(1, 0.0)]
    assert db.continuations(8, [1, 2]) == []                       # another prompt's rollouts are not shared
    tok, par, sc = db.propose(7, [5, 1, 2], depth=3, K=2, N=6, pad=False)
    # level 1: 3 (log 2/3), 4 (log 1/3); level 2: 3->1 (+0), 4->1 (+0); level 3: (3,1)->2, (4,1)->2
    assert tok == [2, 3, 4, 1, 1, 2]
    assert par == [-1, 0, 0, 1, 2, 3]
    np.testing.assert_allclose(sc, [0, math.log(2 / 3), math.log(1 / 3), math.log(2 / 3), math.log(1 / 3), math.log(2 / 3)])


def test_backs_off_to_shorter_contexts():
    db = NGramDB(4)
    db.insert(0, [10, 11, 12, 13])
    assert db.continuations(0, [10, 11, 12]) == [(13, 0.0)]         # full 3-token context
    assert db.continuations(0, [99, 11, 12]) == [(13, 0.0)]         # unseen 3-context -> (11, 12)
    assert db.continuations(0, [99, 98, 12]) == [(13, 0.0)]         # -> (12,)
    assert db.continuations(0, [99, 98, 97]) == []


def test_planted_repeat_is_proposed_as_a_chain_of_certain_tokens():
    rng = np.random.default_rng(0)
    body = rng.permutation(1000)[:40].tolist()                      # all tokens distinct: every context is unique
    db = NGramDB(4)
    db.insert(3, body)
    tok, par, sc = db.propose(3, body[:10], depth=6, K=3, N=7, pad=False)
    assert tok == [body[9]] + body[10:16] and par == [-1, 0, 1, 2, 3, 4, 5] and sc == [0.0] * 7


def test_equal_counts_rank_by_token_id_and_padding_fills_root_children():
    db = NGramDB(2)
    db.insert(1, [5, 9, 5, 3, 5, 7])
    assert [t for t, _ in db.continuations(1, [5])] == [3, 7, 9]
    tok, par, sc = db.propose(1, [5], depth=1, K=2, N=6)
    assert tok == [5, 3, 7, 0, 1, 2] and par == [-1, 0, 0, 0, 0, 0]
    assert sc[3:] == [-math.inf] * 3
    assert db.propose(1, [5], depth=0, K=2, N=3)[0] == [5, 0, 1]      # depth 0 proposes nothing: padding only
    tok, par, _ = db.propose(1, [4], depth=2, K=2, N=4)               # nothing known: root + padding only
    assert tok == [4, 0, 1, 2] and par == [-1, 0, 0, 0]


def test_tree_invariants_on_random_rollouts():
    rng = np.random.default_rng(5)
    db = NGramDB(3)
    for _ in range(6):
        db.insert(0, rng.integers(0, 6, size=60))
    for _ in range(20):
        ctx = rng.integers(0, 6, size=5).tolist()
        K, D, N = int(rng.integers(1, 4)), int(rng.integers(1, 5)), int(rng.integers(1, 12))
        tok, par, sc = db.propose(0, ctx, D, K, N)
        assert len(tok) == N and tok[0] == ctx[-1] and par[0] == -1
        depth = [0] * N
        for i in range(1, N):
            assert 0 <= par[i] < i and sc[i] <= sc[par[i]] + 1e-12
            depth[i] = depth[par[i]] + 1
            assert depth[i] <= D
        for p in range(N):
            kids = [tok[i] for i in range(1, N) if par[i] == p]
            assert len(kids) == len(set(kids))
            if p > 0:
                assert len(kids) <= K
