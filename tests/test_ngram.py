"""The library's model-free drafter (tlt_ngram_*, host only) against its oracle on synthetic
rollouts with planted repeats: identical trees and scores; argument checks."""
import numpy as np
import pytest

from oracle.ngram import NGramDB
from paper_2511_16665_amd import binding as tlt


def _rollouts(rng, vocab, n_prompts, per_prompt, length):
    """Sibling responses of a prompt share planted phrases (the similarity the drafter feeds on)."""
    out = {}
    for p in range(n_prompts):
        phrases = [rng.integers(0, vocab, size=int(rng.integers(4, 12))).tolist() for _ in range(5)]
        seqs = []
        for _ in range(per_prompt):
            s = []
            while len(s) < length:
                s += phrases[int(rng.integers(len(phrases)))] if rng.random() < 0.7 else rng.integers(0, vocab, size=3).tolist()
            seqs.append(s[:length])
        out[p] = seqs
    return out


@pytest.mark.parametrize("seed,order,vocab", [(0, 3, 50), (1, 4, 12), (2, 2, 6), (3, 5, 1000)])
def test_trees_match_the_oracle(seed, order, vocab):
    rng = np.random.default_rng(seed)
    data = _rollouts(rng, vocab, 3, 4, 80)
    ref, db = NGramDB(order), tlt.NGram(order)
    for p, seqs in data.items():
        for s in seqs[:-1]:                       # the last sibling is the one being generated
            ref.insert(p, s)
            db.insert(p, s)
    hits = 0
    for p, seqs in data.items():
        s = seqs[-1]
        for pos in range(1, len(s), 7):
            K, D, N = int(rng.integers(1, 5)), int(rng.integers(0, 6)), int(rng.integers(1, 20))
            ctx = s[max(0, pos - 6):pos]
            want_tok, want_par, want_sc = ref.propose(p, ctx, D, K, N)
            tok, par, sc = db.propose(p, ctx, D, K, N)
            assert tok.tolist() == want_tok and par.tolist() == want_par
            np.testing.assert_array_equal(sc, np.asarray(want_sc, dtype=np.float32))
            hits += sum(np.isfinite(want_sc[1:]))
    assert hits > 0
    db.close()


def test_argument_checks():
    with pytest.raises(tlt.TltError):
        tlt.NGram(1)
    db = tlt.NGram(3)
    with pytest.raises(tlt.TltError):
        db.propose(0, [], 2, 2, 4)
    with pytest.raises(tlt.TltError):
        db.propose(0, [1], 2, 0, 4)
    tok, par, sc = db.propose(0, [3], 4, 2, 3)           # empty database: root + padding
    assert tok.tolist() == [3, 0, 1] and par.tolist() == [-1, 0, 0]
    db.close()
