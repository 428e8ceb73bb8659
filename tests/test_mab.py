"""The library's strategy selector (tlt_mab_*, host only) against the oracle of Algorithm 1: the
same strategies, thresholds and random draws must give the same decisions and bit-identical
rewards / medians; plus the argument checks of the C ABI."""
import math

import numpy as np
import pytest

from oracle.mab import BEG
from paper_2511_16665_amd import binding as tlt


def _random_setup(rng):
    widths = sorted(rng.choice([1, 4, 8, 16, 24, 32, 48, 64], size=int(rng.integers(1, 5)), replace=False).tolist())
    strategies = []
    for w in widths:
        for _ in range(int(rng.integers(1, 4))):
            strategies.append((int(rng.integers(1, 9)), int(rng.integers(1, 11)), int(w)))
    order = rng.permutation(len(strategies))
    strategies = [strategies[i] for i in order]
    thresholds = np.sort(rng.choice(np.arange(1, 40), size=len(widths), replace=False)).tolist()
    return strategies, thresholds


@pytest.mark.parametrize("seed", range(6))
def test_decisions_rewards_and_medians_match_the_oracle(seed):
    rng = np.random.default_rng(seed)
    strategies, thresholds = _random_setup(rng)
    eps, w, thr = float(rng.choice([0.0, 0.1, 0.5])), int(rng.integers(1, 7)), int(rng.integers(8, 64))
    ref = BEG(strategies, thresholds, eps, w, thr)
    mab = tlt.Mab(strategies, thresholds, eps, w, thr)
    for step in range(400):
        B = int(rng.integers(0, 70))
        u1, u2 = int(rng.integers(2 ** 32)), int(rng.integers(2 ** 32))
        want = ref.select(B, u1, u2)
        assert mab.select(B, u1, u2) == want, (step, B)
        if want is None or B == 0:
            continue
        lens = rng.integers(0, strategies[want][0] + 1, size=B).tolist()
        t = float(rng.uniform(1e-3, 5e-2))
        assert mab.record(want, t, lens, B) == ref.record(want, t, lens, B)      # bit-identical doubles
        for s in range(len(strategies)):
            m, n = mab.median_reward(s)
            assert n == len(ref.R[s]) and (m == ref.median(ref.R[s]) or (math.isinf(m) and n == 0))
    mab.close()


def test_argument_checks():
    S, T = [(4, 2, 8), (6, 8, 32)], [1, 16]
    for bad in (dict(thresholds=[1]), dict(thresholds=[16, 1]), dict(epsilon=1.5), dict(window=0), dict(sd_threshold=0),
                dict(strategies=[(4, 2, 0), (6, 8, 32)])):
        kw = dict(strategies=S, thresholds=T, epsilon=0.1, window=4, sd_threshold=32)
        kw.update(bad)
        with pytest.raises(tlt.TltError):
            tlt.Mab(**kw)
    mab = tlt.Mab(S, T, 0.1, 4)
    with pytest.raises(tlt.TltError):
        mab.record(2, 0.1, [1], 1)          # no such strategy
    with pytest.raises(tlt.TltError):
        mab.record(0, 0.0, [1], 1)          # non-positive time
    with pytest.raises(tlt.TltError):
        mab.record(0, 0.1, [-1], 1)         # negative accept length
    # widest trees (32) serve batch sizes 1..15, the 8-token strategy 16 and up; off from 32
    assert mab.select(32, 0, 0) is None and mab.select(31, 0, 0) == 0 and mab.select(3, 0, 0) == 1 and mab.select(0, 0, 0) == 1
    mab.close()
