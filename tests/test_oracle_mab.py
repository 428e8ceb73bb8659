"""Pins for the strategy-selector oracle (Algorithm 1, Section 5.2): bucket mapping, the Record
arithmetic, the |V| = 1 shortcut, window eviction and median-of-window exploitation worked by hand,
exploration frequency, and recovery on a simulated non-stationary bandit."""
import statistics

import numpy as np
import pytest

from oracle.mab import BEG

# (Draft_Depth, topK, Tokens_to_Verify); groups by Tokens_to_Verify descending: {64}, {32, 32}, {16}, {8, 8, 8}
S = [(4, 2, 8), (8, 10, 64), (6, 8, 32), (5, 4, 32), (3, 2, 8), (4, 4, 16), (2, 2, 8)]
T = [1, 3, 9, 17]


def test_groups_are_sorted_by_verify_tokens_descending_and_mapped_to_buckets_in_order():
    m = BEG(S, T, 0.1, 5, sd_threshold=1000)
    assert m.groups == [[1], [2, 3], [5], [0, 4, 6]]
    # B_1 = [1, 2], B_2 = [3, 8], B_3 = [9, 16], B_4 = [17, inf); below t_1 -> B_1
    want = {0: 0, 1: 0, 2: 0, 3: 1, 8: 1, 9: 2, 16: 2, 17: 3, 500: 3}
    assert {b: m.bucket(b) for b in want} == want


def test_thresholds_must_match_the_number_of_verify_token_values():
    with pytest.raises(ValueError):
        BEG(S, [1, 3, 9], 0.1, 5)
    with pytest.raises(ValueError):
        BEG(S, [1, 9, 3, 17], 0.1, 5)


def test_record_is_mean_emitted_tokens_and_tokens_per_unit_time():
    m = BEG(S, T, 0.1, 3)
    # 4 sequences accepted 2, 0, 5, 1 drafts: 8 drafts + 4 bonus tokens = 12 tokens in 0.5 s
    a_bar, r = m.record(2, 0.5, [2, 0, 5, 1], 4)
    assert a_bar == 3.0 and r == 24.0
    assert list(m.R[2]) == [24.0] and list(m.A[2]) == [3.0]


def test_single_candidate_bucket_ignores_the_random_draws():
    m = BEG(S, T, 1.0, 5, sd_threshold=1000)      # epsilon = 1 would always explore
    for U1 in (0, 2 ** 31, 2 ** 32 - 1):
        assert m.select(1, U1, 12345) == 1 and m.select(12, U1, 999) == 5


def test_elastic_rule_switches_speculation_off_at_the_threshold():
    m = BEG(S, T, 0.0, 5)                          # default threshold 32
    assert m.select(31, 0, 0) is not None and m.select(32, 0, 0) is None and m.select(400, 0, 0) is None


def test_exploit_takes_the_largest_window_median_and_untried_arms_first():
    m = BEG(S, T, 0.0, 3, sd_threshold=1000)       # never explores
    assert m.select(5, 0, 0) == 2                  # both untried: first of the group
    m.record(2, 1.0, [0], 1)                       # reward 1
    assert m.select(5, 0, 0) == 3                  # arm 3 still untried (median +inf)
    for t in (1.0, 0.5, 0.25):                     # rewards 1, 2, 4 -> median 2
        m.record(3, t, [0], 1)
    for t in (1 / 3, 1 / 3):                       # arm 2 window: 1, 3, 3 -> median 3
        m.record(2, t, [0], 1)
    assert m.select(5, 0, 0) == 2
    m.record(3, 0.1, [0], 1)                       # window of arm 3 slides to 2, 4, 10 -> median 4
    assert list(m.R[3]) == [2.0, 4.0, 10.0]
    assert m.select(5, 0, 0) == 3
    # even count: mean of the middle pair
    assert BEG.median([1.0, 7.0, 3.0, 5.0]) == 4.0 == statistics.median([1.0, 7.0, 3.0, 5.0])


def test_explore_picks_uniformly_from_the_candidates_with_probability_epsilon():
    m = BEG(S, T, 0.25, 4, sd_threshold=1000)
    for s in (0, 4, 6):
        m.record(s, 1.0 if s != 4 else 0.5, [0], 1)       # arm 4 is the best of bucket 4
    rng = np.random.default_rng(0)
    n = 40000
    picks = [m.select(20, int(rng.integers(2 ** 32)), int(rng.integers(2 ** 32))) for _ in range(n)]
    frac = {s: picks.count(s) / n for s in (0, 4, 6)}
    # exploit (0.75) always arm 4; explore (0.25) uniform over three arms
    assert abs(frac[4] - (0.75 + 0.25 / 3)) < 0.01 and abs(frac[0] - 0.25 / 3) < 0.01 and abs(frac[6] - 0.25 / 3) < 0.01
    # boundary of the explore test: u = (U1 + 0.5) / 2^32 < epsilon
    assert m.select(20, 2 ** 30 - 1, 0) == 0 and m.select(20, 2 ** 30, 0) == 4
    assert m.select(20, 0, 2 ** 32 - 1) == 6


def test_tracks_a_non_stationary_bandit():
    """Two arms whose step latencies swap half way: the windowed median forgets the old regime."""
    m = BEG([(4, 2, 8), (6, 4, 8)], [1], 0.1, 8, sd_threshold=1000)
    rng = np.random.default_rng(1)
    chosen = []
    for step in range(600):
        s = m.select(4, int(rng.integers(2 ** 32)), int(rng.integers(2 ** 32)))
        fast = 0 if step < 300 else 1
        latency = (1.0 if s == fast else 2.0) * (1 + 0.05 * rng.standard_normal())
        m.record(s, latency, [1, 1, 1, 1], 4)
        chosen.append(s)
    assert chosen[100:300].count(0) > 170 and chosen[400:].count(1) > 170
