"""The strategy selector driven by measured steps (bench.adaptive_rollout on a small model): every
choice the library's selector made is replayed through the oracle of Algorithm 1 with the same batch
sizes, random draws, elapsed times and accept lengths, and must be identical; the elastic rule keeps
speculation off at and above the threshold."""
import argparse

import pytest

from oracle.mab import BEG

pytestmark = pytest.mark.gpu


def test_selector_on_measured_steps_replays_identically_through_the_oracle():
    import bench
    args = argparse.Namespace(alpha=0.8, ctx_median=512, ctx_cap=512, steps=1, warmup=0)
    strategies = [(4, 3, 16), (2, 2, 16), (3, 3, 8), (2, 2, 8), (3, 2, 4)]
    thresholds, eps, w, sd_thr = (1, 3, 6), 0.25, 4, 12
    trace = []
    print("adaptive rollout on the mid-sized model", flush=True)
    res = bench.adaptive_rollout(args, model="mid", phases=(16, 12, 8, 5, 2, 1), steps_sd=14, steps_off=2, context=512,
                                 strategies=strategies, thresholds=thresholds, epsilon=eps, window=w, sd_threshold=sd_thr,
                                 seed=5, trace=trace)
    ref = BEG(strategies, list(thresholds), eps, w, sd_thr)
    n_on = 0
    for (B, u1, u2, choice, elapsed, lens) in trace:
        assert ref.select(B, u1, u2) == choice, (B, choice)
        if choice is not None:
            ref.record(choice, elapsed, lens, B)
            assert strategies[choice][2] == {1: 16, 2: 16, 5: 8, 8: 4}[B]       # the bucket's tree size
            n_on += 1
    assert n_on == 4 * 14
    off = [p for p in res["phases"] if p["speculation"] == "off"]
    assert [p["batch"] for p in off] == [16, 12]
    for p in res["phases"]:
        if p["speculation"] == "on":
            assert p["adaptive"] > 0 and set(p["chosen"]) <= set(p["fixed"])
            assert sum(p["chosen"].values()) == 14
