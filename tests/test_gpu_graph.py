"""The HIP-graph pool (bucketed, disaggregated, merged capture of the SD step; Section 5.1), the library's own
(tlt_graph_pool_*) and the one the Python engine keeps with torch's capture: every
replay must reproduce the eager step exactly, across several replays with other GPU work in between,
with strategies alternating so that graphs are shared and re-used; and capturing must not cost
device memory per graph."""
import numpy as np
import pytest
import torch

from paper_2511_16665_amd import binding as tlt
from synth import MID, prompts

from gpu_util import make_engine, make_models

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("native", [False, True], ids=["torch-capture", "library-pool"])
def test_graph_replays_match_eager_steps_and_graphs_are_shared(native):
    cfg = MID
    B, P = 4, 40
    tw_dev, dw_dev, _, _ = make_models(cfg, 21, "bf16", std=0.05)
    pr = prompts(B, P, cfg.vocab, seed=4)
    strategies = [(2, 3, 8), (3, 2, 6), (2, 3, 8), (2, 2, 8), (3, 2, 6), (2, 3, 8), (2, 3, 8)]   # (topK, depth, verify)
    engines = []
    for _ in range(2):
        e, _, _ = make_engine(cfg, "bf16", tw_dev, dw_dev, B, 8, 3, 3, P + 8 * len(strategies) * 4 + 64, seed=7)
        e.prefill(pr)
        engines.append(e)
    eager, graphed = engines
    free0 = torch.cuda.mem_get_info()[0]
    pool = graphed.graph_pool(native=native)
    # the first step runs eagerly on both: it creates the pending hidden state the pool's steps start from
    K, D, N = strategies[0]
    a0, o0 = eager.step(K, D, N)
    a1, o1 = graphed.step(K, D, N)
    np.testing.assert_array_equal(a0, a1)
    np.testing.assert_array_equal(o0, o1)
    for i, (K, D, N) in enumerate(strategies[1:]):
        print(f"step {i + 1}: strategy topK={K} depth={D} verify={N}", flush=True)
        want_al, want_out = eager.step(K, D, N)                    # eager work between the replays
        pool.step(B, K, D, N)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(graphed.accept_len.cpu().numpy(), want_al)
        np.testing.assert_array_equal(graphed.out_tokens.cpu().numpy(), want_out)
        np.testing.assert_array_equal(graphed.kv.seq_len.cpu().numpy(), eager.kv.seq_len.cpu().numpy())
        np.testing.assert_array_equal(graphed.dkv.seq_len.cpu().numpy(), eager.dkv.seq_len.cpu().numpy())
    n_draft, n_target = pool.n_graphs()
    print("graphs captured: draft", n_draft, "target", n_target, flush=True)
    # three distinct strategies; (2,3,8) and (2,2,8) verify 8 and 7 nodes, (3,2,6) verifies 6
    assert n_target == 3 and 3 <= n_draft <= 5
    used = free0 - torch.cuda.mem_get_info()[0]
    print(f"device memory taken by {n_draft + n_target} graphs: {used / 2**20:.1f} MiB", flush=True)
    assert used < 64 * 2**20
    for e in engines:
        e.ctx.close()


@pytest.mark.parametrize("native", [False, True], ids=["torch-capture", "library-pool"])
def test_smaller_batch_uses_the_bucket_graph(native):
    cfg = MID
    B, P = 8, 24
    tw_dev, dw_dev, _, _ = make_models(cfg, 22, "bf16", std=0.05)
    pr = prompts(B, P, cfg.vocab, seed=5)
    e, _, _ = make_engine(cfg, "bf16", tw_dev, dw_dev, B, 8, 3, 2, P + 200, seed=8)
    ref, _, _ = make_engine(cfg, "bf16", tw_dev, dw_dev, B, 8, 3, 2, P + 200, seed=8)
    for x in (e, ref):
        x.prefill(pr)
        x.step(2, 3, 8)
    pool = e.graph_pool(native=native)
    assert pool.bucket(3) == 4 and pool.bucket(5) == 8 and pool.bucket(1) == 1
    want_al, want_out = ref.step(2, 3, 8)
    pool.step(3, 2, 3, 8)                      # 3 running sequences -> bucket of 4: slots 0..3 advance
    torch.cuda.synchronize()
    np.testing.assert_array_equal(e.accept_len.cpu().numpy()[:4], want_al[:4])
    np.testing.assert_array_equal(e.out_tokens.cpu().numpy()[:4], want_out[:4])
    assert (e.kv.seq_len.cpu().numpy()[:4] == ref.kv.seq_len.cpu().numpy()[:4]).all()
    for x in (e, ref):
        x.ctx.close()
