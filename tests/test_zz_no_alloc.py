"""tlt_accept_sample_static (the entry point that allocates nothing: static device scratch inside the
library) against tlt_accept mode 1 on the same inputs, through the C ABI: two calls in a row, the
second on a smaller input (the scratch keeps the first call's contents), bit for bit."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import accept as oa
from paper_2511_16665_amd import binding as tlt
from synth import TINY, make_decoder_weights, synthetic_logits, uniforms_u32

pytestmark = pytest.mark.gpu


def _case(B, n, V, k, seed):
    rng = np.random.default_rng(seed)
    logits = synthetic_logits((B, n, V), seed=seed)
    ql = logits + rng.standard_normal(size=logits.shape).astype(np.float32)
    q = np.exp(ql - ql.max(axis=-1, keepdims=True))
    q = (q / q.sum(axis=-1, keepdims=True)).astype(np.float32)
    token = np.zeros((B, n), dtype=np.int32)
    parent = np.full((B, n), -1, dtype=np.int32)
    for b in range(B):
        nxt = 1
        for p in range(n):
            for t in oa.draw_without_replacement(q[b, p], k, rng):
                if nxt < n:
                    token[b, nxt], parent[b, nxt] = t, p
                    nxt += 1
    return token, parent, logits, q, uniforms_u32((B, n), seed + 1), uniforms_u32((B,), seed + 2)


def test_static_scratch_acceptance_equals_the_workspace_one_twice_in_a_row():
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    tau, stride = 0.9, 6
    for (B, n, V, k, seed) in [(4, 64, 152064, 3, 5), (3, 21, 1000, 4, 6)]:      # the second call is smaller
        token, parent, logits, q, u_acc, u_fin = _case(B, n, V, k, seed)
        cfg = dataclasses.replace(TINY, vocab=V, n_layers=1)
        ctx = tlt.Context(cfg, tlt.TLT_F32, make_decoder_weights(cfg, 1, device="cuda"), None, B, n, 8, 4, 4096)
        tree = tlt.Tree.empty(B, n)
        tree.token.copy_(dev(token))
        tree.parent.copy_(dev(parent))
        args = (dev(logits), dev(q), dev(u_acc), dev(u_fin))
        outs = lambda: [torch.full(s, -7, dtype=torch.int32, device="cuda") for s in ((B,), (B, stride), (B, stride), (B,))]
        want, got = outs(), outs()
        print(f"workspace call B={B} n={n} V={V}", flush=True)
        ctx.accept(B, 1, tau, tree, args[0], None, args[1], args[2], args[3], stride, *want)
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        print(f"static-scratch call B={B} n={n} V={V}", flush=True)
        rc = tlt.accept_sample_static(B, V, tau, tree, *args, stride, *got, status=status)
        assert rc == 0, tlt.ERRORS.get(rc, rc)
        torch.cuda.synchronize()
        assert int(status.item()) == 0 and ctx.device_status() == 0
        for g, w in zip(got, want):
            np.testing.assert_array_equal(g.cpu().numpy(), w.cpu().numpy())
        assert int(want[0].max()) >= 1
        # and both equal the oracle's rule
        o = oa.accept_sample(token, parent, logits, q, u_acc, u_fin, tau, stride)
        for g, w in zip(got, o):
            np.testing.assert_array_equal(g.cpu().numpy(), w)
        ctx.close()


def test_static_scratch_acceptance_rejects_what_does_not_fit():
    B, n, V = 8, 4, 152064                      # 8 * 152064 * 24 bytes > 16 MiB
    tree = tlt.Tree.empty(B, n)
    z = lambda *s: torch.zeros(s, dtype=torch.float32, device="cuda")
    i = lambda *s: torch.zeros(s, dtype=torch.int32, device="cuda")
    rc = tlt.accept_sample_static(B, V, 1.0, tree, z(1), z(1), i(B, n), i(B), 2, i(B), i(B, 2), i(B, 2), i(B))
    assert rc == -2
