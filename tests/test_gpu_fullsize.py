"""One SD step at the benchmark's full size and launch configuration (7B shape, bf16, batch 32,
long-tail contexts, depth 6 / top-k 8 / 48 verify tokens, built by bench.build_workload itself),
checked two ways:

* properties that hold at any size, for every sequence of the batch: tree invariants, acceptance
  bit-exact against the oracle's rule fed with the GPU's own argmax, cache length advance;
* sampled outputs: the shortest-context sequence goes through the oracle end to end (drafter extend
  and expand, all 28 target layers over the GPU's tree, LM head, acceptance, cache commit) and the
  logits, hidden states and committed cache rows are compared element by element (Section 2.2 for
  the verification forward, Section 5.1 for the tree).

Tolerance.  A bf16 decoder rounds its activations to bf16 between operations (the inputs of every
bf16 contraction), the float64 oracle does not.  Each block adds an independent relative error of
about 0.7e-2 this way (test_tolerance_model.py reproduces that figure on the CPU by rounding the
oracle's own activations), so the error of an L-block stack grows like sqrt(L): 2e-2 holds up to
four blocks and is asserted as such on the first four blocks at full width; the full 28-block stack is
held to 1e-2 * sqrt(L).
"""
import argparse
import dataclasses
import time

import numpy as np
import pytest
import torch

from oracle import accept as oacc
from oracle import decoder as dec
from oracle import sd

from paper_2511_16665_amd import binding as tlt

from gpu_util import EmbedRows as _EmbedRows
from gpu_util import LazyLayers as _LazyLayers
from gpu_util import check_draft_tree_against_forced_oracle, dense_cache, rel_err

pytestmark = pytest.mark.gpu

TOL = 2e-2


def stack_tol(n_layers):
    return max(TOL, 1e-2 * np.sqrt(n_layers))


def test_full_size_step_properties_and_sampled_parity():
    import bench

    args = argparse.Namespace(model="7b", batch=32, topk=8, depth=6, verify=48, ctx_median=4096, ctx_cap=16384,
                              steps=1, warmup=0, sweep=False)
    print("building the benchmark workload", flush=True)
    cfg, e, ctx, tw, dw, table, dtable, _ = bench.build_workload(args)
    B, K, D, N = args.batch, args.topk, args.depth, args.verify
    tok0 = e.out_tokens[:, 0].cpu().numpy().copy()
    hid0 = e.pending_hidden.cpu().numpy().astype(np.float64).copy()
    logits = torch.zeros((B * N, cfg.vocab), dtype=torch.float32, device="cuda")
    print("one SD step on the GPU", flush=True)
    al, out = e.step(K, D, N, logits_out=logits)
    g_pool = tuple(x[int(np.argmin(ctx))].cpu().numpy() for x in e.ctx.draft_pool(B, D, K))
    torch.cuda.synchronize()
    tree = e.tree(N)
    g_tok, g_par, g_dep, g_sc = (x.cpu().numpy() for x in (tree.token, tree.parent, tree.depth, tree.score))
    g_mask = tree.anc_mask.cpu().numpy().astype(np.uint64)
    g_am = e._buf("am", N).cpu().numpy()
    g_hid = e._buf("hid", N).cpu().numpy()
    g_path = e.path_idx.cpu().numpy()
    g_nout = e.n_out.cpu().numpy()
    step_logits = logits.view(B, N, -1).cpu().numpy().copy()      # (the device buffer is reused further down)

    # ---- properties, every sequence
    for b in range(B):
        assert g_tok[b, 0] == tok0[b] and g_par[b, 0] == -1 and g_dep[b, 0] == 0
        for i in range(1, N):
            p = g_par[b, i]
            assert 0 <= p < i and g_dep[b, i] == g_dep[b, p] + 1 <= D and g_sc[b, i] <= g_sc[b, p] + 1e-6
            assert g_mask[b, i] == (g_mask[b, p] | np.uint64(1 << i))
        kids = {}
        for i in range(1, N):
            key = (int(g_par[b, i]), int(g_tok[b, i]))
            assert key not in kids, "a parent has two children with one token"
            kids[key] = i
    np.testing.assert_array_equal(step_logits.argmax(-1), g_am)
    o_al, o_path, o_out, o_nout = oacc.accept_greedy(g_tok, g_par, step_logits, e.stride)
    np.testing.assert_array_equal(al, o_al)
    np.testing.assert_array_equal(g_nout, o_nout)
    for b in range(B):
        np.testing.assert_array_equal(g_path[b, : al[b] + 1], o_path[b, : al[b] + 1])
        np.testing.assert_array_equal(out[b, : al[b] + 1], o_out[b, : al[b] + 1])
    np.testing.assert_array_equal(e.kv.seq_len.cpu().numpy(), ctx + al + 1)
    np.testing.assert_array_equal(e.dkv.seq_len.cpu().numpy(), ctx + 1)

    # ---- sampled sequence through the oracle
    b = int(np.argmin(ctx))
    c = int(ctx[b])
    print(f"oracle on sequence {b} (context {c})", flush=True)
    t0 = time.time()
    cap = c + N + D * K + 16
    st = sd.SeqState(cfg, cap, dec.round_to_bf16)
    for l in range(cfg.n_layers):
        st.target[l].k[:c] = dense_cache(e.kv.k_pool[l:l + 1], table, b, c, cfg.page_size)[0]
        st.target[l].v[:c] = dense_cache(e.kv.v_pool[l:l + 1], table, b, c, cfg.page_size)[0]
    st.draft.k[:c] = dense_cache(e.dkv.k_pool, dtable, b, c, cfg.page_size)[0]
    st.draft.v[:c] = dense_cache(e.dkv.v_pool, dtable, b, c, cfg.page_size)[0]
    st.ctx = c
    st.draft_len = c
    tw64 = {"embed": _EmbedRows(tw["embed"]), "lm_head": dec.weights_to_f64(tw["lm_head"]),
            "final_norm": dec.weights_to_f64(tw["final_norm"]), "layers": _LazyLayers(tw["layers"])}
    dw64 = dec.weights_to_f64(dw)
    sd.draft_extend(cfg, tw64, dw64, st, [int(tok0[b])], hid0[b, :1])
    # the GPU's tree judged through the oracle's drafter run on the GPU's own choices (scores, optimality of
    # every choice within the tolerance, pruning, identity when no choice differs)
    seen = check_draft_tree_against_forced_oracle(sd, cfg, tw64, dw64, st, int(tok0[b]), K, D, N, g_pool,
                                                  (g_tok[b], g_par[b], g_dep[b], g_sc[b]), TOL)
    print("  drafter tree against the oracle's drafter on the same choices:", seen, flush=True)
    gtree = sd.Tree(g_tok[b].astype(np.int64), g_par[b].astype(np.int64), g_dep[b].astype(np.int64),
                    g_sc[b].astype(np.float64))
    # the first four blocks + LM head at full width, at the flat 2e-2 (same tree, untouched cache rows)
    L4 = 4
    small = dataclasses.replace(cfg, n_layers=L4)
    tws = dict(tw)
    tws["layers"] = tw["layers"][:L4]
    kv4 = tlt.KV(e.kv.k_pool[:L4].clone(), e.kv.v_pool[:L4].clone(), e.kv.block_table,
                 torch.from_numpy(ctx.astype(np.int32)).cuda(), int(ctx.max()))
    c4 = tlt.Context(small, tlt.TLT_BF16, tws, dw, B, N, D, K, int(ctx.max()) + 256)
    hid4 = torch.zeros((B, N, cfg.hidden), dtype=torch.float32, device="cuda")
    am_fused = torch.full((B, N), -1, dtype=torch.int32, device="cuda")
    c4.verify_forward(B, tree, kv4, out_argmax=am_fused, out_hidden=hid4)      # argmax alone: the fused LM head
    torch.cuda.synchronize()
    am_plain = torch.full((B, N), -1, dtype=torch.int32, device="cuda")
    logits.zero_()
    c4.verify_forward(B, tree, kv4, out_logits=logits, out_argmax=am_plain)   # same rows with the logits stored
    torch.cuda.synchronize()
    np.testing.assert_array_equal(am_plain.cpu().numpy(), logits.view(B, N, -1).argmax(-1).cpu().numpy())
    # Two forwards over the same rows are bit-identical: products that are cut along K keep their partial
    # products apart and the consumer sums them in a fixed order (no atomic accumulation anywhere in the
    # forward), so the fused head must pick exactly the stored logits' argmax.
    logits2 = torch.zeros_like(logits)
    c4.verify_forward(B, tree, kv4, out_logits=logits2)
    torch.cuda.synchronize()
    noise = float((logits2 - logits).abs().max())
    del logits2
    differ = int((am_fused != am_plain).sum().item())
    print(f"  fused LM-head argmax (1536 x 152064): {differ} rows differ from the stored logits' argmax; run-to-run "
          f"difference of the logits {noise:.2e}", flush=True)
    assert noise == 0.0 and differ == 0
    st4 = sd.SeqState(small, cap, dec.round_to_bf16)
    for l in range(L4):
        st4.target[l].k[:c] = st.target[l].k[:c]
        st4.target[l].v[:c] = st.target[l].v[:c]
    st4.ctx = c
    tw64_4 = dict(tw64)
    tw64_4["layers"] = _LazyLayers(tw["layers"][:L4])
    _, o_hid4 = sd.verify(small, tw64_4, st4, gtree)
    e4 = rel_err(hid4[b].cpu().numpy(), o_hid4)
    print(f"  first {L4} blocks: rel err hidden {e4:.3e}", flush=True)
    assert e4 <= TOL
    c4.close()
    del kv4, hid4
    # verification over the GPU's tree, all blocks
    o_logits, o_hidden = sd.verify(cfg, tw64, st, gtree)
    print(f"  oracle done in {time.time() - t0:.1f} s", flush=True)
    g_logits = step_logits[b]
    e_log, e_hid = rel_err(g_logits, o_logits), rel_err(g_hid[b], o_hidden)
    print(f"  rel err logits {e_log:.3e} hidden {e_hid:.3e}", flush=True)
    tol = stack_tol(cfg.n_layers)
    assert e_log <= tol and e_hid <= tol
    scale = np.abs(o_logits).max()
    for i in range(N):
        srt = np.sort(o_logits[i])
        if srt[-1] - srt[-2] > 2 * tol * scale:
            assert g_am[b, i] == int(np.argmax(o_logits[i]))
    # committed cache rows: the accepted path's keys/values at ctx .. ctx+a in every layer
    a = int(al[b])
    sd.commit(st, [int(p) for p in g_path[b, : a + 1]])
    worst = 0.0
    for l in range(cfg.n_layers):
        gk = dense_cache(e.kv.k_pool[l:l + 1], table, b, c + a + 1, cfg.page_size)[0]
        gv = dense_cache(e.kv.v_pool[l:l + 1], table, b, c + a + 1, cfg.page_size)[0]
        np.testing.assert_array_equal(gk[:c], st.target[l].k[:c])
        worst = max(worst, rel_err(gk[c:], st.target[l].k[c:c + a + 1]), rel_err(gv[c:], st.target[l].v[c:c + a + 1]))
    print(f"  committed cache rows rel err {worst:.3e}", flush=True)
    assert worst <= tol
    e.ctx.close()


def test_full_size_sampled_step_long_tail_shape():
    """One SAMPLED step at the long-tail phase's shape (7B, 4 sequences of 24k-32k tokens, static
    template of depth 8 / topK 10 / 64 nodes, temperature 0.9), all 28 blocks and the full
    vocabulary: template shape, every child draw exact given the GPU's own distribution, acceptance
    bit-exact against the oracle's rule on the GPU's logits and distributions, cache lengths; and
    the drafter's distributions of one sequence against the oracle's drafter on the same tokens."""
    import bench
    from oracle import sample_draft as osd

    B, K, D, N, tau = 4, 10, 8, 64, 0.9
    args = argparse.Namespace(model="7b", batch=B, topk=K, depth=D, verify=N, ctx_median=28672, ctx_cap=32768, ctx_lo=24576,
                              steps=1, warmup=0, sweep=False)
    print("building the long-tail workload", flush=True)
    cfg, e, ctx, tw, dw, table, dtable, _ = bench.build_workload(args)
    assert ctx.min() >= 24576 and ctx.max() <= 32768
    parent, rank, depth = osd.static_template(K, D, N)
    n = len(parent)
    rng = np.random.default_rng(17)
    u32 = lambda *s: rng.integers(0, 2**32, size=s, dtype=np.uint64).astype(np.uint32)
    u_d, u_a, u_f = u32(B, n), u32(B, n), u32(B)
    dev = lambda a: torch.from_numpy(a.view(np.int32)).cuda()
    tok0 = e.out_tokens[:, 0].cpu().numpy().copy()
    hid0 = e.pending_hidden.cpu().numpy().astype(np.float64).copy()
    print("one sampled SD step on the GPU", flush=True)
    al, out = e.step_sampled(K, D, N, tau, dev(u_d), dev(u_a), dev(u_f))
    tree = e.tree(n)
    g_tok, g_par, g_dep = (x.cpu().numpy() for x in (tree.token, tree.parent, tree.depth))
    g_q, g_logits = e.draft_q(n).cpu().numpy(), e.logits(n).cpu().numpy()
    kids = [[c for c in range(n) if parent[c] == i] for i in range(n)]
    inner = [i for i in range(n) if kids[i]]
    for b in range(B):
        np.testing.assert_array_equal(g_par[b], parent)
        np.testing.assert_array_equal(g_dep[b], depth)
        assert g_tok[b, 0] == tok0[b]
        rows = g_q[b, inner]
        assert np.abs(rows.astype(np.float64).sum(axis=1) - 1.0).max() < 1e-3
        for i in inner:          # exact draws, given the GPU's distribution
            want = osd.draw_children_rows(g_q[b, i][None, :], u_d[b, kids[i]][None, :])[0]
            np.testing.assert_array_equal(g_tok[b, kids[i]], want)
    print("acceptance against the oracle's rule", flush=True)
    o_al, o_path, o_out, o_nout, near = oacc.accept_sample(g_tok, g_par, g_logits, g_q, u_a, u_f, tau, e.stride,
                                                           with_near=True)
    differ = oacc.assert_equal_unless_near((al, e.path_idx.cpu().numpy(), out, e.n_out.cpu().numpy()),
                                           (o_al, o_path, o_out, o_nout), near, "sampled step")
    print(f"  near-threshold sequences {int(near.sum())}, differing {differ}", flush=True)
    assert near.sum() <= 1
    np.testing.assert_array_equal(e.kv.seq_len.cpu().numpy(), ctx + al + 1)
    np.testing.assert_array_equal(e.dkv.seq_len.cpu().numpy(), ctx + 1)
    print("  accept lengths", al, flush=True)

    # the drafter's distributions of the shortest sequence
    b = int(np.argmin(ctx))
    c = int(ctx[b])
    print(f"oracle drafter on sequence {b} (context {c})", flush=True)
    st = sd.SeqState(dataclasses.replace(cfg, n_layers=1), c + n + 16, dec.round_to_bf16)
    # (the committed drafter cache was not touched by the step: provisional rows sit past it)
    st.draft.k[:c] = dense_cache(e.dkv.k_pool, dtable, b, c, cfg.page_size)[0]
    st.draft.v[:c] = dense_cache(e.dkv.v_pool, dtable, b, c, cfg.page_size)[0]
    st.draft_len = c
    tw64 = {"embed": _EmbedRows(tw["embed"]), "lm_head": dec.weights_to_f64(tw["lm_head"]),
            "final_norm": dec.weights_to_f64(tw["final_norm"])}
    dw64 = dec.weights_to_f64(dw)
    sd.draft_extend(cfg, tw64, dw64, st, [int(tok0[b])], hid0[b, :1])
    _, o_q = osd.draft_sample(cfg, tw64, dw64, st, int(tok0[b]), K, D, N, tau, u_d[b], forced_tokens=g_tok[b])
    worst = 0.0
    for i in inner:
        lq = np.log(o_q[i][o_q[i] > 0].astype(np.float64))
        worst = max(worst, rel_err(g_q[b, i], o_q[i]) / (lq.max() - lq.min()))
    print(f"  worst rel err of q / spread of log q {worst:.3e}", flush=True)
    assert worst <= TOL
    e.ctx.close()
