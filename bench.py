#!/usr/bin/env python3
"""Benchmark of the speculative-decoding step on one MI355X.

Workload (the configuration the metric is quoted on): Qwen2.5-7B-shaped target, random-init bf16,
1-layer drafter of the same width, batch 32, contexts lognormal(median 4096, sigma 0.8, floor 256,
cap 16384) in a paged KV cache with 16-token pages filled with N(0,1), tree depth 6 / top-k 8 /
48 verify tokens, greedy acceptance.  One step = tlt_draft_expand + tlt_verify_forward + tlt_accept
+ tlt_kv_commit over the whole batch, inputs resident in HBM.

Prints ONE JSON line: accepted tokens/s (value), plus the roofline of the dominant kernel (the
bf16 MFMA GEMM of the verification forward, timed per launch with HIP events inside the library),
verify latency versus tree size, and the CPU oracle timed on a bounded sample of the same
workload as a baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0


def build_workload(args, shared=None):
    import torch

    from paper_2511_16665_amd import binding as tlt
    from paper_2511_16665_amd import engine as eng
    from synth import (QWEN7B, QWEN32B, MID, fill_kv_pool, lognormal_contexts, make_decoder_weights,
                       make_drafter_weights, random_block_table)

    cfg = {"7b": QWEN7B, "32b": QWEN32B, "mid": MID}[args.model]
    B, K, D, N = args.batch, args.topk, args.depth, args.verify
    if getattr(args, "ctx_lo", None):   # the long-tail phase's few, long sequences: uniform lengths
        ctx = np.random.default_rng(0).integers(args.ctx_lo, args.ctx_cap + 1, size=B).astype(np.int32)
    else:
        ctx = lognormal_contexts(B, args.ctx_median, 0.8, args.ctx_cap, min(256, args.ctx_median), seed=0)
    grow = (args.steps + args.warmup + 8) * (min(D, N - 1) + 1) * 2 + 64 + N
    caps = ctx + grow + max(D - 1, 0) * K
    table, n_pages = random_block_table(caps, cfg.page_size, seed=1, extra_pages=8)
    dtable, dn_pages = random_block_table(caps, cfg.page_size, seed=2, extra_pages=8)
    dt = torch.bfloat16
    t0 = time.time()
    if shared is None:
        tw = make_decoder_weights(cfg, 1234, device="cuda", dtype=dt)
        dw = make_drafter_weights(cfg, 1234, device="cuda", dtype=dt)
    else:
        tw, dw = shared
    kfill = fill_kv_pool(cfg.n_layers, n_pages, cfg.n_kv_heads, cfg.page_size, cfg.head_dim, 3, "cuda", dt)
    dfill = fill_kv_pool(1, dn_pages, cfg.n_kv_heads, cfg.page_size, cfg.head_dim, 4, "cuda", dt)
    kv = eng.alloc_kv(cfg, tlt.TLT_BF16, cfg.n_layers, table, n_pages, ctx, fill=kfill)
    dkv = eng.alloc_kv(cfg, tlt.TLT_BF16, 1, dtable, dn_pages, ctx, fill=dfill)
    max_ctx = int(caps.max()) + 64
    e = eng.Engine(cfg, tlt.TLT_BF16, tw, dw, B, max(N, 64) if args.sweep else N, D, K, max_ctx, kv, dkv)
    # the drafter starts one entry behind: (root token, hidden state of the last committed position)
    g = torch.Generator(device="cuda").manual_seed(5)
    tok = torch.randint(0, cfg.vocab, (B, 1), generator=g, device="cuda", dtype=torch.int32)
    hid = torch.randn((B, 1, cfg.hidden), generator=g, device="cuda", dtype=torch.float32)
    src = torch.zeros((B, 1), dtype=torch.int32, device="cuda")
    one = torch.ones((B,), dtype=torch.int32, device="cuda")
    e.set_pending(tok, src, one, hid, 1)
    torch.cuda.synchronize()
    setup_s = time.time() - t0
    return cfg, e, ctx, tw, dw, table, dtable, setup_s


def verify_latency_sweep(cfg, e, sizes, iters=3):
    """Latency of tlt_verify_forward alone versus the number of tree nodes (chain trees)."""
    import torch
    out = {}
    B = e.B
    for n in sizes:
        t = e.tree(n)
        t.token.copy_(torch.randint(0, cfg.vocab, (B, n), device="cuda", dtype=torch.int32))
        t.parent.copy_(torch.arange(-1, n - 1, dtype=torch.int32, device="cuda").expand(B, n))
        e.ctx.tree_finalize(B, t)
        am = e._buf("am", n)
        e.ctx.verify_forward(B, t, e.kv, None, am, None)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            e.ctx.verify_forward(B, t, e.kv, None, am, None)
        torch.cuda.synchronize()
        out[str(n)] = round((time.perf_counter() - t0) / iters * 1e3, 3)
    return out


def fixed_acceptance_steps(cfg, e, K, D, N, alpha, steps, warmup=1, seed=17):
    """The same four calls with a stand-in for a TRAINED drafter.  A random-init drafter is almost
    never right, so the headline steps accept nothing; here the verified tree is the static template
    of (topK, Draft_Depth, Tokens_to_Verify) and its tokens are set (outside the timed region) so
    that a node's first child carries the target's own greedy token with probability alpha and every
    other node a random token: the accept length is geometric in alpha along the first-child chain.
    The target's greedy token at a node needs the node's ancestors' tokens, so the labelling takes one
    verification forward per tree level (untimed).  Timed per step (HIP events on the launch stream):
    tlt_draft_expand (the real drafter at the same strategy: it consumes the tokens and hidden
    states the step before accepted; its tree is discarded) and tlt_verify_forward + tlt_accept +
    tlt_kv_commit on the labelled tree."""
    import torch

    from paper_2511_16665_amd import binding as tlt
    B = e.B
    pool = K + (D - 1) * K * K if D >= 1 else 0
    t = e.tree(min(N, 1 + pool))                       # the drafter's own tree (discarded)
    par, rank, dep = tlt.template_build(K, D, N)
    n = len(par)
    ts = tlt.Tree.empty(B, n)
    ts.parent.copy_(torch.from_numpy(par).cuda().expand(B, n))
    e.ctx.tree_finalize(B, ts)
    hid, am = e._buf("hid", n), e._buf("am", n)
    gen = torch.Generator(device="cuda").manual_seed(seed)
    parent = ts.parent.long()
    depth = torch.from_numpy(dep.astype(np.int64)).cuda().expand(B, n)
    first_child = torch.from_numpy(rank == 0).cuda().expand(B, n)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    emitted, ms, accept_hist = 0, 0.0, []
    for it in range(warmup + steps):
        ev[0].record()
        e.ctx.draft_expand(B, D, K, N, e.out_tokens, e.path_idx, e.n_out, e.pending_hidden, None, e.dkv, t)
        ev[1].record()
        e.dkv.seq_len_bound += e.pending_max_new
        # ---- untimed: label the template level by level (the root is the token the last step ended with)
        hit = first_child & (torch.rand((B, n), generator=gen, device="cuda") < alpha)
        rnd = torch.randint(0, cfg.vocab, (B, n), generator=gen, device="cuda", dtype=torch.int32)
        ts.token.copy_(rnd)
        ts.token[:, 0] = t.token[:, 0]
        for d in range(int(dep.max())):
            e.ctx.verify_forward(B, ts, e.kv, out_logits=None, out_argmax=am, out_hidden=None)
            level = depth == d + 1
            from_parent = torch.gather(am, 1, parent.clamp(min=0)).to(torch.int32)
            other = torch.where(rnd == from_parent, (rnd + 1) % cfg.vocab, rnd)   # never the greedy token by chance
            ts.token.copy_(torch.where(level, torch.where(hit, from_parent, other), ts.token))
        # ---- timed: verification, acceptance, commit
        ev[2].record()
        e.ctx.verify_forward(B, ts, e.kv, out_logits=None, out_argmax=am, out_hidden=hid)
        e.ctx.accept(B, 0, 1.0, ts, None, am, None, None, None, e.stride, e.accept_len, e.path_idx, e.out_tokens, e.n_out)
        e.ctx.kv_commit(B, e.kv, e.accept_len, e.path_idx, e.stride)
        ev[3].record()
        torch.cuda.synchronize()
        e.pending_hidden, e.have_pending = hid, True
        al = e.accept_len.cpu().numpy()
        inc = int(al.max()) + 1
        e.kv.seq_len_bound += inc
        e.pending_max_new = inc
        if it >= warmup:
            ms += ev[0].elapsed_time(ev[1]) + ev[2].elapsed_time(ev[3])
            emitted += int(al.sum()) + B
            accept_hist.append(float(al.mean()))
    chain = int(dep[rank == 0].max()) if n > 1 else 0
    return {"alpha": alpha, "steps": steps, "ms_per_step": round(ms / steps, 3),
            "accepted_per_step": round(emitted / steps, 2), "mean_accept_length": round(float(np.mean(accept_hist)), 3),
            "expected_accept_length": round(sum(alpha ** k for k in range(1, chain + 1)), 3),
            "value": round(emitted / (ms * 1e-3), 2), "unit": "accepted tokens/s",
            "note": "stand-in for a trained drafter: static-template tree whose first children are the target's greedy "
                    "token with probability alpha (labelled untimed); timed: draft_expand + verify_forward + accept + kv_commit"}


def noisy_target_steps(cfg, e, K, D, N, steps, warmup=1, sigma=1.0, tau=1.0, seed=23, profile=False):
    """The long-tail workload's step (sampling at temperature tau, rejection-sampling acceptance) with the
    drafter the benchmark spec prescribes for it: draft distributions q = softmax(target logits + N(0, sigma^2)),
    which fixes the acceptance rate (first-child accept probability sum_v min(p_v, q_v), about 0.617 for
    sigma = 1 on a large flat vocabulary).  No trained drafter exists here, so the verified tree is built
    OUTSIDE the timed region, level by level on the static template of (topK, Draft_Depth,
    Tokens_to_Verify): one verification forward per level gives the target logits of that level's nodes,
    q is formed from them and each node's children are drawn from q without replacement with the library's
    integer rule (weights floor(q * 2^32), first index whose running sum exceeds (U * total) >> 32, the
    picked weight zeroed).  Timed per step, HIP events on the launch stream: the real drafter's
    tlt_draft_sample at the same strategy (it consumes the tokens and hidden states the step before
    accepted; its tree and distributions are discarded, its cost counts) and tlt_verify_forward +
    tlt_accept (mode 1) + tlt_kv_commit on the labelled tree.  profile: the library's per-launch events are
    switched on for the timed calls only (the caller reads them afterwards)."""
    import torch

    from paper_2511_16665_amd import binding as tlt
    B, V = e.B, cfg.vocab
    par, rank, dep = tlt.template_build(K, D, N)
    n = len(par)
    kids = [[c for c in range(n) if par[c] == i] for i in range(n)]
    t_draft, q_draft = e.tree(n), e.draft_q(n)             # what the real drafter writes (discarded)
    ts = tlt.Tree.empty(B, n)
    ts.parent.copy_(torch.from_numpy(par).cuda().expand(B, n))
    e.ctx.tree_finalize(B, ts)
    q = torch.zeros((B, n, V), dtype=torch.float32, device="cuda")
    logits, hid = e.logits(n), e._buf("hid", n)
    gen = torch.Generator(device="cuda").manual_seed(seed)
    u32 = lambda *shape: torch.randint(-2**31, 2**31 - 1, shape, generator=gen, device="cuda", dtype=torch.int32)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    emitted, ms, ms_draft, tests, hits, closed_form, accept_hist = 0, 0.0, 0.0, 0, 0, [], []
    for it in range(warmup + steps):
        u_draw, u_acc, u_fin = u32(B, n), u32(B, n), u32(B)
        if profile:
            e.ctx.profile_begin(1 if it == 0 else 2)
        ev[0].record()
        e.ctx.draft_sample(B, D, K, N, tau, e.out_tokens, e.path_idx, e.n_out, e.pending_hidden, None, e.dkv, u_draw,
                           t_draft, q_draft)
        ev[1].record()
        if profile:
            e.ctx.profile_begin(0)
        e.dkv.seq_len_bound += e.pending_max_new
        # ---- untimed: the noisy-target drafter's tree, level by level
        ts.token.fill_(0)
        ts.token[:, 0] = t_draft.token[:, 0]               # the root: the token the last step ended with
        U = (u_draw.cpu().numpy().astype(np.int64) & 0xFFFFFFFF)
        for d in range(int(dep.max())):
            e.ctx.verify_forward(B, ts, e.kv, out_logits=logits, out_argmax=None, out_hidden=None)
            for i in [i for i in range(n) if dep[i] == d and kids[i]]:
                noisy = logits[:, i] + sigma * torch.randn((B, V), generator=gen, device="cuda")
                qi = torch.softmax(noisy / tau, dim=-1)
                q[:, i] = qi
                if i == 0 and it >= warmup:
                    p0 = torch.softmax(logits[:, 0].double() / tau, dim=-1)
                    closed_form.extend(torch.minimum(p0, qi.double()).sum(-1).tolist())
                w = torch.floor(qi.double() * 4294967296.0).to(torch.int64)
                for c in kids[i]:
                    tot = w.sum(dim=1).tolist()
                    thr = torch.tensor([(int(U[b, c]) * int(tot[b])) >> 32 for b in range(B)], dtype=torch.int64, device="cuda")
                    pick = torch.searchsorted(torch.cumsum(w, dim=1), thr.unsqueeze(1), right=True).squeeze(1).clamp(max=V - 1)
                    ts.token[:, c] = pick.to(torch.int32)
                    w.scatter_(1, pick.unsqueeze(1), 0)
        # ---- timed: verification, acceptance, commit
        if profile:
            e.ctx.profile_begin(2)
        ev[2].record()
        e.ctx.verify_forward(B, ts, e.kv, out_logits=logits, out_argmax=None, out_hidden=hid)
        e.ctx.accept(B, 1, tau, ts, logits, None, q, u_acc, u_fin, e.stride, e.accept_len, e.path_idx, e.out_tokens, e.n_out)
        e.ctx.kv_commit(B, e.kv, e.accept_len, e.path_idx, e.stride)
        ev[3].record()
        if profile:
            e.ctx.profile_begin(0)
        torch.cuda.synchronize()
        e.ctx.device_status()
        e.pending_hidden, e.have_pending = hid, True
        al = e.accept_len.cpu().numpy()
        path = e.path_idx.cpu().numpy()
        inc = int(al.max()) + 1
        e.kv.seq_len_bound += inc
        e.pending_max_new = inc
        if it >= warmup:
            ms_draft += ev[0].elapsed_time(ev[1])
            ms += ev[0].elapsed_time(ev[1]) + ev[2].elapsed_time(ev[3])
            emitted += int(al.sum()) + B
            accept_hist.append(float(al.mean()))
            for b in range(B):             # every visited node with children tested its first child first
                for j in range(int(al[b]) + 1):
                    node = int(path[b, j])
                    if kids[node] and j + 1 < e.stride:
                        tests += 1
                        hits += int(j + 1 <= al[b] and path[b, j + 1] == kids[node][0])
    rate = hits / max(tests, 1)
    return {"sigma": sigma, "temperature": tau, "steps": steps, "ms_per_step": round(ms / steps, 3),
            "ms_draft_sample": round(ms_draft / steps, 3), "accepted_per_step": round(emitted / steps, 2),
            "mean_accept_length": round(float(np.mean(accept_hist)), 3),
            "first_child_accept_rate": round(rate, 4), "first_child_tests": tests,
            "first_child_accept_rate_ci95": round(1.96 * float(np.sqrt(max(rate * (1 - rate), 1e-9) / max(tests, 1))), 4),
            "closed_form_sum_min_p_q_at_root": round(float(np.mean(closed_form)), 4) if closed_form else None,
            "closed_form_flat_vocab": 0.6171,
            "value": round(emitted / (ms * 1e-3), 2), "unit": "accepted tokens/s"}


def _gather_rows(pool_layer, table_row, c, page_size):
    """First c cache rows of one sequence in one layer as float64 [c, Hkv, d]."""
    import torch
    slots = np.arange(c)
    pg = torch.from_numpy(table_row[slots // page_size].astype(np.int64)).cuda()
    off = torch.from_numpy((slots % page_size).astype(np.int64)).cuda()
    return pool_layer[pg, :, off].double().cpu().numpy()


class _EmbedRows:
    """Embedding table kept on the device; rows are widened to float64 when the oracle indexes it."""

    def __init__(self, t):
        self.t = t

    def __getitem__(self, idx):
        import torch
        return self.t[torch.as_tensor(np.asarray(idx), device=self.t.device)].double().cpu().numpy()


def cpu_baseline(cfg, tw, dw, ctx, table, dtable, e, args):
    """The oracle's SD step (as it stands in oracle/) for EIGHT sequences of the batch (every fourth
    one in order of context length, so the sample keeps the batch's length mix), one after another,
    with 6 of the target's decoder layers, timed on the host cores; the layer part is scaled to the
    full depth.  Weight widening to float64 happens before the clock starts.  Sized to about 10-30 s
    of CPU work."""
    import dataclasses

    from oracle import decoder as dec
    from oracle import sd

    L_sample = min(6, cfg.n_layers)
    order = np.argsort(ctx)
    picks = [int(order[i]) for i in range(len(order) // 16, len(order), max(len(order) // 8, 1))][:8]
    to64 = dec.weights_to_f64
    tw64 = {"embed": _EmbedRows(tw["embed"]), "lm_head": to64(tw["lm_head"]), "final_norm": to64(tw["final_norm"]),
            "layers": [to64(tw["layers"][l]) for l in range(L_sample)]}
    dw64 = to64(dw)
    small = dataclasses.replace(cfg, n_layers=L_sample)
    rng = np.random.default_rng(0)
    tokens, t_scaled, t_measured = 0, 0.0, 0.0
    for b in picks:
        c = int(ctx[b])
        st = sd.SeqState(small, c + args.verify + args.depth * args.topk + 16, dec.round_to_bf16)
        for l in range(L_sample):
            st.target[l].k[:c] = _gather_rows(e.kv.k_pool[l], table[b], c, cfg.page_size)
            st.target[l].v[:c] = _gather_rows(e.kv.v_pool[l], table[b], c, cfg.page_size)
        st.draft.k[:c] = _gather_rows(e.dkv.k_pool[0], dtable[b], c, cfg.page_size)
        st.draft.v[:c] = _gather_rows(e.dkv.v_pool[0], dtable[b], c, cfg.page_size)
        st.ctx = c
        st.draft_len = c
        t0 = time.perf_counter()
        sd.draft_extend(small, tw64, dw64, st, [int(rng.integers(cfg.vocab))], rng.normal(size=(1, cfg.hidden)))
        tree, _ = sd.draft_expand(small, tw64, dw64, st, 1, args.topk, args.depth, args.verify)
        t_draft = time.perf_counter() - t0
        t0 = time.perf_counter()
        logits, hidden = sd.verify(small, tw64, st, tree)
        t_verify = time.perf_counter() - t0
        t0 = time.perf_counter()
        dec.lm_logits(small, tw64, hidden)
        t_head = time.perf_counter() - t0
        t0 = time.perf_counter()
        a, path, out = sd.accept_greedy(tree, logits)
        sd.commit(st, path)
        t_tail = time.perf_counter() - t0
        t_layers = max(t_verify - t_head, 0.0)
        t_scaled += t_draft + t_layers * cfg.n_layers / L_sample + t_head + t_tail
        t_measured += t_draft + t_verify + t_head + t_tail
        tokens += a + 1
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    return {"value": round(tokens / t_scaled, 4), "unit": "accepted tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{len(picks)} of the batch's {len(ctx)} sequences (contexts {sorted(int(ctx[b]) for b in picks)}), one "
                      f"after another: drafter extend + expand, {L_sample} of {cfg.n_layers} target layers + LM head, "
                      f"accept, commit; layer time scaled by {cfg.n_layers}/{L_sample}",
            "seconds_measured": round(t_measured, 2)}


def recorded_traffic(key):
    """HBM-side bytes per launch from the committed counter summary (two rocprofv3 --pmc runs of this
    same command, scaled by a plain copy of known size); None when there is no such record."""
    import re
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic_and_mfma_sd_step_7b_b32_n48.md")
    try:
        m = re.search(r"traffic_bytes_per_launch %s = (\d+)" % re.escape(key), open(path).read())
        return float(m.group(1)) if m else None
    except OSError:
        return None


def strategy_grid(args):
    """The strategy sweep on the 7B shape (context fixed at 8192, greedy): for every batch size and
    tree size the SD step with the trained-drafter stand-in of fixed_acceptance_steps (Draft_Depth =
    min(8, N - 1), topK 8), and plain decoding for N = 1.  One JSON line with latency and accepted
    tokens/s per cell: the grid the strategy selector's arms live on, and where speculative decoding
    stops paying as the batch grows."""
    import copy

    import torch
    shared, cells = None, []
    for B in args.grid_batches:
        a = copy.copy(args)
        a.batch, a.verify, a.depth, a.topk = B, 64, 8, 8
        a.ctx_lo, a.ctx_cap, a.steps, a.warmup, a.sweep = 8192, 8192, (max(2, -(-24 // B)) + 1) * len(args.grid_nodes), 2, True
        cfg, e, ctx, tw, dw, table, dtable, _ = build_workload(a, shared)
        shared = (tw, dw)
        for N in args.grid_nodes:
            if N == 1:
                t = e.tree(1)
                t.token.copy_(torch.randint(0, cfg.vocab, (B, 1), device="cuda", dtype=torch.int32))
                t.parent.fill_(-1)
                e.ctx.tree_finalize(B, t)
                am = e._buf("am", 1)
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                ms = 0.0
                for it in range(4):
                    ev[0].record()
                    e.ctx.verify_forward(B, t, e.kv, out_logits=None, out_argmax=am, out_hidden=None)
                    e.ctx.accept(B, 0, 1.0, t, None, am, None, None, None, e.stride, e.accept_len, e.path_idx,
                                 e.out_tokens, e.n_out)
                    e.ctx.kv_commit(B, e.kv, e.accept_len, e.path_idx, e.stride)
                    ev[1].record()
                    torch.cuda.synchronize()
                    e.kv.seq_len_bound += 1
                    ms += ev[0].elapsed_time(ev[1]) if it > 0 else 0.0
                cell = {"batch": B, "nodes": 1, "ms_per_step": round(ms / 3, 3), "accepted_per_step": float(B),
                        "value": round(B / (ms / 3 * 1e-3), 1)}
                # the drafter was not run: start its bookkeeping afresh for the cells that follow
                g = torch.Generator(device="cuda").manual_seed(5)
                e.set_pending(torch.randint(0, cfg.vocab, (B, 1), generator=g, device="cuda", dtype=torch.int32),
                              torch.zeros((B, 1), dtype=torch.int32, device="cuda"),
                              torch.ones((B,), dtype=torch.int32, device="cuda"),
                              torch.randn((B, 1, cfg.hidden), generator=g, device="cuda", dtype=torch.float32), 1)
            else:
                # (enough sequence-steps per cell for a mean: 24 or more, each cell with draws of its own)
                r = fixed_acceptance_steps(cfg, e, 8, min(8, N - 1), N, args.alpha, steps=max(2, -(-24 // B)),
                                           seed=17 + 1000 * N + B)
                cell = {"batch": B, "nodes": N, "ms_per_step": r["ms_per_step"], "accepted_per_step": r["accepted_per_step"],
                        "expected_per_step": round(B * (1 + r["expected_accept_length"]), 2), "value": r["value"]}
            cells.append(cell)
            print(json.dumps(cell), file=sys.stderr, flush=True)
        del e
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "strategy grid: accepted tokens/s per (batch, tree nodes)", "unit": "accepted tokens/s",
                      "alpha": args.alpha, "context": 8192, "cells": cells}))


def kv_commit_stress(args):
    """tlt_kv_commit where it is not launch-bound: 128 sequences each keeping a 16-token path whose
    nodes sit at every other provisional slot (so every kept row really moves), on the 7B cache layout
    (28 layers x 4 kv heads x 256-byte rows).  One JSON line with the achieved HBM rate (bytes read
    plus bytes written over the time of the call, the length update included)."""
    import copy

    import torch
    a = copy.copy(args)
    a.batch, a.ctx_lo, a.ctx_cap, a.steps, a.warmup, a.sweep = 128, 1024, 1024, (60 if args.kv_rows <= 16 else 140), 2, False
    cfg, e, ctx, tw, dw, table, dtable, _ = build_workload(a)
    B, stride, calls = a.batch, args.kv_rows + 1, 20
    al = torch.full((B,), stride - 1, dtype=torch.int32, device="cuda")
    path = (torch.arange(stride, dtype=torch.int32, device="cuda") * 2).expand(B, stride).contiguous()
    for _ in range(3):
        e.ctx.kv_commit(B, e.kv, al, path, stride)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record()
    for _ in range(calls):
        e.ctx.kv_commit(B, e.kv, al, path, stride)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / calls
    moved = B * (stride - 1) * cfg.kv_bytes_per_token(2) * 2
    print(json.dumps({"metric": "tlt_kv_commit on a stress shape", "value": round(moved / ms / 1e6, 1), "unit": "GB/s",
                      "peak": PEAK_HBM_GBS, "frac": round(moved / ms / 1e6 / PEAK_HBM_GBS, 4), "us_per_call": round(ms * 1e3, 2),
                      "bytes_moved_per_call": moved,
                      "config": {"workload": f"{cfg.name} cache layout, batch {B}, {stride - 1} rows moved per sequence, "
                                             "layer and kv head (256-byte rows, sources at every other slot)"}}))


class StandIn:
    """One SD step at a time for the first Bk slots of an engine, with the stand-in for a trained drafter
    (see fixed_acceptance_steps): the real drafter's expansion is run and timed, the verified tree is the
    static template labelled so that a node's first child carries the target's greedy token with
    probability alpha; plain decoding (one node) for comparison.  Times are HIP-event times of the timed
    calls only."""

    def __init__(self, cfg, e, alpha, seed=17):
        import torch
        self.cfg, self.e, self.alpha = cfg, e, alpha
        self.gen = torch.Generator(device="cuda").manual_seed(seed)
        self.ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        self.templates = {}

    def _template(self, K, D, N):
        import torch

        from paper_2511_16665_amd import binding as tlt
        key = (K, D, N)
        if key not in self.templates:
            par, rank, dep = tlt.template_build(K, D, N)
            n = len(par)
            ts = tlt.Tree.empty(self.e.B, n)
            ts.parent.copy_(torch.from_numpy(par).cuda().expand(self.e.B, n))
            self.e.ctx.tree_finalize(self.e.B, ts)
            self.templates[key] = (ts, torch.from_numpy(dep.astype(np.int64)).cuda().expand(self.e.B, n),
                                   torch.from_numpy(rank == 0).cuda().expand(self.e.B, n), int(dep.max()))
        return self.templates[key]

    def reset_drafter(self, Bk):
        """Fresh drafter bookkeeping for the first Bk slots (after steps that did not run the drafter)."""
        import torch
        e, cfg = self.e, self.cfg
        e.set_pending(torch.randint(0, cfg.vocab, (e.B, 1), generator=self.gen, device="cuda", dtype=torch.int32),
                      torch.zeros((e.B, 1), dtype=torch.int32, device="cuda"), torch.ones((e.B,), dtype=torch.int32, device="cuda"),
                      torch.randn((e.B, 1, cfg.hidden), generator=self.gen, device="cuda", dtype=torch.float32), 1)

    def plain_step(self, Bk):
        """Plain decoding of the first Bk sequences: one node per sequence.  Returns (ms, accept_lens)."""
        import torch
        e = self.e
        t = e.tree(1)
        t.token.copy_(torch.randint(0, self.cfg.vocab, (e.B, 1), generator=self.gen, device="cuda", dtype=torch.int32))
        t.parent.fill_(-1)
        e.ctx.tree_finalize(e.B, t)
        am = e._buf("am", 1)
        self.ev[0].record()
        e.ctx.verify_forward(Bk, t, e.kv, out_logits=None, out_argmax=am, out_hidden=None)
        e.ctx.accept(Bk, 0, 1.0, t, None, am, None, None, None, e.stride, e.accept_len, e.path_idx, e.out_tokens, e.n_out)
        e.ctx.kv_commit(Bk, e.kv, e.accept_len, e.path_idx, e.stride)
        self.ev[1].record()
        torch.cuda.synchronize()
        e.kv.seq_len_bound += 1
        e.have_pending = False
        return self.ev[0].elapsed_time(self.ev[1]), [0] * Bk

    def sd_step(self, Bk, K, D, N):
        """One SD step of strategy (Draft_Depth D, topK K, Tokens_to_Verify N) for the first Bk sequences.
        Returns (ms of draft_expand + verify_forward + accept + kv_commit, accept_lens)."""
        import torch
        e, cfg = self.e, self.cfg
        if not e.have_pending:
            self.reset_drafter(Bk)
        pool = K + (D - 1) * K * K if D >= 1 else 0
        t = e.tree(min(N, 1 + pool))                       # the drafter's own tree (discarded)
        ts, depth, first_child, levels = self._template(K, D, N)
        n = ts.n
        hid, am = e._buf("hid", n), e._buf("am", n)
        parent = ts.parent.long()
        self.ev[0].record()
        e.ctx.draft_expand(Bk, D, K, N, e.out_tokens, e.path_idx, e.n_out, e.pending_hidden, None, e.dkv, t)
        self.ev[1].record()
        e.dkv.seq_len_bound += e.pending_max_new
        hit = first_child & (torch.rand((e.B, n), generator=self.gen, device="cuda") < self.alpha)
        rnd = torch.randint(0, cfg.vocab, (e.B, n), generator=self.gen, device="cuda", dtype=torch.int32)
        ts.token.copy_(rnd)
        ts.token[:, 0] = t.token[:, 0]
        for d in range(levels):
            e.ctx.verify_forward(Bk, ts, e.kv, out_logits=None, out_argmax=am, out_hidden=None)
            level = depth == d + 1
            from_parent = torch.gather(am, 1, parent.clamp(min=0)).to(torch.int32)
            other = torch.where(rnd == from_parent, (rnd + 1) % cfg.vocab, rnd)
            ts.token.copy_(torch.where(level, torch.where(hit, from_parent, other), ts.token))
        self.ev[2].record()
        e.ctx.verify_forward(Bk, ts, e.kv, out_logits=None, out_argmax=am, out_hidden=hid)
        e.ctx.accept(Bk, 0, 1.0, ts, None, am, None, None, None, e.stride, e.accept_len, e.path_idx, e.out_tokens, e.n_out)
        e.ctx.kv_commit(Bk, e.kv, e.accept_len, e.path_idx, e.stride)
        self.ev[3].record()
        torch.cuda.synchronize()
        e.pending_hidden, e.have_pending = hid, True
        al = e.accept_len[:Bk].cpu().numpy()
        inc = int(al.max()) + 1
        e.kv.seq_len_bound += inc
        e.pending_max_new = inc
        return self.ev[0].elapsed_time(self.ev[1]) + self.ev[2].elapsed_time(self.ev[3]), [int(a) for a in al]


def adaptive_rollout(args, model="7b", phases=(128, 64, 32, 16, 8, 4, 2, 1), steps_sd=24, steps_off=4, context=8192,
                     strategies=None, thresholds=(1, 2, 3, 8), epsilon=0.1, window=8, sd_threshold=32, seed=3, trace=None):
    """The adaptive engine's loop on measured steps (Algorithm 1 with the elastic rule of Section 5.1): the
    running batch of one rollout shrinks phase by phase; every step the selector (tlt_mab_select) picks
    a strategy for the current batch size or keeps speculation off (batch >= sd_threshold), the step is
    run and timed, and its elapsed time and accept lengths are fed back (tlt_mab_record).  Per phase the
    selector's throughput is compared with every fixed strategy and with plain decoding, each measured
    in the same run on the same state.  `trace` (a list) receives one record per selector step:
    (batch, u1, u2, choice, elapsed seconds, accept_lens)."""
    import copy

    import torch

    from paper_2511_16665_amd import binding as tlt
    if strategies is None:      # (Draft_Depth, topK, Tokens_to_Verify): two shapes per tree size
        strategies = [(8, 8, 64), (4, 4, 64), (8, 8, 32), (4, 4, 32), (8, 8, 16), (4, 4, 16), (7, 8, 8), (3, 2, 8)]
    a = copy.copy(args)
    a.model, a.batch, a.verify, a.depth, a.topk = model, max(phases), 64, 8, 8
    n_steps = sum(steps_off if B >= sd_threshold else steps_sd + (max(3, -(-16 // B) + 1)) * len(strategies) + 3 for B in phases)
    a.ctx_lo, a.ctx_cap, a.steps, a.warmup, a.sweep = context, context, n_steps, 2, True
    cfg, e, ctx, tw, dw, table, dtable, _ = build_workload(a)
    run = StandIn(cfg, e, args.alpha)
    mab = tlt.Mab(strategies, list(thresholds), epsilon, window, sd_threshold)
    rng = np.random.default_rng(seed)
    out = []
    for B in phases:
        rec = {"batch": B}
        if B >= sd_threshold:
            ms = [run.plain_step(B)[0] for _ in range(steps_off)]
            for _ in range(steps_off):
                u1, u2 = int(rng.integers(2 ** 32)), int(rng.integers(2 ** 32))
                assert mab.select(B, u1, u2) is None
                if trace is not None:
                    trace.append((B, u1, u2, None, 0.0, []))
            rec.update({"speculation": "off", "ms_per_step": round(float(np.mean(ms[1:])), 3),
                        "value": round(B / (np.mean(ms[1:]) * 1e-3), 1)})
            out.append(rec)
            print(json.dumps(rec), file=sys.stderr, flush=True)
            continue
        # baselines on the same state: plain decoding, then every fixed strategy
        ms = [run.plain_step(B)[0] for _ in range(3)]
        rec["no_sd"] = round(B / (np.mean(ms[1:]) * 1e-3), 1)
        fixed = {}
        n_base = max(3, -(-16 // B) + 1)            # (few sequences: more steps for a mean accept length)
        for (D, K, N) in strategies:
            r = [run.sd_step(B, K, D, N) for _ in range(n_base)]
            fixed[f"D{D}K{K}N{N}"] = round(sum(sum(al) + B for _, al in r[1:]) / (sum(m for m, _ in r[1:]) * 1e-3), 1)
        rec["fixed"] = fixed
        rec["best_fixed"] = max(fixed, key=fixed.get)
        # the selector
        emitted, total_ms, chosen = 0, 0.0, {}
        for _ in range(steps_sd):
            u1, u2 = int(rng.integers(2 ** 32)), int(rng.integers(2 ** 32))
            si = mab.select(B, u1, u2)
            D, K, N = strategies[si]
            ms_step, al = run.sd_step(B, K, D, N)
            mab.record(si, ms_step * 1e-3, al, B)
            if trace is not None:
                trace.append((B, u1, u2, si, ms_step * 1e-3, al))
            emitted += sum(al) + B
            total_ms += ms_step
            chosen[f"D{D}K{K}N{N}"] = chosen.get(f"D{D}K{K}N{N}", 0) + 1
        rec.update({"speculation": "on", "adaptive": round(emitted / (total_ms * 1e-3), 1), "chosen": chosen,
                    "adaptive_vs_best_fixed": round(emitted / (total_ms * 1e-3) / fixed[rec["best_fixed"]], 3),
                    "adaptive_vs_no_sd": round(emitted / (total_ms * 1e-3) / rec["no_sd"], 3)})
        out.append(rec)
        print(json.dumps(rec), file=sys.stderr, flush=True)
    mab.close()
    e.ctx.close()
    return {"metric": "adaptive rollout: accepted tokens/s per phase (selector vs fixed strategies vs plain decoding)",
            "unit": "accepted tokens/s", "alpha": args.alpha, "context": context, "epsilon": epsilon, "window": window,
            "sd_threshold": sd_threshold, "thresholds": list(thresholds), "strategies": [list(s) for s in strategies],
            "steps_per_sd_phase": steps_sd, "phases": out,
            "note": "drafter stand-in with fixed first-child acceptance (see fixed_acceptance_steps); the drafter's re-activation "
                    "when speculation switches on (Engine.activate_drafter) is not part of the timed steps"}


def graph_pool_report(args):
    """The HIP-graph pool (Section 5.1, "Memory-Efficient CUDAGraph Capture") against naive capture on the 7B
    shape at context 8192: the naive scheme captures one graph of the whole step per (batch size, strategy);
    the pool captures per batch-size BUCKET, the drafter's and the target's halves separately, and strategies
    with equal keys share a graph.  Reported: graphs captured, device memory they take (free-memory
    difference around the captures), capture time, and the step's latency eager against replayed at small
    batches (host time from launch to completion, where launch overhead would show)."""
    import copy

    import torch
    batches = list(range(1, args.graph_max_batch + 1))
    strategies = [(8, 8, 64), (4, 4, 64), (8, 8, 32), (4, 4, 16), (7, 8, 8), (3, 2, 8)]   # (Draft_Depth, topK, Tokens_to_Verify)
    a = copy.copy(args)
    a.batch, a.verify, a.depth, a.topk = max(batches), 64, 8, 8
    a.ctx_lo, a.ctx_cap, a.steps, a.warmup, a.sweep = 8192, 8192, 400, 2, True
    cfg, e, ctx, tw, dw, table, dtable, _ = build_workload(a)
    e.step(8, 8, 64)                                     # creates the pending state graphs start from
    for (D, K, N) in strategies:                         # every buffer a step touches exists before memory is compared
        n = min(N, 1 + K + (D - 1) * K * K)
        e.tree(n), e._buf("hid", n), e._buf("am", n)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()

    def free():
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        return torch.cuda.mem_get_info()[0]

    # --- the pool (the library's own: tlt_graph_pool_*)
    pool = e.graph_pool(native=True)
    torch_capture = e.graph_pool()                       # only its capture routine is used, for the naive scheme below
    f0, t0 = free(), time.perf_counter()
    for B in batches:
        for (D, K, N) in strategies:
            pool.step(B, K, D, N)
    torch.cuda.synchronize()
    pool_s, pool_bytes = time.perf_counter() - t0, f0 - free()
    n_draft, n_target = pool.n_graphs()
    # --- naive: one whole-step graph per (batch size, strategy)
    naive = {}
    f0, t0 = free(), time.perf_counter()
    for B in batches:
        for (D, K, N) in strategies:
            n = min(N, 1 + K + (D - 1) * K * K)
            t, hid, am = e.tree(n), e._buf("hid", n), e._buf("am", n)
            hid_prev = e.pending_hidden

            def whole(B=B, D=D, K=K, N=N, t=t, hid=hid, am=am, hid_prev=hid_prev):
                e.ctx.draft_expand(B, D, K, N, e.out_tokens, e.path_idx, e.n_out, hid_prev, None, e.dkv, t)
                e.ctx.verify_forward(B, t, e.kv, out_logits=None, out_argmax=am, out_hidden=hid)
                e.ctx.accept(B, 0, 1.0, t, None, am, None, None, None, e.stride, e.accept_len, e.path_idx, e.out_tokens, e.n_out)
                e.ctx.kv_commit(B, e.kv, e.accept_len, e.path_idx, e.stride)
            naive[(B, D, K, N)] = torch_capture._capture(whole, also_keep=(hid_prev,))
    naive_s, naive_bytes = time.perf_counter() - t0, f0 - free()
    # --- latency at small batches: eager launches against one replay of the two pool graphs
    lat = {}
    for B in [b for b in (1, 2, 4) if b <= max(batches)]:
        D, K, N = 7, 8, 8
        for mode in ("eager", "replayed"):
            ts = []
            for it in range(6):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                if mode == "eager":
                    n = min(N, 1 + K + (D - 1) * K * K)
                    t, hid, am = e.tree(n), e._buf("hid", n), e._buf("am", n)
                    e.ctx.draft_expand(B, D, K, N, e.out_tokens, e.path_idx, e.n_out, e.pending_hidden, None, e.dkv, t)
                    e.dkv.seq_len_bound += e.pending_max_new
                    e.ctx.verify_forward(B, t, e.kv, out_logits=None, out_argmax=am, out_hidden=hid)
                    e.ctx.accept(B, 0, 1.0, t, None, am, None, None, None, e.stride, e.accept_len, e.path_idx, e.out_tokens, e.n_out)
                    e.ctx.kv_commit(B, e.kv, e.accept_len, e.path_idx, e.stride)
                    e.pending_hidden = hid
                    e.kv.seq_len_bound += min(D, n - 1) + 1
                    e.pending_max_new = min(D, n - 1) + 1
                else:
                    pool.step(B, K, D, N)
                torch.cuda.synchronize()
                ts.append((time.perf_counter() - t0) * 1e3)
            lat[f"batch {B} {mode}"] = round(float(np.median(ts[1:])), 3)
    print(json.dumps({"metric": "HIP-graph pool against naive per-(batch, strategy) capture", "unit": "MiB of device memory",
                      "batch_sizes": [batches[0], batches[-1]], "strategies": [list(x) for x in strategies],
                      "pool": {"implementation": "tlt_graph_pool (C ABI)", "graphs": n_draft + n_target, "drafter_graphs": n_draft, "target_graphs": n_target,
                               "MiB": round(pool_bytes / 2 ** 20, 1), "capture_s": round(pool_s, 2), "buckets": list(pool.buckets)},
                      "naive": {"graphs": len(naive), "MiB": round(naive_bytes / 2 ** 20, 1), "capture_s": round(naive_s, 2)},
                      "step_latency_ms_D7_K8_N8": lat,
                      "config": {"workload": f"{cfg.name}, context 8192, every batch size 1..{batches[-1]} x {len(strategies)} strategies"}}))


def attention_only(args):
    """The tree-attention kernel on its own (tlt_attention) at a workload's shape: batch, contexts, page
    tables and tree size as in the step, queries and cache N(0,1), chain-free random trees.  Two layers'
    pools are used in turn so that no launch finds its keys and values in a cache from the launch before.
    One JSON line: time per launch (HIP events on the launch stream), achieved HBM rate on the algorithmic
    bytes (one pass over every sequence's cached keys and values) and the matrix rate of the same launches
    (4 * d * Hq * n flops per cached token)."""
    import torch

    from paper_2511_16665_amd import binding as tlt
    from synth import QWEN7B, QWEN32B, MID, fill_kv_pool, lognormal_contexts, random_block_table
    cfg = {"7b": QWEN7B, "32b": QWEN32B, "mid": MID}[args.model]
    B, n = args.batch, args.verify
    if args.ctx_lo:
        ctx = np.random.default_rng(0).integers(args.ctx_lo, args.ctx_cap + 1, size=B).astype(np.int32)
    else:
        ctx = lognormal_contexts(B, args.ctx_median, 0.8, args.ctx_cap, min(256, args.ctx_median), seed=0)
    table, n_pages = random_block_table(ctx + n + 64, cfg.page_size, seed=1, extra_pages=8)
    pools = [fill_kv_pool(1, n_pages, cfg.n_kv_heads, cfg.page_size, cfg.head_dim, 3 + l, "cuda", torch.bfloat16) for l in range(2)]
    g = torch.Generator(device="cuda").manual_seed(5)
    qkv = torch.randn((B, n, cfg.qkv_dim), generator=g, device="cuda").bfloat16()
    rng = np.random.default_rng(1)
    parent = np.full((B, n), -1, dtype=np.int64)
    mask = np.zeros((B, n), dtype=np.uint64)
    for b in range(B):
        for i in range(n):
            if i > 0:
                parent[b, i] = rng.integers(max(0, i - 6), i)
            mask[b, i] = (mask[b, parent[b, i]] if i > 0 else np.uint64(0)) | np.uint64(1 << i)
    anc = torch.from_numpy(mask.view(np.int64)).cuda()
    tbl = torch.from_numpy(table.astype(np.int32)).cuda()
    sl = torch.from_numpy(ctx.astype(np.int32)).cuda()
    kvs = [tlt.KV(k[0], v[0], tbl, sl, int(ctx.max())) for k, v in pools]
    out = torch.zeros((B, n, cfg.q_dim), dtype=torch.bfloat16, device="cuda")
    ws = tlt.attention_workspace(B, n, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, int(ctx.max()) + n + 64)

    def launch(i):
        rc = tlt.attention(tlt.TLT_BF16, cfg.n_q_heads, cfg.page_size, qkv, anc, kvs[i & 1], out, ws, args.attn_impl)
        assert rc == 0, tlt.ERRORS.get(rc, rc)

    for i in range(args.warmup + 1):
        launch(i)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record()
    for i in range(args.steps):
        launch(i)
    ev[1].record()
    torch.cuda.synchronize()
    us = ev[0].elapsed_time(ev[1]) / args.steps * 1e3
    tokens = float(ctx.sum() + B * n)
    nbytes = tokens * 2 * cfg.n_kv_heads * cfg.head_dim * 2
    flops = 4.0 * cfg.head_dim * cfg.n_q_heads * n * tokens
    print(json.dumps({"metric": "tlt_attention (plan + main + combine kernels) per launch", "value": round(us, 2), "unit": "us",
                      "higher_is_better": False,
                      "roofline": {"bound": "hbm", "achieved": round(nbytes / us / 1e3, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                   "frac": round(nbytes / us / 1e3 / PEAK_HBM_GBS, 4), "bytes_per_launch": nbytes,
                                   "mfma_tflops": round(flops / us / 1e6, 1), "mfma_frac": round(flops / us / 1e6 / PEAK_BF16_TFLOPS, 4)},
                      "config": {"workload": f"{cfg.name} attention shape ({cfg.n_q_heads} query / {cfg.n_kv_heads} kv heads, head "
                                             f"dim {cfg.head_dim}), batch {B}, {int(ctx.sum())} cached tokens, {n} tree rows per "
                                             f"sequence = {n * cfg.group} query rows per cached key"}}))


def measured_ceilings(cfg, M):
    """What this machine delivers to plain kernels, in the same run: a device-to-device copy (HBM read +
    write) and the vendor library's bf16 GEMM (torch.matmul) on the verification forward's gate/up
    and down shapes.  Context for the roofline fractions, which are quoted against the published peaks."""
    import torch

    def timed(fn, it):
        fn()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(it):
            fn()
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / it * 1e-3

    out = {}
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()   # 1 GiB
    dst = torch.empty_like(src)
    out["hbm_copy_GBs"] = round(2 * src.numel() * 4 / timed(lambda: dst.copy_(src), 5) / 1e9, 1)
    del src, dst
    try:
        a = torch.randn((M, cfg.hidden), device="cuda").bfloat16()
        af = torch.randn((M, cfg.mlp), device="cuda").bfloat16()
        ws = [(torch.randn((2 * cfg.mlp, cfg.hidden), device="cuda") * 0.02).bfloat16() for _ in range(3)]
        wd = [(torch.randn((cfg.hidden, cfg.mlp), device="cuda") * 0.02).bfloat16() for _ in range(3)]
        i = [0]

        def gate_up():
            i[0] = (i[0] + 1) % 3
            return a @ ws[i[0]].T

        def down():
            i[0] = (i[0] + 1) % 3
            return af @ wd[i[0]].T

        out["vendor_gemm_TFLOPs"] = {
            "gate_up": round(4.0 * M * cfg.mlp * cfg.hidden / timed(gate_up, 6) / 1e12, 1),
            "down": round(2.0 * M * cfg.mlp * cfg.hidden / timed(down, 6) / 1e12, 1)}
        # this library's fused gate/up kernel on the same shape, once with these random operands and once
        # with constant ones: the matrix pipes then toggle few bits and the chip keeps a higher clock under
        # its power limit, which separates what the kernel's schedule sustains from what the power limit
        # leaves of it on random data
        from paper_2511_16665_amd import binding as tlt
        act = torch.empty((M, cfg.mlp), dtype=torch.bfloat16, device="cuda")
        halves = [(w[: cfg.mlp], w[cfg.mlp:]) for w in ws]

        def own():
            i[0] = (i[0] + 1) % 3
            tlt.gemm_glu(a, halves[i[0]][0], halves[i[0]][1], act)

        own_random = 4.0 * M * cfg.mlp * cfg.hidden / timed(own, 30) / 1e12
        a.fill_(1.0)
        for w in ws:
            w.fill_(1.0)
        out["own_gate_up_TFLOPs"] = {"random_operands": round(own_random, 1),
                                     "constant_operands": round(4.0 * M * cfg.mlp * cfg.hidden / timed(own, 30) / 1e12, 1)}
        # the matrix pipes alone: every wave of the chip looping over a wave tile's MFMAs on random register
        # operands, no memory traffic at all.  Under the power limit this, not the 2.4 GHz figure, is the rate a
        # GEMM kernel on such data can approach.
        frags = torch.randn(16384, device="cuda").bfloat16()
        sums = torch.empty(65536, dtype=torch.float32, device="cuda")
        iters = 20000
        t = timed(lambda: tlt.mfma_stream(frags, sums, iters), 3)
        out["mfma_only_TFLOPs"] = round(1024.0 * iters * 64 * 32768 / t / 1e12, 1)
    except Exception as ex:   # the library GEMM is context only
        out["vendor_gemm_TFLOPs"] = None
        out["vendor_gemm_error"] = str(ex)[:120]
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--model", default="7b", choices=["7b", "32b", "mid"])
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--depth", type=int, default=6)
    ap.add_argument("--topk", type=int, default=8)
    ap.add_argument("--verify", type=int, default=48)
    ap.add_argument("--ctx-median", type=int, default=4096)
    ap.add_argument("--ctx-cap", type=int, default=16384)
    ap.add_argument("--ctx-lo", type=int, default=0,
                    help="contexts uniform in [ctx-lo, ctx-cap] instead of lognormal (the long-tail phase's few long sequences)")
    ap.add_argument("--mode", default="greedy", choices=["greedy", "sampled", "target-only"],
                    help="greedy (the headline workload); sampled = static-template drafting + rejection-sampling "
                         "acceptance; target-only = the drafter's top-k tree + target-only sampling acceptance")
    ap.add_argument("--temperature", type=float, default=0.9)
    ap.add_argument("--drafter", default="random-init", choices=["random-init", "noisy-target"],
                    help="sampled mode: noisy-target = draft distributions softmax(target logits + N(0, sigma^2)), the "
                         "long-tail workload's drafter with its fixed acceptance rate (tree built untimed, the real "
                         "drafter's cost still timed)")
    ap.add_argument("--sigma", type=float, default=1.0)
    ap.add_argument("--workload", default="", choices=["", "longtail"],
                    help="longtail = configs[2]: batch 4, contexts uniform in [24576, 32768], depth 8 / top-k 10 / 64 verify "
                         "tokens, temperature 1.0, sampled with the noisy-target drafter")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", dest="sweep", action="store_false")
    ap.add_argument("--alpha", type=float, default=0.8,
                    help="greedy mode: also time a few steps with a stand-in for a trained drafter whose first "
                         "children match the target with this probability (0 = skip)")
    ap.add_argument("--pmc-copy-mib", type=int, default=0,
                    help="end with one plain device copy of this many MiB: the known-size kernel that hardware "
                         "counter readings (FETCH_SIZE / WRITE_SIZE) of a profiler run are scaled by")
    ap.add_argument("--grid", action="store_true",
                    help="instead of the benchmark line: the strategy sweep (batch x tree nodes at context 8192)")
    ap.add_argument("--kv-commit-stress", action="store_true",
                    help="instead of the benchmark line: the HBM rate of tlt_kv_commit on a shape that is not launch-bound")
    ap.add_argument("--graph-pool", action="store_true",
                    help="instead of the benchmark line: graphs, memory and small-batch latency of the HIP-graph pool against "
                         "naive per-(batch, strategy) capture")
    ap.add_argument("--graph-max-batch", type=int, default=16)
    ap.add_argument("--adaptive", action="store_true",
                    help="instead of the benchmark line: a rollout whose running batch shrinks from 128 to 1 with the strategy "
                         "selector choosing the step's strategy from measured rewards")
    ap.add_argument("--attention-only", action="store_true",
                    help="instead of the benchmark line: the tree-attention kernel alone at the workload's shape")
    ap.add_argument("--attn-impl", type=int, default=-1)
    ap.add_argument("--kv-rows", type=int, default=16, help="--kv-commit-stress: rows moved per sequence, layer and kv head (<= 64)")
    ap.add_argument("--grid-batches", type=int, nargs="+", default=[1, 4, 16, 64, 128])
    ap.add_argument("--grid-nodes", type=int, nargs="+", default=[1, 8, 16, 32, 64])
    args = ap.parse_args()
    if args.workload == "longtail":
        args.batch, args.ctx_lo, args.ctx_cap, args.depth, args.topk, args.verify = 4, 24576, 32768, 8, 10, 64
        args.mode, args.drafter, args.temperature = "sampled", "noisy-target", 1.0
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (sequences are independent and would "
                 "shard by sequence); run with --gpus 1")
    import torch
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    if args.grid:
        return strategy_grid(args)
    if args.kv_commit_stress:
        return kv_commit_stress(args)
    if args.attention_only:
        return attention_only(args)
    if args.adaptive:
        print(json.dumps(adaptive_rollout(args)))
        return
    if args.graph_pool:
        return graph_pool_report(args)
    cfg, e, ctx, tw, dw, table, dtable, setup_s = build_workload(args)
    K, D, N, B = args.topk, args.depth, args.verify, args.batch

    if args.mode != "greedy":
        from paper_2511_16665_amd import binding as tlt
        n_nodes = len(tlt.template_build(K, D, N)[0]) if args.mode == "sampled" else min(N, 1 + K + (D - 1) * K * K)
        gen = torch.Generator(device="cuda").manual_seed(11)
        u32 = lambda *shape: torch.randint(-2**31, 2**31 - 1, shape, generator=gen, device="cuda", dtype=torch.int32)

    def one_step():
        if args.mode == "greedy":
            return e.step(K, D, N)
        if args.mode == "sampled":
            return e.step_sampled(K, D, N, args.temperature, u32(B, n_nodes), u32(B, n_nodes), u32(B))
        return e.step(K, D, N, sample=(args.temperature, u32(B, n_nodes), u32(B)))

    noisy = None
    if args.mode == "sampled" and args.drafter == "noisy-target":
        # the tree is built between the timed calls (see noisy_target_steps): the step time is the sum of the
        # timed calls' HIP-event times, not the wall clock around the loop
        noisy = noisy_target_steps(cfg, e, K, D, N, args.steps, args.warmup, args.sigma, args.temperature)
        emitted, dt = int(round(noisy["accepted_per_step"] * args.steps)), noisy["ms_per_step"] * args.steps * 1e-3
        ms_per_step = noisy["ms_per_step"]
        prof_run = noisy_target_steps(cfg, e, K, D, N, args.steps, 0, args.sigma, args.temperature, seed=29, profile=True)
        ms_prof = prof_run["ms_per_step"]
        prof = e.ctx.profile_read()
    else:
        for _ in range(args.warmup):
            one_step()
        torch.cuda.synchronize()
        emitted = 0
        t0 = time.perf_counter()
        for _ in range(args.steps):
            al, _ = one_step()
            emitted += int(al.sum()) + B
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ms_per_step = dt / args.steps * 1e3

        # same steps again with per-launch HIP events inside the library (roofline of each kernel class)
        e.ctx.profile_begin(True)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one_step()
        torch.cuda.synchronize()
        ms_prof = (time.perf_counter() - t0) / args.steps * 1e3
        prof = e.ctx.profile_read()
        e.ctx.profile_begin(False)
    g = prof["gemm"]
    gemm_tflops = g["flops"] / (g["ms"] * 1e-3) / 1e12 if g["ms"] > 0 else 0.0
    at = prof["attention"]
    # algorithmic bytes of the tree attention: one pass over every sequence's cached keys and values
    # (actual contexts, all layers) plus the tree rows; the library only knows the host-side bound
    attn_bytes_per_step = float(ctx.sum() + B * N) * cfg.kv_bytes_per_token(2)
    attn_gbs = attn_bytes_per_step * args.steps / (at["ms"] * 1e-3) / 1e9 if at["ms"] > 0 else 0.0
    # (actual context lengths, like the bytes: the library's own accounting only knows the host-side bound)
    attn_flops_per_step = 4.0 * cfg.head_dim * cfg.n_q_heads * N * float(ctx.sum() + B * N) * cfg.n_layers
    attn_tflops = attn_flops_per_step * args.steps / (at["ms"] * 1e-3) / 1e12 if at["ms"] > 0 else 0.0
    per_class = {k: {"ms_per_step": round(v["ms"] / args.steps, 4), "launches_per_step": v["launches"] // args.steps}
                 for k, v in prof.items()}

    default_workload = (args.model, B, D, K, N, args.ctx_median, args.ctx_cap, args.ctx_lo, args.mode) == \
        ("7b", 32, 6, 8, 48, 4096, 16384, 0, "greedy")
    ctx_desc = f"uniform in [{args.ctx_lo}, {args.ctx_cap}]" if args.ctx_lo else \
        f"lognormal(median {args.ctx_median}, sigma 0.8, cap {args.ctx_cap})"
    mode_desc = {"greedy": "greedy", "sampled": f"sampled on the static template at temperature {args.temperature} "
                 "(rejection-sampling acceptance)", "target-only": f"top-k tree, target-only sampling acceptance at "
                 f"temperature {args.temperature}"}[args.mode]
    result = {
        "metric": "accepted tokens/s per GPU in SD rollout step; verify latency vs tree size",
        "value": round(emitted / dt, 2), "unit": "accepted tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name} random-init bf16, 1-layer drafter, batch {B}, contexts {ctx_desc} = "
                               f"{int(ctx.sum())} cached tokens, 16-token pages, tree depth {D} top-k {K} verify {N}, "
                               f"{mode_desc}",
                   "accepted_per_step": round(emitted / args.steps, 2),
                   "drafter": "random-init (accept length ~0)" if noisy is None else
                   f"draft distributions softmax(target logits + N(0, {args.sigma}^2)), tree built between the timed calls; "
                   "timed per step: tlt_draft_sample of the real drafter (discarded) + tlt_verify_forward + tlt_accept + tlt_kv_commit"},
        "roofline": {"bound": "mfma", "kernel": "gemm_bf16_pipe_k (GEMMs of the verification forward; one launch here = one library GEMM = one or two kernel launches)",
                     "achieved": round(gemm_tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(gemm_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": recorded_traffic("gemm_bf16_pipe_k_verify") if default_workload else None,
                     "avg_launch_us": round(g["ms"] / max(g["launches"], 1) * 1e3, 2),
                     "flops_per_launch": round(g["flops"] / max(g["launches"], 1), 0),
                     # the kernel's time per step over ALL its launches (drafter included): the figure a
                     # kernel trace of the same command sums to over the kernel's instantiations
                     "kernel_ms_per_step_all": round((g["ms"] + prof["gemm_draft"]["ms"]) / args.steps, 3)},
        "attention_roofline": {"bound": "hbm", "kernel": "attn_plan_k + attn_mfma_k + attn_combine_k (verification forward)",
                               "achieved": round(attn_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                               "frac": round(attn_gbs / PEAK_HBM_GBS, 4),
                               "bytes_per_launch": round(attn_bytes_per_step / cfg.n_layers, 0),
                               # at N*G = 336 query rows per cached key the kernel sits at the ridge: the same
                               # launches against the MFMA roof (4*d*Hq*N flops per cached token and layer)
                               "mfma_tflops": round(attn_tflops, 1),
                               "mfma_frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                               "avg_launch_us": round(at["ms"] / max(at["launches"], 1) * 1e3, 2)},
        "per_class": per_class, "ms_per_step_profiled": round(ms_prof, 3), "setup_s": round(setup_s, 1),
    }
    if noisy is not None:
        result["noisy_target"] = noisy
    if args.sweep:
        result["verify_latency_ms_vs_tree_size"] = verify_latency_sweep(cfg, e, [1, 8, 16, 32, 48, 64])
    if args.sweep:
        result["measured_ceilings"] = measured_ceilings(cfg, B * N)
        # beside the fraction of the published peak: the fraction of what the matrix pipes alone sustain on
        # random operands under this box's power limit, measured in this run
        sustained = result["measured_ceilings"].get("mfma_only_TFLOPs")
        if sustained and result["roofline"].get("unit") == "TFLOP/s":
            result["roofline"]["frac_of_measured_mfma_only"] = round(result["roofline"]["achieved"] / sustained, 4)
    if args.alpha > 0 and args.mode == "greedy" and args.sweep:
        result["fixed_acceptance"] = fixed_acceptance_steps(cfg, e, K, D, N, args.alpha, steps=5)
    if not args.no_cpu_baseline and args.mode == "greedy":
        result["cpu_baseline"] = cpu_baseline(cfg, tw, dw, ctx, table, dtable, e, args)
    if args.pmc_copy_mib > 0:
        src = torch.ones(args.pmc_copy_mib << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
