"""Host-side driver of the speculative-decoding step: owns the device buffers (torch tensors) and
issues the four library calls per step.  No arithmetic of the method happens here.

    draft_expand -> verify_forward -> accept -> kv_commit          (one SD step)

The only host synchronisation per step is the read-back of accept_len / emitted tokens, which is
also what the rollout loop's feedback needs (accept length and step latency, Section 3
"Architecture & Workflow", and Algorithm 1's Record procedure).
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as tlt


def alloc_kv(cfg, dtype_code, n_layers, block_table: np.ndarray, n_pages: int, seq_len: np.ndarray, fill=None) -> tlt.KV:
    dt = tlt.torch_dtype(dtype_code)
    shape = (n_layers, n_pages, cfg.n_kv_heads, cfg.page_size, cfg.head_dim)
    if fill is None:
        k = torch.zeros(shape, dtype=dt, device="cuda")
        v = torch.zeros(shape, dtype=dt, device="cuda")
    else:
        k, v = fill
    return tlt.KV(k, v, torch.from_numpy(np.ascontiguousarray(block_table, dtype=np.int32)).cuda(),
                  torch.from_numpy(np.ascontiguousarray(seq_len, dtype=np.int32)).cuda(), int(np.max(seq_len)))


class Engine:
    def __init__(self, cfg, dtype_code, target_w, draft_w, batch, max_n, max_depth, max_topk, max_ctx, kv: tlt.KV,
                 draft_kv: tlt.KV):
        self.cfg, self.B = cfg, batch
        self.ctx = tlt.Context(cfg, dtype_code, target_w, draft_w, batch, max_n, max_depth, max_topk, max_ctx)
        self.kv, self.dkv = kv, draft_kv
        self.max_n, self.max_depth = max_n, max_depth
        dev = "cuda"
        B = batch
        self.stride = min(max_depth, max_n - 1) + 1      # longest accepted path + bonus token
        i32 = lambda *s: torch.full(s, -1, dtype=torch.int32, device=dev)
        self.accept_len, self.n_out = i32(B), i32(B)
        self.path_idx, self.out_tokens = i32(B, self.stride), i32(B, self.stride)
        self.pending_hidden, self.pending_max_new = None, 0
        self.root = i32(B)
        self._trees = {}
        self.have_pending = False

    def tree(self, n) -> tlt.Tree:
        if n not in self._trees:
            self._trees[n] = tlt.Tree.empty(self.B, n)
        return self._trees[n]

    # -- prompt ingestion: chain trees through the same verify / commit / extend calls
    def prefill(self, prompts: np.ndarray, chunk=None):
        """prompts [B, P] int32, equal lengths: prompts[:, :-1] goes into both caches, the last token
        becomes the first root."""
        B, P = prompts.shape
        chunk = chunk or self.max_n
        body = P - 1
        for o in range(0, body, chunk):
            m = min(chunk, body - o)
            t = self.tree(m)
            t.token.copy_(torch.from_numpy(np.ascontiguousarray(prompts[:, o:o + m])).cuda())
            t.parent.copy_(torch.arange(-1, m - 1, dtype=torch.int32, device="cuda").expand(B, m))
            self.ctx.tree_finalize(B, t)
            hid = self._buf("hid", m)
            self.ctx.verify_forward(B, t, self.kv, out_hidden=hid)
            al = torch.full((B,), m - 1, dtype=torch.int32, device="cuda")
            path = torch.arange(m, dtype=torch.int32, device="cuda").expand(B, m).contiguous()
            self.ctx.kv_commit(B, self.kv, al, path, m)
            self.kv.seq_len_bound += m
            nxt = torch.from_numpy(np.ascontiguousarray(prompts[:, o + 1:o + 1 + m])).cuda()
            n_new = torch.full((B,), m, dtype=torch.int32, device="cuda")
            self.ctx.draft_expand(B, 0, 1, 1, nxt, path, n_new, hid, None, self.dkv, None)
            self.dkv.seq_len_bound += m
        self.root.copy_(torch.from_numpy(np.ascontiguousarray(prompts[:, -1])).cuda())
        self.have_pending = False

    def set_pending(self, new_tokens, new_src, n_new, hidden, max_new):
        """Entries the drafter still has to catch up on at the start of the next step:
        new_tokens/new_src [B, w] int32, n_new [B] int32, hidden [B, m, h] fp32 (device tensors);
        max_new = host-known upper bound of n_new.  The next root is each sequence's last new token."""
        self.out_tokens.fill_(-1)
        self.path_idx.fill_(-1)
        self.out_tokens[:, : new_tokens.shape[1]].copy_(new_tokens)
        self.path_idx[:, : new_src.shape[1]].copy_(new_src)
        self.n_out.copy_(n_new)
        self.pending_hidden = hidden.contiguous()
        self.pending_max_new = int(max_new)
        self.have_pending = True

    # -- one speculative-decoding step
    def step(self, topk, depth, n_verify, sync=True, logits_out=None, sample=None):
        """Runs the four calls.  With sync=True returns (accept_len [B], out_tokens [B, stride]) as
        numpy arrays and keeps the host-side length bounds exact; with sync=False nothing is read
        back and the bounds advance by the largest possible accept length.
        sample = (temperature, u_accept [B, n], u_final [B]) switches the acceptance from greedy to
        the target-only sampling rule (the drafter's top-k tree stays as it is)."""
        B = self.B
        pool = topk + (depth - 1) * topk * topk if depth >= 1 else 0
        n = min(n_verify, 1 + pool)
        t = self.tree(n)
        if self.have_pending:
            # root = last new token of each sequence (derived inside the library)
            self.ctx.draft_expand(B, depth, topk, n_verify, self.out_tokens, self.path_idx, self.n_out,
                                  self.pending_hidden, None, self.dkv, t)
            self.dkv.seq_len_bound += self.pending_max_new
        else:
            self.ctx.draft_expand(B, depth, topk, n_verify, None, None, None, None, self.root, self.dkv, t)
        hid, am = self._buf("hid", n), self._buf("am", n)
        if sample is None:
            self.ctx.verify_forward(B, t, self.kv, out_logits=logits_out, out_argmax=am, out_hidden=hid)
            self.ctx.accept(B, 0, 1.0, t, None, am, None, None, None, self.stride, self.accept_len, self.path_idx,
                            self.out_tokens, self.n_out)
        else:
            temperature, u_accept, u_final = sample
            logits = logits_out if logits_out is not None else self.logits(n)
            self.ctx.verify_forward(B, t, self.kv, out_logits=logits, out_argmax=None, out_hidden=hid)
            self.ctx.accept(B, 2, temperature, t, logits, None, None, u_accept, u_final, self.stride, self.accept_len,
                            self.path_idx, self.out_tokens, self.n_out)
        self.ctx.kv_commit(B, self.kv, self.accept_len, self.path_idx, self.stride)
        self.pending_hidden = hid
        self.have_pending = True
        if sync:
            al = self.accept_len.cpu().numpy()
            out = self.out_tokens.cpu().numpy()
            self.ctx.device_status()          # raises when a kernel saw a length beyond its bound or could not rendezvous
            inc = int(al.max()) + 1
        else:
            al = out = None
            inc = min(depth, n - 1) + 1
        self.kv.seq_len_bound += inc
        self.pending_max_new = inc
        return al, out

    # -- one sampled speculative-decoding step (static template, rejection-sampling acceptance)
    def step_sampled(self, topk, depth, n_verify, temperature, u_draw, u_accept, u_final):
        """u_draw, u_accept [B, n] and u_final [B]: uint32 device tensors (as int32 storage) with the
        step's random numbers, n = node count of the template.  Returns (accept_len [B], out_tokens
        [B, stride]) as numpy arrays; the tree, the draft distributions and the target logits of the
        step stay available as self.tree(n), self.draft_q(n), self.logits(n)."""
        B = self.B
        n = len(tlt.template_build(topk, depth, n_verify)[0])
        t, q, logits = self.tree(n), self.draft_q(n), self.logits(n)
        if self.have_pending:
            self.ctx.draft_sample(B, depth, topk, n_verify, temperature, self.out_tokens, self.path_idx, self.n_out,
                                  self.pending_hidden, None, self.dkv, u_draw, t, q)
            self.dkv.seq_len_bound += self.pending_max_new
        else:
            self.ctx.draft_sample(B, depth, topk, n_verify, temperature, None, None, None, None, self.root, self.dkv,
                                  u_draw, t, q)
        hid = self._buf("hid", n)
        self.ctx.verify_forward(B, t, self.kv, out_logits=logits, out_argmax=None, out_hidden=hid)
        self.ctx.accept(B, 1, temperature, t, logits, None, q, u_accept, u_final, self.stride, self.accept_len,
                        self.path_idx, self.out_tokens, self.n_out)
        self.ctx.kv_commit(B, self.kv, self.accept_len, self.path_idx, self.stride)
        self.pending_hidden = hid
        self.have_pending = True
        al = self.accept_len.cpu().numpy()
        out = self.out_tokens.cpu().numpy()
        self.ctx.device_status()
        inc = int(al.max()) + 1
        self.kv.seq_len_bound += inc
        self.pending_max_new = inc
        return al, out

    def draft_q(self, n):
        return self._big("q", n)

    def logits(self, n):
        return self._big("logits", n)

    def _big(self, kind, n):
        key = (kind, n)
        if key not in self._trees:
            self._trees[key] = torch.zeros((self.B, n, self.cfg.vocab), dtype=torch.float32, device="cuda")
        return self._trees[key]

    # -- a step whose trees come from somewhere else (the model-free drafter, tlt_ngram_propose)
    def _flush_pending(self):
        """Brings the learned drafter's cache up to the committed length (extend only, no tree)."""
        if self.have_pending:
            self.ctx.draft_expand(self.B, 0, 1, 1, self.out_tokens, self.path_idx, self.n_out, self.pending_hidden, None,
                                  self.dkv, None)
            self.dkv.seq_len_bound += self.pending_max_new
            self.have_pending = False

    def step_trees(self, token: np.ndarray, parent: np.ndarray, keep_drafter=False):
        """token/parent [B, n] int32 host arrays (node 0 = root = last emitted token, parents before
        children).  Verifies, accepts greedily and commits; returns (accept_len [B], out_tokens [B, stride]).
        With keep_drafter the learned drafter's cache follows along (one extend per step over the
        accepted positions, from the target's hidden states), so that `step` can take over at any
        time; without it the drafter's cache is left where it was."""
        B, n = token.shape
        assert B == self.B and n <= self.max_n
        if keep_drafter:
            self._flush_pending()
        t = self.tree(n)
        t.token.copy_(torch.from_numpy(np.ascontiguousarray(token, dtype=np.int32)).cuda())
        t.parent.copy_(torch.from_numpy(np.ascontiguousarray(parent, dtype=np.int32)).cuda())
        self.ctx.tree_finalize(B, t)
        am = self._buf("am", n)
        hid = self._buf("hid", n) if keep_drafter else None
        self.ctx.verify_forward(B, t, self.kv, out_logits=None, out_argmax=am, out_hidden=hid)
        self.ctx.accept(B, 0, 1.0, t, None, am, None, None, None, self.stride, self.accept_len, self.path_idx,
                        self.out_tokens, self.n_out)
        self.ctx.kv_commit(B, self.kv, self.accept_len, self.path_idx, self.stride)
        al = self.accept_len.cpu().numpy()
        out = self.out_tokens.cpu().numpy()
        inc = int(al.max()) + 1
        self.kv.seq_len_bound += inc
        if keep_drafter:
            self.pending_hidden, self.pending_max_new, self.have_pending = hid, inc, True
            self._flush_pending()
            # the next root: each sequence's bonus token
            self.root.copy_(self.out_tokens.gather(1, (self.n_out - 1).long().unsqueeze(1)).squeeze(1))
        else:
            self.have_pending = False
        return al, out

    # -- switching speculative decoding on in the middle of a rollout
    def activate_drafter(self, tokens: np.ndarray, lens: np.ndarray, chunk=None):
        """Builds the learned drafter's cache for sequences that were decoded without it (Section 5.1:
        SD is switched on once the running batch has shrunk).  tokens [B, >= max(lens)+1] int32 holds
        each sequence's committed tokens 0 .. lens[b]-1 followed by its pending root at lens[b]; lens
        must equal the target cache's lengths.  A drafter entry needs the target's hidden state of its
        position, which is not kept, so the target is run again over the context, `chunk` positions
        at a time (chain trees at a rewound length; the rows it rewrites in the target cache are the
        ones already there, recomputed), each chunk followed by the drafter's extend.  Sequences
        shorter than the longest simply run out of valid rows."""
        B = self.B
        m = chunk or self.max_n
        lens = np.ascontiguousarray(lens, dtype=np.int32)
        assert tokens.shape[0] == B and tokens.shape[1] >= int(lens.max()) + 1
        np.testing.assert_array_equal(self.kv.seq_len.cpu().numpy(), lens)
        full_bound = self.kv.seq_len_bound
        t = self.tree(m)
        t.parent.copy_(torch.arange(-1, m - 1, dtype=torch.int32, device="cuda").expand(B, m))
        hid = self._buf("hid", m)
        src = torch.arange(m, dtype=torch.int32, device="cuda").expand(B, m).contiguous()
        padded = np.zeros((B, int(lens.max()) + m + 1), dtype=np.int32)
        padded[:, : tokens.shape[1]] = tokens[:, : padded.shape[1]]
        for o in range(0, int(lens.max()), m):
            start = np.minimum(o, lens).astype(np.int32)                 # rewound length of each sequence
            n_new = np.clip(lens - o, 0, m).astype(np.int32)
            rows = np.stack([padded[b, start[b]: start[b] + m] for b in range(B)])
            nxt = np.stack([padded[b, start[b] + 1: start[b] + 1 + m] for b in range(B)])
            t.token.copy_(torch.from_numpy(rows).cuda())
            self.ctx.tree_finalize(B, t)
            self.kv.seq_len.copy_(torch.from_numpy(start).cuda())
            self.dkv.seq_len.copy_(torch.from_numpy(start).cuda())
            self.kv.seq_len_bound = self.dkv.seq_len_bound = int(start.max())
            self.ctx.verify_forward(B, t, self.kv, out_hidden=hid)
            self.ctx.draft_expand(B, 0, 1, 1, torch.from_numpy(nxt).cuda(), src, torch.from_numpy(n_new).cuda(), hid, None,
                                  self.dkv, None)
        self.kv.seq_len.copy_(torch.from_numpy(lens).cuda())
        self.dkv.seq_len.copy_(torch.from_numpy(lens).cuda())
        self.kv.seq_len_bound = full_bound
        self.dkv.seq_len_bound = int(lens.max())
        self.root.copy_(torch.from_numpy(np.array([tokens[b, lens[b]] for b in range(B)], dtype=np.int32)).cuda())
        self.have_pending = False

    # -- the same step replayed from captured HIP graphs
    def graph_pool(self, capacity_bound=None, native=False):
        """Graph pool over this engine's buffers: the library's own (tlt_graph_pool_*, native=True) or the one
        kept here with torch's capture (see GraphPool); same keys, buckets and step() either way."""
        return NativeGraphPool(self, capacity_bound) if native else GraphPool(self, capacity_bound)

    def _buf(self, kind, n):
        key = (kind, n)
        if key not in self._trees:
            if kind == "hid":
                self._trees[key] = torch.zeros((self.B, n, self.cfg.hidden), dtype=torch.float32, device="cuda")
            else:
                self._trees[key] = torch.zeros((self.B, n), dtype=torch.int32, device="cuda")
        return self._trees[key]


class GraphPool:
    """Bucketed, disaggregated, merged HIP-graph capture of the SD step (Section 5.1, "Memory-Efficient
    CUDAGraph Capture", re-thought for this library).

    * Bucketed: a graph is captured per batch-size bucket, not per batch size; a step with B running
      sequences replays the graph of the smallest bucket >= B over the first `bucket` slots of the
      engine's buffers (slots B..bucket-1 must hold valid sequences: the caller keeps finished ones
      there until it compacts).
    * Disaggregated: the drafter's graph (tlt_draft_expand) is keyed by (bucket, Draft_Depth, topK,
      Tokens_to_Verify, rows of the previous step's hidden buffer); the target's graph
      (tlt_verify_forward + tlt_accept + tlt_kv_commit) by (bucket, nodes per tree).
    * Merged: strategies that share a key share the graph.

    What makes this cheap here: every buffer a kernel touches (workspace, trees, caches, outputs) is
    owned by the caller and shared by all graphs, and sequence lengths are read on the device, so a graph
    holds kernel nodes and their arguments only: no per-graph activation memory.  The host-side length
    bounds that size the attention grids are frozen at capture time, so graphs are captured with the
    caches' capacity as the bound (`capacity_bound`, default: what the block tables can hold).

    Greedy acceptance only; the caller reads accept_len / out_tokens when it needs them (no host
    synchronisation happens inside a replay)."""

    def __init__(self, engine: Engine, capacity_bound=None, buckets=(1, 2, 4, 8, 16, 32, 64, 128)):
        self.e = engine
        self.buckets = tuple(b for b in buckets if b < engine.B) + (engine.B,)
        page = engine.cfg.page_size
        cap = min(engine.kv.block_table.shape[1], engine.dkv.block_table.shape[1]) * page
        self.bound = int(capacity_bound) if capacity_bound is not None else cap - 2 * engine.max_n - 64
        self.draft_graphs, self.target_graphs = {}, {}
        self.stream = torch.cuda.Stream()          # default priority

    def bucket(self, B):
        for b in self.buckets:
            if b >= B:
                return b
        raise ValueError(f"batch {B} exceeds the engine's {self.e.B}")

    def _capture(self, fn, also_keep=()):
        """Runs fn once eagerly (first-use set-up such as kernel attributes must not fall into a
        capture), then captures it.  The eager run's side effects on the step's state are undone."""
        e = self.e
        saved = (e.kv.seq_len_bound, e.dkv.seq_len_bound)
        e.kv.seq_len_bound = e.dkv.seq_len_bound = self.bound
        # the eager run changes state (cache lengths, pending tokens): snapshot and restore it
        state = (e.kv.seq_len, e.dkv.seq_len, e.accept_len, e.n_out, e.path_idx, e.out_tokens) + tuple(also_keep)
        keep = [t.clone() for t in state]
        torch.cuda.synchronize()
        with torch.cuda.stream(self.stream):
            fn()
        torch.cuda.synchronize()
        for dst, src in zip(state, keep):
            dst.copy_(src)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=self.stream):
            fn()
        torch.cuda.synchronize()
        e.kv.seq_len_bound, e.dkv.seq_len_bound = saved
        return g

    def step(self, B, topk, depth, n_verify):
        """One SD step for the first B slots, replayed from the pool (captured on first use).
        Requires a pending hidden buffer from a previous step (Engine.step / set_pending)."""
        e = self.e
        assert e.have_pending and e.pending_hidden is not None
        Bk = self.bucket(B)
        pool = topk + (depth - 1) * topk * topk if depth >= 1 else 0
        n = min(n_verify, 1 + pool)
        t = e.tree(n)
        hid_prev = e.pending_hidden
        hid, am = e._buf("hid", n), e._buf("am", n)
        dkey = (Bk, depth, topk, n_verify, hid_prev.data_ptr(), hid_prev.shape[1])
        tkey = (Bk, n)
        if dkey not in self.draft_graphs:
            self.draft_graphs[dkey] = self._capture(lambda: e.ctx.draft_expand(
                Bk, depth, topk, n_verify, e.out_tokens, e.path_idx, e.n_out, hid_prev, None, e.dkv, t))
        if tkey not in self.target_graphs:
            def target():
                e.ctx.verify_forward(Bk, t, e.kv, out_logits=None, out_argmax=am, out_hidden=hid)
                e.ctx.accept(Bk, 0, 1.0, t, None, am, None, None, None, e.stride, e.accept_len, e.path_idx,
                             e.out_tokens, e.n_out)
                e.ctx.kv_commit(Bk, e.kv, e.accept_len, e.path_idx, e.stride)
            self.target_graphs[tkey] = self._capture(target, also_keep=(hid_prev,))   # hid may alias hid_prev
        self.draft_graphs[dkey].replay()
        self.target_graphs[tkey].replay()
        e.pending_hidden = hid
        inc = min(depth, n - 1) + 1
        e.dkv.seq_len_bound += e.pending_max_new
        e.kv.seq_len_bound += inc
        e.pending_max_new = inc

    def n_graphs(self):
        return len(self.draft_graphs), len(self.target_graphs)


class NativeGraphPool:
    """GraphPool's interface over the library's pool (tlt_graph_pool_create / _step / _count): capture, keys and
    replay live behind the C ABI; this class only hands over the engine's buffers and keeps the host-side
    length bounds, as GraphPool.step does."""

    def __init__(self, engine: Engine, capacity_bound=None, buckets=(1, 2, 4, 8, 16, 32, 64, 128)):
        self.e = engine
        self.buckets = tuple(b for b in buckets if b < engine.B) + (engine.B,)
        page = engine.cfg.page_size
        cap = min(engine.kv.block_table.shape[1], engine.dkv.block_table.shape[1]) * page
        self.bound = int(capacity_bound) if capacity_bound is not None else cap - 2 * engine.max_n - 64
        self.pool = tlt.GraphPool(engine.ctx, self.buckets, self.bound)

    def bucket(self, B):
        for b in self.buckets:
            if b >= B:
                return b
        raise ValueError(f"batch {B} exceeds the engine's {self.e.B}")

    def step(self, B, topk, depth, n_verify):
        e = self.e
        assert e.have_pending and e.pending_hidden is not None
        pool = topk + (depth - 1) * topk * topk if depth >= 1 else 0
        n = min(n_verify, 1 + pool)
        t = e.tree(n)
        hid_prev = e.pending_hidden
        hid, am = e._buf("hid", n), e._buf("am", n)
        self.pool.step(B, depth, topk, n_verify, e.out_tokens, e.path_idx, e.n_out, hid_prev, e.dkv, t, e.kv, am, hid,
                       e.stride, e.accept_len, e.path_idx, e.out_tokens, e.n_out)
        e.pending_hidden = hid
        inc = min(depth, n - 1) + 1
        e.dkv.seq_len_bound += e.pending_max_new
        e.kv.seq_len_bound += inc
        e.pending_max_new = inc

    def n_graphs(self):
        return self.pool.count()
