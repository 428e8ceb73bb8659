"""Helpers shared by the GPU parity tests (host-side plumbing only)."""
import numpy as np
import torch

from oracle import decoder as dec
from paper_2511_16665_amd import binding as tlt
from paper_2511_16665_amd import engine as eng
from synth import make_decoder_weights, make_drafter_weights, random_block_table


def dtype_code(name):
    return tlt.TLT_F32 if name == "fp32" else tlt.TLT_BF16


def make_models(cfg, seed, dtype_name, std=0.02, qkv_bias=False):
    """Weights drawn on the CPU in the storage dtype; returns (device dicts, float64 oracle dicts)."""
    dt = torch.float32 if dtype_name == "fp32" else torch.bfloat16
    tw = make_decoder_weights(cfg, seed, device="cpu", dtype=dt, std=std, qkv_bias=qkv_bias)
    dw = make_drafter_weights(cfg, seed, device="cpu", dtype=dt, std=std)
    to_dev = lambda w: {k: ([{kk: vv.cuda() for kk, vv in l.items()} for l in v] if isinstance(v, list)
                            else ({kk: vv.cuda() for kk, vv in v.items()} if isinstance(v, dict) else v.cuda()))
                        for k, v in w.items()}
    return to_dev(tw), to_dev(dw), dec.weights_to_f64(tw), dec.weights_to_f64(dw)


def make_engine(cfg, dtype_name, tw_dev, dw_dev, B, max_n, max_depth, max_topk, capacity, seed=0, seq_len=None):
    """Engine with empty caches able to hold `capacity` tokens per sequence, pages scattered."""
    code = dtype_code(dtype_name)
    caps = np.full(B, capacity)
    table, n_pages = random_block_table(caps, cfg.page_size, seed, extra_pages=3)
    dtable, dn_pages = random_block_table(caps, cfg.page_size, seed + 1, extra_pages=2)
    sl = np.zeros(B, np.int32) if seq_len is None else seq_len
    kv = eng.alloc_kv(cfg, code, cfg.n_layers, table, n_pages, sl)
    dkv = eng.alloc_kv(cfg, code, 1, dtable, dn_pages, sl)
    e = eng.Engine(cfg, code, tw_dev, dw_dev, B, max_n, max_depth, max_topk, capacity, kv, dkv)
    return e, table, dtable


def dense_cache(pool: torch.Tensor, table: np.ndarray, b: int, length: int, page_size: int):
    """Gather sequence b's first `length` cache rows of every layer: [L, length, Hkv, d] float64."""
    slots = np.arange(length)
    pg = torch.from_numpy(table[b, slots // page_size].astype(np.int64))
    off = torch.from_numpy((slots % page_size).astype(np.int64))
    rows = pool.cpu()[:, pg, :, off, :]                     # advanced indices split by a slice: [length, L, Hkv, d]
    return rows.permute(1, 0, 2, 3).double().numpy()


def rel_err(got, want):
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    return float(np.max(np.abs(got - want)) / max(np.max(np.abs(want)), 1e-30))


class LazyLayers:
    """Widens one decoder layer at a time to float64 on the host (all layers of a 7B shape at once
    would be tens of GB); prints the layer index so a long oracle run shows progress."""

    def __init__(self, layers):
        self.layers = layers

    def __len__(self):
        return len(self.layers)

    def __iter__(self):
        for l, lw in enumerate(self.layers):
            print(f"  oracle layer {l}", flush=True)
            yield dec.weights_to_f64(lw)


class EmbedRows:
    """Embedding table kept on the device; rows are widened to float64 when the oracle indexes it."""

    def __init__(self, w):
        self.w = w

    def __getitem__(self, idx):
        return self.w[torch.as_tensor(np.asarray(idx), device=self.w.device).long()].double().cpu().numpy()


def match_tree_to_pool(pool_token, pool_parent, pool_score, tree_token, tree_parent, tree_score):
    """Pool index of every tree node (node 0, the root, maps to -1).  Kept candidates appear in the tree
    in creation order with their pool score copied bit for bit, so the match is a single ordered walk."""
    node_pool, at = [-1], 0
    for i in range(1, len(tree_token)):
        want_parent = node_pool[int(tree_parent[i])]
        while at < len(pool_token) and not (pool_token[at] == tree_token[i] and pool_parent[at] == want_parent
                                            and np.float32(pool_score[at]) == np.float32(tree_score[i])):
            at += 1
        assert at < len(pool_token), f"tree node {i} is not a candidate of the pool (in creation order)"
        node_pool.append(at)
        at += 1
    return node_pool


def check_draft_tree_against_forced_oracle(sd, cfg, tw, dw, st, root, K, D, N, g_pool, g_tree, tol):
    """Judges a drafter tree built in lower precision (Section 5.1's tree: topK options per step, the
    Tokens_to_Verify most confident candidates kept) when it may legitimately differ from the oracle's.

    The oracle's own expansion is replayed with every choice forced to the GPU's (root tokens, each
    frontier node's children, each next frontier, the kept set), so the oracle's float64 drafter
    scores exactly the GPU's candidates.  Required: (1) every GPU pool score within the path's
    tolerance of the oracle's; (2) every choice optimal within twice that tolerance: no candidate
    left out beats one taken by more; (3) the GPU's tree arrays equal the oracle's pruning of the
    forced pool exactly; (4) when every choice was also the oracle's own, the tree equals the
    oracle's unforced tree.  The tolerance of one log-probability is tol * (spread of its row): a
    logit and the row's log-sum-exp may each be off by tol * max|logit|, and for logits centred on zero
    that is half the spread each; a path's tolerance is the sum over its steps.
    g_pool = (token, parent, score) of the sequence's pool, g_tree = (token, parent, depth, score).
    Returns a dict of what was seen (for the test's print-out)."""
    p_tok, p_par, p_sc = (np.asarray(a) for a in g_pool)
    t_tok, t_par, t_dep, t_sc = (np.asarray(a) for a in g_tree)
    KK = K * K
    node_pool = match_tree_to_pool(p_tok, p_par, p_sc, t_tok, t_par, t_sc)
    seen = {"choices": 0, "own": 0, "worst_slack": -np.inf, "worst_score_err": 0.0}
    e_path = {-1: 0.0}          # pool index -> tolerance of its path score
    frontier = [-1]             # pool indices of the nodes whose children the next "children" calls rank

    def judge(where, vals, chosen, tol_of):
        vals = np.asarray(vals, dtype=np.float64)
        out = np.setdiff1d(np.arange(len(vals)), chosen)
        assert len(set(chosen)) == len(chosen) and all(0 <= c < len(vals) for c in chosen), (where, chosen)
        seen["choices"] += 1
        own = sd.topk_desc(vals, len(chosen))
        seen["own"] += int((sorted(chosen) == sorted(own)) if where[0] == "keep" else (list(chosen) == own))
        if len(out) == 0 or len(chosen) == 0:
            return
        for c in chosen:      # no left-out candidate beats a taken one by more than both tolerances
            worst = max(vals[o] - 2 * max(tol_of(o), tol_of(c)) for o in out)
            slack = (worst - vals[c]) / max(tol_of(c), 1e-30)
            seen["worst_slack"] = max(seen["worst_slack"], float(slack))
            assert vals[c] >= worst, (where, int(c), float(vals[c]), float(worst))

    def pick(where, values, k):
        values = np.asarray(values, dtype=np.float64)
        if where[0] in ("root", "children"):
            level, fr = (0, 0) if where[0] == "root" else (where[1], where[2])
            base = 0 if level == 0 else K + (level - 1) * KK + fr * K
            chosen = [int(t) for t in p_tok[base: base + k]]
            finite = values[np.isfinite(values)]
            e_row = tol * float(finite.max() - finite.min())
            judge(where, values, chosen, lambda j: e_row)
            parent = frontier[fr]
            for r in range(k):
                assert p_par[base + r] == parent, (where, r)
                e_path[base + r] = e_path[parent] + e_row
            return chosen
        if where[0] == "frontier":
            level = where[1]
            base = K + (level - 1) * KK
            if level + 1 < D:      # the GPU's next frontier = the parents of the next level's candidates, in rank order
                nxt = [int(p_par[K + level * KK + r * K]) for r in range(K)]
                chosen = [p - base for p in nxt]
                judge(where, values, chosen, lambda j: e_path[base + j])
                frontier[:] = nxt
                return chosen
            return sd.topk_desc(values, k)        # the last level's frontier is never expanded
        assert where[0] == "keep"
        chosen = [p for p in node_pool[1:]]
        judge(where, values, chosen, lambda j: e_path[j])
        return chosen

    def root_pick(where, values, k):
        out = pick(where, values, k)
        if where[0] == "root":
            frontier[:] = list(range(k))
        return out

    forced_tree, forced_pool = sd.draft_expand(cfg, tw, dw, st, root, K, D, N, pick=root_pick)
    for j, cand in enumerate(forced_pool):          # (1)
        err = abs(float(p_sc[j]) - cand.score)
        seen["worst_score_err"] = max(seen["worst_score_err"], err / max(e_path[j], 1e-30))
        assert err <= e_path[j], (j, float(p_sc[j]), cand.score, e_path[j])
    np.testing.assert_array_equal(t_tok, forced_tree.token)          # (3)
    np.testing.assert_array_equal(t_par, forced_tree.parent)
    np.testing.assert_array_equal(t_dep, forced_tree.depth)
    seen["identical"] = seen["own"] == seen["choices"]
    if seen["identical"]:                           # (4)
        own_tree, _ = sd.draft_expand(cfg, tw, dw, st, root, K, D, N)
        np.testing.assert_array_equal(t_tok, own_tree.token)
        np.testing.assert_array_equal(t_par, own_tree.parent)
    return seen
