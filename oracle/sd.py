"""Oracle speculative-decoding step: drafter extend, tree expansion, pruning, target
verification, cache commit, plus the autoregressive definition it must reproduce.

Test infrastructure only (see the package docstring).

What the paper fixes and where:
  * Section 2.2 "Mechanism of Speculative Decoding": the drafter proposes tokens, the target
    checks all of them in one forward pass, the drafted prefix up to the first disagreement is
    kept together with the target's own token at that position; the result is distributed
    exactly like plain decoding of the target ("lossless").
  * Section 4.1 "Model Architecture" / "Training Process": the drafter is ONE decoder block that
    reuses the target's embedding and LM head; its input is the target's hidden state joined with
    the token embedding and passed through a linear layer (2h -> h); it then drafts
    autoregressively from its own output.
  * Section 5.1 "Tree-based Drafting" and the tree-decoding figure: explore the topK most likely
    continuations per step for Draft_Depth steps, then keep the Tokens_to_Verify nodes of highest
    draft confidence for verification.
  * Algorithm 1, procedure Record: accept lengths exclude the target's own ("bonus") token:
    mean emitted tokens = sum(accept_lens)/batch + 1.

Readings taken where the paper is silent (each also listed in the design document):
  * hidden state handed to the drafter = output of the last decoder block before the final norm;
  * drafter cache entry s pairs (token s+1, hidden state s) and uses rotary position s;
  * node confidence = sum of draft log-probabilities along the path from the root (the only
    choice that keeps the selected set closed under "parent of"); ties go to the candidate
    created earlier;
  * the next frontier is the topK of the K*K candidates of the level just expanded;
  * Tokens_to_Verify counts the root; tree node 0 is the root (the last emitted token, not yet in
    the cache) and the other nodes follow in creation order, so a parent precedes its children;
  * verification writes node i's key/value at cache slot ctx+i with rotary position ctx+depth;
    commit moves the accepted nodes' rows to slots ctx+0..ctx+a and advances the length by a+1.

Pins (tests/test_oracle_sd.py): greedy SD output == cache-free autoregressive greedy decoding;
verification of a tree == cache-free causal forward of every root-to-node path; chain tree from an
empty cache == dense causal forward; committed cache == keys/values of the dense forward of the
emitted tokens; tree invariants and a brute-force re-derivation of frontier and selection on a
toy Markov drafter; the pool size 2+3*4 = 14 of the paper's topK=2, depth=4 example; the real
drafter's expansion (`draft_expand`: provisional rows, positions, visibility) against a cache-free
drafter forward over (committed entries ++ root-to-node path) for every candidate of the pool.
The exact tree of the paper's figure (its tokens and probabilities are not in the text) and
every accept length or speed-up the paper prints need trained weights: parity unpinned.
"""
from __future__ import annotations

import dataclasses
from typing import Callable, List

import numpy as np

from . import decoder as dec


# ----------------------------------------------------------------------------- data
@dataclasses.dataclass
class Cand:
    token: int
    score: float  # sum of draft log-probabilities from the root
    parent: int  # pool index of the parent candidate, -1 = child of the root
    depth: int  # 1 = child of the root


@dataclasses.dataclass
class Tree:
    token: np.ndarray  # [n] int; node 0 = root
    parent: np.ndarray  # [n] int; -1 for the root
    depth: np.ndarray  # [n] int; root = 0
    score: np.ndarray  # [n] float; root = 0

    @property
    def n(self):
        return len(self.token)

    def ancestors_or_self(self, i):
        out = []
        while i >= 0:
            out.append(i)
            i = int(self.parent[i])
        return out[::-1]


class SeqState:
    """One sequence: committed target cache, committed drafter cache, the pending root token."""

    def __init__(self, cfg, capacity, store=dec.identity):
        self.cfg = cfg
        self.store = store
        self.target = [dec.LayerCache(cfg, capacity) for _ in range(cfg.n_layers)]
        self.draft = dec.LayerCache(cfg, capacity)
        self.ctx = 0  # committed target tokens
        self.draft_len = 0  # committed drafter entries
        self.root_feat = None  # drafter output for the entry holding the root token
        self.root_logp = None  # its log-probabilities over the token after the root


def topk_desc(values, k):
    """Indices of the k largest values; equal values keep the lower index first."""
    values = np.asarray(values)
    order = np.lexsort((np.arange(len(values)), -values))
    return [int(i) for i in order[:k]]


# ----------------------------------------------------------------------------- tree expansion / pruning
def pick_best(where, values, k):
    """Every choice of the tree building goes through a function of this signature: `where` names
    the decision (("root",), ("children", level, frontier rank), ("frontier", level), ("keep",)),
    `values` are the quantities it ranks and the result lists the k chosen indices, best first.
    The method's own choice is the k largest (lower index on ties); tests that judge a tree built
    in lower precision pass a function that replays that tree's choices instead and inspects
    `values` to see how far from the best each one was."""
    return topk_desc(values, k)


def expand_tree(root_logp, level_fn: Callable[[int, List[int], List[Cand]], np.ndarray], K: int, D: int, pick=pick_best):
    """Candidate pool of Section 5.1's tree: level 0 = the K most likely tokens after the root;
    for each further level the K frontier nodes are run through the drafter (`level_fn(level,
    frontier_pool_indices, pool)` returns their [K, V] log-probabilities), each gives its K most
    likely children, and the K best of those K*K (by path score) form the next frontier.
    Pool order = creation order: level, then frontier rank, then child rank."""
    pool: List[Cand] = []
    for t in pick(("root",), root_logp, K):
        pool.append(Cand(t, float(root_logp[t]), -1, 1))
    frontier = list(range(len(pool)))
    for level in range(1, D):
        logp = level_fn(level, frontier, pool)
        base = len(pool)
        for fr, pi in enumerate(frontier):
            for t in pick(("children", level, fr), logp[fr], K):
                pool.append(Cand(t, pool[pi].score + float(logp[fr][t]), pi, level + 1))
        frontier = [base + i for i in pick(("frontier", level), [c.score for c in pool[base:]], K)]
    return pool


def prune_tree(pool: List[Cand], root_token: int, N: int, pick=pick_best) -> Tree:
    """Keep the N-1 pool candidates of highest path score (+ the root as node 0), in pool order."""
    keep = sorted(pick(("keep",), [c.score for c in pool], max(0, min(N - 1, len(pool)))))
    node_of = {pi: i + 1 for i, pi in enumerate(keep)}
    token, parent, depth, score = [root_token], [-1], [0], [0.0]
    for pi in keep:
        c = pool[pi]
        token.append(c.token)
        parent.append(0 if c.parent < 0 else node_of[c.parent])
        depth.append(c.depth)
        score.append(c.score)
    return Tree(np.array(token, dtype=np.int64), np.array(parent, dtype=np.int64),
                np.array(depth, dtype=np.int64), np.array(score, dtype=np.float64))


def chain_tree(tokens) -> Tree:
    n = len(tokens)
    return Tree(np.asarray(tokens, dtype=np.int64), np.arange(-1, n - 1, dtype=np.int64),
                np.arange(n, dtype=np.int64), np.zeros(n))


# ----------------------------------------------------------------------------- drafter
def drafter_input(cfg, tw, dw, tokens, hiddens):
    """fc([embed(token) ; hidden]) for each (token, hidden) pair (Section 4.1)."""
    e = tw["embed"][np.asarray(tokens, dtype=np.int64)]
    return np.concatenate([e, np.asarray(hiddens)], axis=1) @ dw["fc"].T


def draft_extend(cfg, tw, dw, st: SeqState, new_tokens, new_hiddens):
    """Append drafter cache entries for newly committed positions.

    Entry s pairs token s+1 with the target's hidden state at position s; `new_tokens[j]`,
    `new_hiddens[j]` are those pairs for s = draft_len + j.  Afterwards the last entry's output
    gives the drafter's distribution for the token after the root."""
    n = len(new_tokens)
    if n == 0:
        return
    x = drafter_input(cfg, tw, dw, new_tokens, new_hiddens)
    pos = st.draft_len + np.arange(n)
    T = st.draft_len + n
    visible = np.arange(T)[None, :] <= pos[:, None]
    x = dec.block_rows(cfg, dw["layer"], x, pos, pos, visible, st.draft, st.store)
    st.draft_len += n
    st.root_feat = x[-1]
    st.root_logp = dec.log_softmax(dec.lm_logits(cfg, tw, x[-1]))


def draft_expand(cfg, tw, dw, st: SeqState, root_token: int, K: int, D: int, N: int, pick=pick_best):
    """Tree expansion with the real drafter, then pruning.  Returns (Tree, pool).

    A frontier node at depth s (its token is a candidate for position ctx+s) becomes drafter
    entry ctx+s-1: its input joins its token's embedding with its parent's drafter output; it
    attends to every committed entry, to its ancestors' provisional entries and to itself.
    Provisional entries of level `lv` sit at cache rows draft_len + (lv-1)*K + frontier rank and
    are simply overwritten by the next extend."""
    feats = {}  # pool index -> drafter output feature
    slot_of = {}  # pool index -> provisional cache row
    base_len = st.draft_len

    def level_fn(level, frontier, pool):
        toks = [pool[pi].token for pi in frontier]
        par = [st.root_feat if pool[pi].parent < 0 else feats[pool[pi].parent] for pi in frontier]
        x = drafter_input(cfg, tw, dw, toks, par)
        slots = base_len + (level - 1) * K + np.arange(len(frontier))
        pos = np.full(len(frontier), base_len + level - 1)
        T = int(slots.max()) + 1
        visible = np.zeros((len(frontier), T), dtype=bool)
        visible[:, :base_len] = True
        for r, pi in enumerate(frontier):
            slot_of[pi] = int(slots[r])
            a = pi
            while a >= 0:
                visible[r, slot_of[a]] = True
                a = pool[a].parent
        x = dec.block_rows(cfg, dw["layer"], x, pos, slots, visible, st.draft, st.store)
        for r, pi in enumerate(frontier):
            feats[pi] = x[r]
        return dec.log_softmax(dec.lm_logits(cfg, tw, x))

    pool = expand_tree(st.root_logp, level_fn, K, D, pick) if (D >= 1 and N > 1) else []
    return prune_tree(pool, root_token, N, pick), pool


# ----------------------------------------------------------------------------- target verification
def verify(cfg, tw, st: SeqState, tree: Tree):
    """One target forward over all tree nodes (Section 2.2): node i attends to the committed
    context and to its ancestors-or-self; its rotary position is ctx + depth; its key/value go to
    the provisional cache row ctx + i.  Returns (logits [n, V], hidden [n, h])."""
    n = tree.n
    ctx = st.ctx
    x = tw["embed"][tree.token]
    pos = ctx + tree.depth
    slots = ctx + np.arange(n)
    visible = np.zeros((n, ctx + n), dtype=bool)
    visible[:, :ctx] = True
    for i in range(n):
        for a in tree.ancestors_or_self(i):
            visible[i, ctx + a] = True
    for l, lw in enumerate(tw["layers"]):
        x = dec.block_rows(cfg, lw, x, pos, slots, visible, st.target[l], st.store)
    return dec.lm_logits(cfg, tw, x), x


def accept_greedy(tree: Tree, logits):
    """Section 2.2's rule at temperature 0: from the root, follow the child whose token equals the
    target's most likely token at the current node; stop at the first miss and emit the target's
    token there.  Returns (accept_len, path node indices [a+1], emitted tokens [a+1]).
    (Reference form in float64; the fp32, batch form used for parity is in accept.c.)"""
    cur, path, out = 0, [0], []
    while True:
        t = int(np.argmax(logits[cur]))
        nxt = [c for c in range(tree.n) if tree.parent[c] == cur and tree.token[c] == t]
        out.append(t)
        if not nxt:
            return len(path) - 1, path, out
        cur = nxt[0]
        path.append(cur)


def commit(st: SeqState, path):
    """Keep the accepted nodes: row ctx+path[j] -> row ctx+j in every layer, length += len(path).
    The emitted bonus token is not cached: it is the next step's root."""
    ctx = st.ctx
    for c in st.target:
        for j, p in enumerate(path):
            c.k[ctx + j] = c.k[ctx + p].copy()
            c.v[ctx + j] = c.v[ctx + p].copy()
    st.ctx += len(path)


def commit_rows(k_rows, v_rows, ctx: int, path):
    """Same move on bare arrays [slots, ...] (used where commit is tested apart from the model)."""
    for j, p in enumerate(path):
        k_rows[ctx + j] = k_rows[ctx + p].copy()
        v_rows[ctx + j] = v_rows[ctx + p].copy()
    return ctx + len(path)


# ----------------------------------------------------------------------------- whole step / loops
def prefill(cfg, tw, dw, st: SeqState, prompt, chunk=64):
    """Put prompt[:-1] into both caches (chain trees of <= chunk tokens through `verify`, all rows
    committed); prompt[-1] stays outside as the first root.  Returns the root token."""
    body = [int(t) for t in prompt[:-1]]
    for o in range(0, len(body), chunk):
        part = body[o : o + chunk]
        _, hid = verify(cfg, tw, st, chain_tree(part))
        commit(st, list(range(len(part))))
        nxt = [int(t) for t in prompt[o + 1 : o + 1 + len(part)]]
        draft_extend(cfg, tw, dw, st, nxt, hid)
    return int(prompt[-1])


def sd_step(cfg, tw, dw, st: SeqState, root: int, K: int, D: int, N: int, tree_fn=None):
    """One greedy speculative-decoding step.  Returns (emitted tokens, accept_len, tree, logits,
    hidden, path, pool).  `tree_fn(st, root) -> Tree` replaces the drafter's tree when given
    (tests use it to verify trees from other proposers: losslessness must hold for any tree)."""
    if tree_fn is None:
        tree, pool = draft_expand(cfg, tw, dw, st, root, K, D, N)
    else:
        tree, pool = tree_fn(st, root), None
    logits, hidden = verify(cfg, tw, st, tree)
    a, path, out = accept_greedy(tree, logits)
    commit(st, path)
    draft_extend(cfg, tw, dw, st, out, hidden[path])
    return out, a, tree, logits, hidden, path, pool


def sd_generate(cfg, tw, dw, prompt, n_steps, K, D, N, capacity=None, store=dec.identity, tree_fn=None):
    cap = capacity or (len(prompt) + n_steps * (D + 1) + N + K * D + 8)
    st = SeqState(cfg, cap, store)
    root = prefill(cfg, tw, dw, st, prompt)
    emitted, accept_lens = [], []
    for _ in range(n_steps):
        out, a, *_ = sd_step(cfg, tw, dw, st, root, K, D, N, tree_fn)
        emitted.extend(out)
        accept_lens.append(a)
        root = out[-1]
    return emitted, accept_lens, st


def ar_greedy(cfg, tw, prompt, n_new):
    """The definition SD must reproduce: y_t = argmax target(prompt, y_<t), one token at a time,
    recomputed from scratch with no cache."""
    seq = [int(t) for t in prompt]
    for _ in range(n_new):
        logits, *_ = dec.dense_forward(cfg, tw, seq)
        seq.append(int(np.argmax(logits[-1])))
    return seq[len(prompt) :]


def record_reward(elapsed_time, accept_lens, batch_size):
    """Algorithm 1, procedure Record: mean emitted tokens and the reward (tokens per unit time)."""
    a_bar = sum(accept_lens) / batch_size + 1
    return a_bar, a_bar * batch_size / elapsed_time
