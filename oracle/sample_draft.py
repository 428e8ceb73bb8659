"""Oracle for sampled drafting on a static tree template (the drafting half of the sampling mode).

Test infrastructure only (see the package docstring).

What the paper fixes: rollouts are sampled (temperature 0.9 in the RL runs, Section 6.1) and the
speculative step must leave the output distribution exactly the target's (Section 1 "Mathematically
Lossless", Section 3 principle (a)); drafting is tree-based with the three parameters Draft_Depth,
topK and Tokens_to_Verify (Section 5.1).  It gives no drafting rule for the sampled case.

Reading taken here (also listed in the design document).  The acceptance rule of accept.c is
lossless only if every sibling list is a prefix of without-replacement draws from its parent's draft
distribution q and the SHAPE of the tree does not depend on the drawn values.  So:

  * shape = a static template fixed by (topK, Draft_Depth, Tokens_to_Verify) alone: of the full
    K-ary tree of depth D, in which a node is the sequence of child ranks (r_1 .. r_d) leading to it,
    keep the N-1 nodes of highest prior weight  prod_j a0 (1-a0)^(r_j)  with a0 = 0.6 (the chance
    that a first-ranked child is accepted, geometric in the rank), plus the root.  The weight falls
    with depth and with every rank, so the kept set is closed under "parent of" and "earlier
    sibling of".  Equal weights: the shallower node first, then the lexicographically smaller rank
    sequence.  Nodes are numbered by depth, then parent number, then rank (parents precede children);
  * tokens: the children of a node are drawn one after the other from q = softmax(logits / tau) of
    the drafter at that node, each draw removing the drawn token.  The arithmetic is the integer
    arithmetic of accept.c's final draw, so that the acceptance rule sees exactly the process it
    presupposes: Qw_j = floor(q_j * 2^32) with q in fp32; a draw with the 32-bit uniform U picks the
    first index whose running integer sum exceeds (U * sum(Qw)) >> 32; then Qw_pick = 0.

Pins (tests/test_oracle_sample_draft.py): the template against a brute-force ranking of the fully
enumerated tree, its closed forms (chain for K=1, star for D=1, the whole tree when N is large) and
a hand-worked case; draws against the closed form q_a q_b / (1 - q_a) of successive sampling and
hand-worked thresholds; the chi-square test of two generated tokens against p(x1) p(x2|x1) with
trees produced by exactly these two functions.
"""
from __future__ import annotations

import heapq
import math
from typing import List, Tuple

import numpy as np

from . import decoder as dec
from . import sd

ALPHA0 = 0.6
TWO32 = 4294967296.0


def _weight(ranks: Tuple[int, ...]) -> float:
    return len(ranks) * math.log(ALPHA0) + sum(ranks) * math.log(1.0 - ALPHA0)


def static_template(K: int, D: int, N: int):
    """(parent [n], rank [n], depth [n]) of the template; node 0 is the root (parent -1, rank -1)."""
    kept: List[Tuple[int, ...]] = []
    heap = [((-_weight((0,)), 1, (0,)))] if (K >= 1 and D >= 1) else []
    while heap and len(kept) < N - 1:
        _, _, ranks = heapq.heappop(heap)
        kept.append(ranks)
        if len(ranks) < D:  # its first child
            c = ranks + (0,)
            heapq.heappush(heap, (-_weight(c), len(c), c))
        if ranks[-1] + 1 < K:  # its next sibling
            s = ranks[:-1] + (ranks[-1] + 1,)
            heapq.heappush(heap, (-_weight(s), len(s), s))
    # number by depth, then parent number, then rank
    number = {(): 0}
    parent, rank, depth = [-1], [-1], [0]
    for d in range(1, D + 1):
        level = [r for r in kept if len(r) == d]
        level.sort(key=lambda r: (number[r[:-1]], r[-1]))
        for r in level:
            number[r] = len(parent)
            parent.append(number[r[:-1]])
            rank.append(r[-1])
            depth.append(d)
    return np.array(parent, dtype=np.int64), np.array(rank, dtype=np.int64), np.array(depth, dtype=np.int64)


def draw_children(q_row, uniforms):
    """Tokens drawn one after the other without replacement from the fp32 distribution q_row [V]
    with the 32-bit uniforms given (one per child)."""
    qw = [int(math.floor(float(x) * TWO32)) for x in np.asarray(q_row, dtype=np.float32).astype(np.float64)]
    picks = []
    for u in uniforms:
        total = sum(qw)
        thr = (int(u) * total) >> 32
        run, pick = 0, len(qw) - 1
        for j, w in enumerate(qw):
            run += w
            if run > thr:
                pick = j
                break
        picks.append(pick)
        qw[pick] = 0
    return picks


def draw_children_rows(q, u):
    """The same draw for many rows at once: q [B, V] fp32, u [B, k] uint32 -> tokens [B, k]
    (vectorised so that the statistical pins can afford 1e6 rows; identical integer arithmetic,
    with the 96-bit product U * sum split into exact 64-bit pieces)."""
    q = np.asarray(q, dtype=np.float32)
    u = np.asarray(u, dtype=np.uint64)
    B, V = q.shape
    qw = np.floor(q.astype(np.float64) * TWO32).astype(np.uint64)
    out = np.zeros((B, u.shape[1]), dtype=np.int64)
    rows = np.arange(B)
    for c in range(u.shape[1]):
        total = qw.sum(axis=1)
        thr = u[:, c] * (total >> np.uint64(32)) + ((u[:, c] * (total & np.uint64(0xFFFFFFFF))) >> np.uint64(32))
        run = np.cumsum(qw, axis=1)
        hit = run > thr[:, None]
        pick = np.where(hit.any(axis=1), hit.argmax(axis=1), V - 1)
        out[:, c] = pick
        qw[rows, pick] = 0
    return out


def softmax_temperature(logits, temperature):
    """softmax(logits / temperature) in float64, returned in fp32 (the precision the boundary hands
    the distribution over in)."""
    z = np.asarray(logits, dtype=np.float64) / float(temperature)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return (e / e.sum(axis=-1, keepdims=True)).astype(np.float32)


def draft_sample(cfg, tw, dw, st: sd.SeqState, root_token: int, K: int, D: int, N: int, temperature: float, u_draw,
                 forced_tokens=None):
    """Sampled drafting of one sequence on the static template.  u_draw [n] uint32: entry i is the
    uniform that draws node i (entry 0 unused).  Returns (Tree, q [n, V] fp32) where row i of q is
    the distribution node i's children were drawn from (zero rows for nodes without children).
    With forced_tokens [n] the nodes take those tokens instead of drawn ones (the distributions of
    somebody else's tree: used to compare q where a draw may legitimately differ).

    A node at depth s with children becomes drafter entry ctx+s-1 exactly as in the deterministic
    expansion: input = its token's embedding joined with its parent's drafter output; it attends to
    every committed entry, to its ancestors' provisional entries and to itself.  Provisional entries
    sit at cache rows draft_len + j, j counting the nodes with children in node order (root excluded)."""
    parent, rank, depth = static_template(K, D, N)
    n = len(parent)
    V = len(st.root_logp)
    kids = [[c for c in range(n) if parent[c] == i] for i in range(n)]
    token = np.zeros(n, dtype=np.int64)
    token[0] = root_token
    q = np.zeros((n, V), dtype=np.float32)
    feats = {0: st.root_feat}
    slot_of = {}
    base_len = st.draft_len

    def draw(i):
        if kids[i] and forced_tokens is not None:
            for c in kids[i]:
                token[c] = int(forced_tokens[c])
        elif kids[i]:
            for c, t in zip(kids[i], draw_children(q[i], [u_draw[c] for c in kids[i]])):
                token[c] = t

    q[0] = softmax_temperature(st.root_logp, temperature)
    draw(0)
    next_slot = base_len
    for d in range(1, D):
        inner = [i for i in range(n) if depth[i] == d and kids[i]]
        if not inner:
            break
        x = sd.drafter_input(cfg, tw, dw, [int(token[i]) for i in inner], [feats[int(parent[i])] for i in inner])
        slots = next_slot + np.arange(len(inner))
        next_slot += len(inner)
        pos = np.full(len(inner), base_len + d - 1)
        visible = np.zeros((len(inner), int(slots.max()) + 1), dtype=bool)
        visible[:, :base_len] = True
        for r, i in enumerate(inner):
            slot_of[i] = int(slots[r])
            a = i
            while a > 0:
                visible[r, slot_of[a]] = True
                a = int(parent[a])
        x = dec.block_rows(cfg, dw["layer"], x, pos, slots, visible, st.draft, st.store)
        logits = dec.lm_logits(cfg, tw, x)
        for r, i in enumerate(inner):
            feats[i] = x[r]
            q[i] = softmax_temperature(logits[r], temperature)
            draw(i)
    return sd.Tree(token, parent, depth, np.zeros(n)), q
