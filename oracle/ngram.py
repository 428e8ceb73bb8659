"""Oracle (test infrastructure, not part of the product path): the model-free drafter of Section 5.3
("Model-free Drafter"): an n-gram retrieval database per prompt, filled from that prompt's rollout
responses, queried with the tokens that precede the position to predict, and turned into a candidate
tree by the same confidence-ordered expansion as the learned drafter's (Section 5.1).

Readings (the section describes the mechanism in two sentences):
* order n: every window of k+1 consecutive tokens of an inserted response, k = 1 .. n-1, adds one
  count to (context = first k tokens) -> (next token = last one);
* a query uses the longest suffix of its context (at most n-1 tokens) that has been seen, backing
  off to shorter ones; continuations are ranked by count, equal counts by lower token id; their
  "confidence" is log(count / total count of that context);
* tree: node 0 is the root (the last context token).  Level 1 = the K best continuations of the
  context; at every further level each frontier node (context + the path's tokens) proposes its K
  best continuations, and the K best new candidates by path score (ties: created earlier) form the
  next frontier, for `depth` levels; the N-1 best candidates by path score (+ root) are kept in
  creation order.  A node without continuations proposes nothing;
* when fewer than N-1 candidates exist the tree is padded with children of the root carrying the
  smallest token ids the root has no child for yet (score -inf): any token is a legitimate draft,
  the target decides; this keeps the tree shape [n] the verification call expects.
"""
import math
from collections import defaultdict


class NGramDB:
    def __init__(self, n):
        assert n >= 2
        self.n = n
        self.tables = defaultdict(lambda: defaultdict(lambda: defaultdict(int)))   # prompt -> context tuple -> token -> count

    def insert(self, prompt_id, tokens):
        t = [int(x) for x in tokens]
        table = self.tables[prompt_id]
        for k in range(1, self.n):
            for i in range(len(t) - k):
                table[tuple(t[i:i + k])][t[i + k]] += 1

    def continuations(self, prompt_id, context):
        """[(token, log-probability)] of the longest seen suffix of `context`, best first."""
        table = self.tables.get(prompt_id)
        if not table:
            return []
        c = [int(x) for x in context]
        for k in range(min(self.n - 1, len(c)), 0, -1):
            nxt = table.get(tuple(c[len(c) - k:]))
            if nxt:
                total = sum(nxt.values())
                ranked = sorted(nxt.items(), key=lambda kv: (-kv[1], kv[0]))
                return [(tok, math.log(cnt / total)) for tok, cnt in ranked]
        return []

    def propose(self, prompt_id, context, depth, K, N, pad=True):
        """Tree as (token, parent, score) lists of length N (or fewer without padding)."""
        context = [int(x) for x in context]
        pool = []                                    # (token, score, parent pool index or -1, path tokens)
        frontier = []
        for tok, lp in (self.continuations(prompt_id, context)[:K] if depth >= 1 else []):   # depth 0: no drafts
            pool.append((tok, lp, -1, [tok]))
            frontier.append(len(pool) - 1)
        for _ in range(1, depth):
            base = len(pool)
            for pi in frontier:
                _, score, _, path = pool[pi]
                for tok, lp in self.continuations(prompt_id, context + path)[:K]:
                    pool.append((tok, score + lp, pi, path + [tok]))
            new = list(range(base, len(pool)))
            new.sort(key=lambda i: (-pool[i][1], i))
            frontier = new[:K]
            if not frontier:
                break
        order = sorted(range(len(pool)), key=lambda i: (-pool[i][1], i))[:max(N - 1, 0)]
        keep = sorted(order)
        node_of = {pi: j + 1 for j, pi in enumerate(keep)}
        token, parent, score = [context[-1]], [-1], [0.0]
        for pi in keep:
            tok, sc, par, _ = pool[pi]
            token.append(tok)
            parent.append(0 if par < 0 else node_of[par])
            score.append(sc)
        if pad:
            used = {token[i] for i in range(1, len(token)) if parent[i] == 0}
            t = 0
            while len(token) < N:
                if t not in used:
                    token.append(t)
                    parent.append(0)
                    score.append(-math.inf)
                t += 1
        return token, parent, score
