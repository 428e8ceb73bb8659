/* Oracle acceptance rules of the speculative-decoding step, plain C, one sequence at a time.
 *
 * Test infrastructure only: never linked into or called by the HIP library.
 *
 * Greedy (Section 2.2, "Mechanism of Speculative Decoding"): keep the drafted tokens up to the
 * first one that differs from the target's prediction, plus the target's own token there.
 * On a tree: from the root follow the child whose token is the target's argmax at the current
 * node.  argmax is taken on the fp32 logits, lowest index on ties.
 *
 * Sampling: the paper only states that the output must be distributed exactly as the target's
 * (Section 1 "Mathematically Lossless", Section 3 principle (a)) and gives no rule.  The rule
 * here is recursive rejection sampling over sibling lists drawn without replacement from the
 * draft distribution q of their parent: child c is accepted with probability min(1, p(c)/q(c));
 * after a rejection p <- normalise(max(p - q, 0)) and q <- normalise(q with c removed); when no
 * child is left the emitted token is drawn from the current p.
 *
 * Arithmetic, chosen so that any implementation reproduces every decision bit for bit:
 *   - weights are integers: W_j = floor(exp(l_j/tau - max) * 2^32) with exp in double,
 *     Qw_j = floor(q_j * 2^32); every sum over the vocabulary is an exact integer sum;
 *   - p_j = W_j / S and q_j = Qw_j / SQ are single IEEE double divisions; the accept test is
 *     u * q_c < p_c with u = (U + 0.5) / 2^32 for the caller's 32-bit uniform U;
 *   - the residual is floor(max(W_j/S - Qw_j/SQ, 0) * 2^32);
 *   - the final draw is the first index whose running integer sum exceeds (U_final * S) >> 32.
 * Quantising to 2^-32 perturbs each probability by at most 2^-32 / p_max, which bounds the
 * departure from exact losslessness by V * 2^-32 in total variation.
 *
 * Sampling on trees whose shape DOES depend on the drafter's values (the deterministic top-K trees of
 * Section 5.1): the draft distribution may then not enter the rule at all.  "Target only": with the
 * current target weights, child c is accepted with probability weight(c) / total -- the chance that
 * a draw from the target would have been c -- and on rejection its weight is removed; when no child
 * is left the emitted token is drawn from what remains.  By the chain rule this emits exactly a draw
 * from the target at every node, for any tree.  All integer: accept iff (U * total) >> 32 < weight(c)
 * (the inverse-CDF draw with c placed first), then total -= weight(c), weight(c) = 0; the final draw as above.
 *
 * A child whose token lies outside the vocabulary is skipped by both sampling rules (it has probability
 * zero under any distribution: never accepted, nothing else changes).
 *
 * Near-threshold flags.  Given identical weights every decision above is exact; computed from
 * identical LOGITS, two platforms can still differ in the last bit of a double `exp`, i.e. by one
 * unit in a weight W_j (and so by a few units in S or in a running sum).  The *_near variants below
 * report, per sequence, whether any decision taken was within 8 units of 2^-32 of going the other
 * way: |u q_c - p_c| < 8 * 2^-32 for an accept test of the p/q rule, |thr - W_c| <= 8 for one of the
 * target-only rule, and a final draw whose threshold lies within 8 units of either end of the picked
 * token's interval.  A parity test may tolerate a mismatch only in a flagged sequence.
 *
 * Pins (tests/test_oracle_accept.py): brute force over all root-to-leaf paths (greedy); a
 * chi-square test of two generated tokens against p(x1) p(x2|x1) on a 16-token vocabulary over
 * 1e6 draws with a negative control; the closed form sum_v min(p_v, q_v) for the first accept;
 * for the target-only rule the same chi-square test on deterministic top-K trees (the ones the
 * p/q rule is biased on), the closed form P(accept first child) = p(c) and hand-worked thresholds.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#define NEAR_UNITS 8 /* weight units (2^-32 of probability mass) a platform's exp may plausibly move a threshold by */

static void target_weights(const float *logit, int V, double tau, uint64_t *W, uint64_t *S) {
    double m = -INFINITY;
    for (int j = 0; j < V; ++j) {
        double x = (double)logit[j] / tau;
        if (x > m) m = x;
    }
    uint64_t s = 0;
    for (int j = 0; j < V; ++j) {
        double x = (double)logit[j] / tau;
        W[j] = (uint64_t)floor(exp(x - m) * 4294967296.0);
        s += W[j];
    }
    *S = s;
}

static void draft_weights(const float *q, int V, uint64_t *Qw, uint64_t *SQ) {
    uint64_t s = 0;
    for (int j = 0; j < V; ++j) {
        Qw[j] = (uint64_t)floor((double)q[j] * 4294967296.0);
        s += Qw[j];
    }
    *SQ = s;
}

/* All arrays are for one batch of B sequences with n tree nodes each; path/out rows have
 * `stride` entries.  token/parent [B][n]; logits [B][n][V] fp32. */
void oracle_accept_greedy(int B, int n, int V, int stride, const int32_t *token, const int32_t *parent,
                          const float *logits, int32_t *accept_len, int32_t *path_idx,
                          int32_t *out_tokens, int32_t *n_out) {
    for (int b = 0; b < B; ++b) {
        const int32_t *tok = token + (size_t)b * n, *par = parent + (size_t)b * n;
        int32_t *path = path_idx + (size_t)b * stride, *out = out_tokens + (size_t)b * stride;
        for (int j = 0; j < stride; ++j) { path[j] = -1; out[j] = -1; }
        int cur = 0, a = 0;
        path[0] = 0;
        for (;;) {
            const float *l = logits + ((size_t)b * n + cur) * V;
            int best = 0;
            for (int j = 1; j < V; ++j)
                if (l[j] > l[best]) best = j;
            out[a] = best;
            int next = -1;
            for (int c = cur + 1; c < n; ++c)
                if (par[c] == cur && tok[c] == best) { next = c; break; }
            if (next < 0 || a + 1 >= stride) break;
            cur = next;
            path[++a] = cur;
        }
        accept_len[b] = a;
        n_out[b] = a + 1;
    }
}

/* draft_q [B][n][V]: row i is the distribution node i's children were drawn from.
 * u_accept [B][n]: uniform used when node i is tested; u_final [B]: uniform of the final draw. */
void oracle_accept_sample_near(int B, int n, int V, int stride, float temperature, const int32_t *token,
                               const int32_t *parent, const float *logits, const float *draft_q,
                               const uint32_t *u_accept, const uint32_t *u_final, int32_t *accept_len,
                               int32_t *path_idx, int32_t *out_tokens, int32_t *n_out, int32_t *near) {
    uint64_t *W = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)V);
    uint64_t *Qw = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)V);
    uint64_t *R = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)V);
    const double tau = (double)temperature;
    for (int b = 0; b < B; ++b) {
        const int32_t *tok = token + (size_t)b * n, *par = parent + (size_t)b * n;
        int32_t *path = path_idx + (size_t)b * stride, *out = out_tokens + (size_t)b * stride;
        for (int j = 0; j < stride; ++j) { path[j] = -1; out[j] = -1; }
        int cur = 0, a = 0, nr = 0;
        path[0] = 0;
        uint64_t S, SQ;
        for (;;) { /* one iteration per node on the accepted path */
            target_weights(logits + ((size_t)b * n + cur) * V, V, tau, W, &S);
            draft_weights(draft_q + ((size_t)b * n + cur) * V, V, Qw, &SQ);
            int next = -1;
            for (int c = cur + 1; c < n && a + 1 < stride; ++c) {
                if (par[c] != cur) continue;
                int t = tok[c];
                if (t < 0 || t >= V) continue;
                double p = (double)W[t] / (double)S;
                double q = SQ > 0 ? (double)Qw[t] / (double)SQ : 0.0;
                double u = ((double)u_accept[(size_t)b * n + c] + 0.5) / 4294967296.0;
                if (fabs(u * q - p) < NEAR_UNITS / 4294967296.0) nr = 1;
                if (u * q < p) { next = c; break; }
                /* rejected: residual target (kept only if it has mass: it has none exactly when
                   p <= q everywhere, i.e. p == q, a case the accept test above never rejects
                   except through quantisation), then the draft without c */
                uint64_t s2 = 0;
                for (int j = 0; j < V; ++j) {
                    double pj = (double)W[j] / (double)S;
                    double qj = SQ > 0 ? (double)Qw[j] / (double)SQ : 0.0;
                    double r = pj - qj;
                    if (r < 0.0) r = 0.0;
                    R[j] = (uint64_t)floor(r * 4294967296.0);
                    s2 += R[j];
                }
                if (s2 > 0) {
                    for (int j = 0; j < V; ++j) W[j] = R[j];
                    S = s2;
                }
                Qw[t] = 0;
                SQ = 0;
                for (int j = 0; j < V; ++j) SQ += Qw[j];
            }
            if (next < 0) break;
            out[a] = tok[next];
            cur = next;
            path[++a] = cur;
        }
        /* emit one token from the current target weights */
        unsigned __int128 thr128 = ((unsigned __int128)u_final[b] * (unsigned __int128)S) >> 32;
        uint64_t thr = (uint64_t)thr128, run = 0;
        int pick = V - 1;
        for (int j = 0; j < V; ++j) {
            run += W[j];
            if (run > thr) { pick = j; break; }
        }
        if (run <= thr || run - thr <= NEAR_UNITS || thr - (run - W[pick]) < NEAR_UNITS) nr = 1;
        out[a] = pick;
        accept_len[b] = a;
        n_out[b] = a + 1;
        if (near) near[b] = nr;
    }
    free(W);
    free(Qw);
    free(R);
}

void oracle_accept_sample(int B, int n, int V, int stride, float temperature, const int32_t *token,
                          const int32_t *parent, const float *logits, const float *draft_q,
                          const uint32_t *u_accept, const uint32_t *u_final, int32_t *accept_len,
                          int32_t *path_idx, int32_t *out_tokens, int32_t *n_out) {
    oracle_accept_sample_near(B, n, V, stride, temperature, token, parent, logits, draft_q, u_accept, u_final,
                              accept_len, path_idx, out_tokens, n_out, NULL);
}

/* Target-only rule (see the header): u_accept [B][n] is the uniform used when node i is tested,
 * u_final [B] the uniform of the final draw. */
void oracle_accept_target_only_near(int B, int n, int V, int stride, float temperature, const int32_t *token,
                                    const int32_t *parent, const float *logits, const uint32_t *u_accept,
                                    const uint32_t *u_final, int32_t *accept_len, int32_t *path_idx,
                                    int32_t *out_tokens, int32_t *n_out, int32_t *near) {
    uint64_t *W = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)V);
    const double tau = (double)temperature;
    for (int b = 0; b < B; ++b) {
        const int32_t *tok = token + (size_t)b * n, *par = parent + (size_t)b * n;
        int32_t *path = path_idx + (size_t)b * stride, *out = out_tokens + (size_t)b * stride;
        for (int j = 0; j < stride; ++j) { path[j] = -1; out[j] = -1; }
        int cur = 0, a = 0, nr = 0;
        path[0] = 0;
        uint64_t S;
        for (;;) {
            target_weights(logits + ((size_t)b * n + cur) * V, V, tau, W, &S);
            int next = -1;
            for (int c = cur + 1; c < n && a + 1 < stride; ++c) {
                if (par[c] != cur) continue;
                int t = tok[c];
                if (t < 0 || t >= V) continue;
                uint64_t thr = (uint64_t)(((unsigned __int128)u_accept[(size_t)b * n + c] * (unsigned __int128)S) >> 32);
                if ((thr < W[t] ? W[t] - thr : thr - W[t]) <= NEAR_UNITS && W[t] > 0) nr = 1;
                if (thr < W[t]) { next = c; break; }
                S -= W[t];
                W[t] = 0;
            }
            if (next < 0) break;
            out[a] = tok[next];
            cur = next;
            path[++a] = cur;
        }
        uint64_t thr = (uint64_t)(((unsigned __int128)u_final[b] * (unsigned __int128)S) >> 32), run = 0;
        int pick = V - 1;
        for (int j = 0; j < V; ++j) {
            run += W[j];
            if (run > thr) { pick = j; break; }
        }
        if (run <= thr || run - thr <= NEAR_UNITS || thr - (run - W[pick]) < NEAR_UNITS) nr = 1;
        out[a] = pick;
        accept_len[b] = a;
        n_out[b] = a + 1;
        if (near) near[b] = nr;
    }
    free(W);
}

void oracle_accept_target_only(int B, int n, int V, int stride, float temperature, const int32_t *token,
                               const int32_t *parent, const float *logits, const uint32_t *u_accept,
                               const uint32_t *u_final, int32_t *accept_len, int32_t *path_idx,
                               int32_t *out_tokens, int32_t *n_out) {
    oracle_accept_target_only_near(B, n, V, stride, temperature, token, parent, logits, u_accept, u_final, accept_len,
                                   path_idx, out_tokens, n_out, NULL);
}
