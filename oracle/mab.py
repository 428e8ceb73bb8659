"""Oracle (test infrastructure, not part of the product path): the Bucketed-Epsilon-Greedy strategy
selector of Algorithm 1 (Section 5.2, "Auto-Tune Algorithm") and the elastic activation rule of
Section 5.1 ("Adaptivity is Necessary"), written out in the paper's notation with Python deques.

Strategy s = (Draft_Depth, topK, Tokens_to_Verify).  Random numbers the selector draws are passed in
by the caller as 32-bit integers (U1 decides explore/exploit, U2 picks the explored arm), so a test
can feed the same draws to this oracle and to the library.

Readings where Algorithm 1 is silent:
* the number of distinct Tokens_to_Verify values must equal the number of thresholds m;
* a batch size below t_1 falls into bucket B_1 (there is no smaller bucket to put it in);
* u = (U1 + 0.5) / 2^32; "random s in V" = V[floor(U2 * |V| / 2^32)], V in the caller's strategy order;
* Median of an empty deque = +infinity, so arms never tried are exploited first; median of an even
  count = mean of the two middle values; argmax ties go to the earlier strategy in V;
* elastic activation: speculative decoding is on only while batch_size < sd_threshold (default 32);
  select returns None when it is off.
"""
from collections import deque


class BEG:
    def __init__(self, strategies, thresholds, epsilon, w, sd_threshold=32):
        """Procedure Initialize."""
        self.S = [tuple(s) for s in strategies]
        self.T = list(thresholds)
        self.epsilon, self.w, self.sd_threshold = float(epsilon), int(w), int(sd_threshold)
        verify_values = sorted({s[2] for s in self.S}, reverse=True)     # GroupByVerifyTokens, descending
        if len(verify_values) != len(self.T) or any(self.T[i] >= self.T[i + 1] for i in range(len(self.T) - 1)):
            raise ValueError("need one strictly increasing threshold per Tokens_to_Verify value")
        self.groups = [[i for i, s in enumerate(self.S) if s[2] == v] for v in verify_values]   # S_1 .. S_m
        self.R = [deque(maxlen=self.w) for _ in self.S]
        self.A = [deque(maxlen=self.w) for _ in self.S]

    def bucket(self, batch_size):
        """Index i (0-based) of the bucket B_i = [t_i, t_{i+1} - 1] (B_m = [t_m, inf)) holding batch_size."""
        i = 0
        for j, t in enumerate(self.T):
            if batch_size >= t:
                i = j
        return i

    def record(self, s, elapsed_time, accept_lens, batch_size):
        """Procedure Record for strategy index s."""
        a_bar = sum(accept_lens) / batch_size + 1
        r = a_bar * batch_size / elapsed_time
        self.R[s].append(r)
        self.A[s].append(a_bar)
        return a_bar, r

    @staticmethod
    def median(values):
        v = sorted(values)
        n = len(v)
        if n == 0:
            return float("inf")
        return v[n // 2] if n % 2 else (v[n // 2 - 1] + v[n // 2]) / 2

    def select(self, batch_size, U1, U2):
        """Procedure SelectStrategy (strategy index), or None when the elastic rule keeps SD off."""
        if batch_size >= self.sd_threshold:
            return None
        V = self.groups[self.bucket(batch_size)]
        if len(V) == 1:
            return V[0]
        u = (U1 + 0.5) / 2.0 ** 32
        if u < self.epsilon:
            return V[(U2 * len(V)) >> 32]
        best, best_m = V[0], self.median(self.R[V[0]])
        for s in V[1:]:
            m = self.median(self.R[s])
            if m > best_m:
                best, best_m = s, m
        return best
