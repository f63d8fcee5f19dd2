"""TEST INFRASTRUCTURE ONLY -- pure-Python, list-based simulation of WeightedKV.

One (sequence, head) unit, Python floats (IEEE double), Python lists with
`append` and `del`: the shape of the paper's Algorithm 1 taken literally, slow
and meant for tiny inputs.  It exists to pin the C oracle (wkv_oracle.c): the
two are written separately and must agree exactly on small random streams.

Readings taken where the paper is silent:
  * logits are scaled by 1/sqrt(d) (Section III-B writes the scale, III-A omits it);
  * the attention of step t runs over the cache *including* the new token and
    *before* compression (Algorithm 1 obtains A_t ahead of the capacity test);
  * Algorithm 1 excludes only the newest token from the arg-min; the
    recent window R generalises this to the R newest tokens (R=1 is the
    algorithm verbatim; Section V-A keeps a recent region in its experiments);
  * ties in the arg-min go to the oldest token;
  * the survivor keeps its own key, score sum and count (Algorithm 1 removes
    only index j).

Nothing on the product path may import this module.
"""
import math


class BruteUnit:
    def __init__(self, d, m, R, n_sink=0, merge=True, rounder=None):
        assert 1 <= R <= m and n_sink >= 0 and n_sink + R <= m
        self.d, self.m, self.R = d, m, R
        self.n_sink, self.merge, self.rounder = n_sink, merge, rounder
        self.K, self.V = [], []          # lists of d-lists
        self.a, self.n = [], []          # score sums, counts   (Algorithm 1: the two lists)
        self.pos, self.nmerged = [], []  # bookkeeping for tests only
        self.t = 0

    def step(self, q, k, v):
        """Returns (o, evict_slot, evict_pos); evict_* are -1 when nothing was evicted."""
        d = self.d
        # K_t = [K_{t-1}, k_t], V_t = [V_{t-1}, v_t]            (Section III-A)
        self.K.append(list(k)); self.V.append(list(v))
        self.pos.append(self.t); self.nmerged.append(1)
        L = len(self.K)
        # A_t = softmax(q^T K_t / sqrt(d)),  o_t = A_t^T V_t    (Section III-A, III-B)
        s = [sum(q[c] * self.K[i][c] for c in range(d)) / math.sqrt(d) for i in range(L)]
        mx = max(s)
        e = [math.exp(x - mx) for x in s]
        S = sum(e)
        A = [x / S for x in e]
        o = [sum(A[i] * self.V[i][c] for i in range(L)) for c in range(d)]
        # a = [a, 0] + A_t ; n = [n, 0] + 1                      (Algorithm 1: bookkeeping)
        self.a = [x + y for x, y in zip(self.a + [0.0], A)]
        self.n = [x + 1 for x in self.n + [0]]
        ev_slot, ev_pos = -1, -1
        if L > self.m:                                           # cache exceeds m
            abar = [self.a[i] / self.n[i] for i in range(L)]     # average scores
            cand = range(self.n_sink, L - self.R)                # arg-min outside protected regions
            j = min(cand, key=lambda i: (abar[i], i))
            if self.merge:                                       # convex merge
                den = abar[j] + abar[j + 1]
                if den > 0:
                    merged = [(abar[j] * self.V[j][c] + abar[j + 1] * self.V[j + 1][c]) / den
                              for c in range(d)]
                else:
                    merged = [0.5 * self.V[j][c] + 0.5 * self.V[j + 1][c] for c in range(d)]
                if self.rounder is not None:
                    merged = [self.rounder(x) for x in merged]
                self.V[j + 1] = merged
                self.nmerged[j + 1] += self.nmerged[j]
            ev_slot, ev_pos = j, self.pos[j]
            for lst in (self.K, self.V, self.a, self.n, self.pos, self.nmerged):  # removal
                del lst[j]
        self.t += 1
        return o, ev_slot, ev_pos

    def prefill(self, Q, Kp, Vp):
        """Bulk prefill of the empty cache with a prompt (lists of d-lists).  Reading (the paper
        has no such procedure): causal attention over the uncompressed prompt, the scores that
        Algorithm 1's bookkeeping would accumulate over those rows, then selection and merge
        repeated until m entries remain, with no attention in between; merged rows are rounded to
        the cache format once, when the compression is over.
        Returns (outputs, removed tokens in order)."""
        assert self.t == 0
        d, P = self.d, len(Q)
        outs = []
        for t in range(P):
            self.K.append(list(Kp[t])); self.V.append(list(Vp[t]))
            self.pos.append(t); self.nmerged.append(1)
            s = [sum(Q[t][c] * self.K[i][c] for c in range(d)) / math.sqrt(d) for i in range(t + 1)]
            mx = max(s)
            e = [math.exp(x - mx) for x in s]
            S = sum(e)
            A = [x / S for x in e]
            outs.append([sum(A[i] * self.V[i][c] for i in range(t + 1)) for c in range(d)])
            self.a = [x + y for x, y in zip(self.a + [0.0], A)]
            self.n = [x + 1 for x in self.n + [0]]
        removed = []
        while len(self.K) > self.m:
            L = len(self.K)
            abar = [self.a[i] / self.n[i] for i in range(L)]
            j = min(range(self.n_sink, L - self.R), key=lambda i: (abar[i], i))
            if self.merge:
                den = abar[j] + abar[j + 1]
                merged = [(abar[j] * self.V[j][c] + abar[j + 1] * self.V[j + 1][c]) / den if den > 0
                          else 0.5 * self.V[j][c] + 0.5 * self.V[j + 1][c] for c in range(d)]
                self.V[j + 1] = merged                                   # not rounded: never stored as such
                self.nmerged[j + 1] += self.nmerged[j]
            removed.append(self.pos[j])
            for lst in (self.K, self.V, self.a, self.n, self.pos, self.nmerged):
                del lst[j]
        if self.rounder is not None:                                     # rows enter the cache: one rounding
            self.V = [[self.rounder(x) for x in row] for row in self.V]
        self.t = P
        return outs, removed
