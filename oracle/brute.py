"""TEST INFRASTRUCTURE ONLY -- a token-table simulation of WeightedKV for tiny inputs.

One (sequence, head) unit.  Where the C oracle (wkv_oracle.c) keeps ordered arrays and an
explicit list of counts, this simulator keeps a table keyed by token index: every retained
token owns a record with its key, its (possibly merged) value, the attention mass it has
collected, the step at which it entered and the weight it got in the latest step.  Counts are
not stored: a token that entered at step b has been attended b..t, i.e. t - b + 1 times.
Token order is the order of the table's keys.  Python floats (IEEE double) throughout.

It exists to pin the C oracle: the two are written separately, organised differently, and
must agree on small random streams -- for WeightedKV itself (Algorithm 1, Section IV) and for
the variants around it: dropping the value instead of merging it (the ablation of Section V-B)
and ranking by accumulated mass or by the latest weight (the two eviction rules described in
Section II).

Readings taken where the paper is silent:
  * logits are scaled by 1/sqrt(d) (Section III-B writes the scale, III-A omits it);
  * a step attends over the table *with* the incoming token and *before* anything is removed
    (Algorithm 1 obtains the attention weights ahead of its capacity test);
  * Algorithm 1 spares only the newest token from removal; `R` spares the R newest (R = 1 is
    the algorithm as printed; Section V-A keeps a recent region), `n_sink` the first tokens;
  * equal importance: the oldest token goes;
  * the token that absorbs a value keeps its own key, mass and age (Algorithm 1 removes the
    victim's entries only);
  * both importances zero: the two values are averaged.

Nothing on the product path may import this module.
"""
import math

AVERAGE, CUMULATIVE, LATEST = 0, 1, 2


class Rec:
    __slots__ = ("key", "value", "mass", "born", "folded", "latest")

    def __init__(self, key, value, born):
        self.key, self.value = list(key), list(value)
        self.mass, self.born, self.folded, self.latest = 0.0, born, 1, 0.0


def _softmax_weights(q, keys):
    d = len(q)
    logit = [math.fsum(qc * kc for qc, kc in zip(q, key)) / math.sqrt(d) for key in keys]
    top = max(logit)
    ex = [math.exp(x - top) for x in logit]
    total = sum(ex)
    return [x / total for x in ex]


class BruteUnit:
    def __init__(self, d, m, R, n_sink=0, merge=True, rounder=None, rule=AVERAGE):
        assert 1 <= R <= m and n_sink >= 0 and n_sink + R <= m
        assert rule == AVERAGE or not merge          # the two other rules only evict
        self.d, self.m, self.R = d, m, R
        self.n_sink, self.merge, self.rounder, self.rule = n_sink, merge, rounder, rule
        self.table = {}                  # token index -> Rec; insertion order is token order
        self.t = 0                       # tokens seen

    # ---- views in token order, shaped like the C oracle's state
    def _recs(self):
        return [self.table[tok] for tok in sorted(self.table)]

    pos = property(lambda self: sorted(self.table))
    K = property(lambda self: [r.key for r in self._recs()])
    V = property(lambda self: [r.value for r in self._recs()])
    a = property(lambda self: [r.mass for r in self._recs()])
    n = property(lambda self: [self.t - r.born for r in self._recs()])     # steps attended so far
    nmerged = property(lambda self: [r.folded for r in self._recs()])

    def _importance(self, rec, now):
        """How much a token matters when token `now` has just been attended."""
        if self.rule == AVERAGE:
            return rec.mass / (now - rec.born + 1)       # mass per step attended (Section IV)
        if self.rule == CUMULATIVE:
            return rec.mass                               # accumulated attention (Section II)
        return rec.latest                                 # the latest step's weight (Section II)

    def _shrink(self, now):
        """Remove the least important unprotected token; returns (its rank, its index)."""
        order = sorted(self.table)
        free = order[self.n_sink:len(order) - self.R]
        victim = min(free, key=lambda tok: (self._importance(self.table[tok], now), tok))
        rank = order.index(victim)
        if self.merge:
            heir = self.table[order[rank + 1]]            # the next token in token order
            gone = self.table[victim]
            wg, wh = self._importance(gone, now), self._importance(heir, now)
            if wg + wh > 0:
                mixed = [(wg * x + wh * y) / (wg + wh) for x, y in zip(gone.value, heir.value)]
            else:
                mixed = [0.5 * x + 0.5 * y for x, y in zip(gone.value, heir.value)]
            heir.value = mixed
            heir.folded += gone.folded
        del self.table[victim]
        return rank, victim

    def step(self, q, k, v):
        """One generated token.  Returns (o, rank of the removed token, its index); -1, -1 when
        nothing was removed."""
        now = self.t
        self.table[now] = Rec(k, v, now)
        recs = self._recs()
        w = _softmax_weights(q, [r.key for r in recs])                    # Section III-A
        o = [sum(wi * r.value[c] for wi, r in zip(w, recs)) for c in range(self.d)]
        for wi, r in zip(w, recs):                                        # Algorithm 1's bookkeeping
            r.mass += wi
            r.latest = wi
        rank, victim = -1, -1
        if len(self.table) > self.m:
            rank, victim = self._shrink(now)
            if self.merge and self.rounder is not None and rank < len(self.table):
                heir = self._recs()[rank]
                heir.value = [self.rounder(x) for x in heir.value]        # the row is stored
        self.t += 1
        return o, rank, victim

    def prefill(self, Q, Kp, Vp):
        """A prompt given at once to the empty table (a reading: the paper streams).  Every
        prompt token attends causally over the whole, uncompressed prompt and the masses add up
        as in step(); then tokens are removed, by the same rule with the masses as they stand,
        until m remain.  Values are rounded once, when the removal is over.  The latest-weight
        rule has no meaning here.  Returns (outputs, removed tokens in order)."""
        assert self.t == 0 and self.rule != LATEST
        outs = []
        for now, (q, k, v) in enumerate(zip(Q, Kp, Vp)):
            self.table[now] = Rec(k, v, now)
            recs = self._recs()
            w = _softmax_weights(q, [r.key for r in recs])
            outs.append([sum(wi * r.value[c] for wi, r in zip(w, recs)) for c in range(self.d)])
            for wi, r in zip(w, recs):
                r.mass += wi
        last = len(Q) - 1
        removed = []
        while len(self.table) > self.m:
            removed.append(self._shrink(last)[1])
        if self.rounder is not None:
            for r in self.table.values():
                r.value = [self.rounder(x) for x in r.value]
        self.t = len(Q)
        return outs, removed
