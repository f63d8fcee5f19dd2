"""TEST INFRASTRUCTURE ONLY -- the "ideal merging" of the paper's Section III-B.

Dropping k_1 while keeping k_2 leaves the attention output of the current query
unchanged if v_1, v_2 are replaced by one vector v~ (Section III-B solves the
output equality for it).  The method does not execute this formula (it costs
O(t d) per step); it motivates the convex merge.  Here it serves two purposes:
the identity is an independent check of the oracle's attention conventions
(softmax over keys, 1/sqrt(d) scale, row/column layout), and the diagnostic
below compares merge, eviction and full attention on synthetic streams.
"""
import math

import numpy as np


def ideal_merge(q, K, V):
    """v~ for the first two positions of K, V ([t, d] arrays, t >= 2), query q ([d])."""
    q = np.asarray(q, np.float64); K = np.asarray(K, np.float64); V = np.asarray(V, np.float64)
    d = K.shape[1]
    s = K @ q / math.sqrt(d)
    e = np.exp(s - s.max())                 # a common shift cancels in every ratio below
    S = e.sum()
    ratio = e[0] / e[1]                     # e^{q.(k_1 - k_2)/sqrt(d)}
    rest = (e[2:, None] * V[2:]).sum(0)     # the O(t d) term the method drops
    return (1.0 - e[0] / S) * (ratio * V[0] + V[1]) - (ratio / S) * rest


def single_step_merge(q, K, V):
    """The convex approximation of Section III-B: weights are this step's two exponentials."""
    q = np.asarray(q, np.float64); K = np.asarray(K, np.float64); V = np.asarray(V, np.float64)
    s = K[:2] @ q / math.sqrt(K.shape[1])
    e = np.exp(s - s.max())
    return (e[0] * V[0] + e[1] * V[1]) / (e[0] + e[1])
