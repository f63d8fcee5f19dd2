"""Pins of the CPU oracle against things other than itself.

Each test names what fixes the expected value: a number the paper prints, a
closed form, a textbook/library routine, an invariant, or the separately
written list-based brute-force simulator.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

import oracle
from oracle.brute import BruteUnit


def rng(seed):
    return np.random.default_rng(seed)


def rand_stream(seed, n, units, d, dtype=np.float32):
    g = rng(seed)
    return (g.standard_normal((n, units, d)).astype(dtype),
            g.standard_normal((n, units, d)).astype(dtype),
            g.standard_normal((n, units, d)).astype(dtype))


def parse_golden(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        out[key] = vals
    return out


# --------------------------------------------------------------------------
# number formats: pinned to numpy's / torch's own conversions
# --------------------------------------------------------------------------
def test_round_fp16_matches_numpy():
    g = rng(1)
    xs = np.concatenate([
        g.standard_normal(4000) * np.exp(g.uniform(-20, 12, 4000)),
        [0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e-8, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25,
         2.0 ** -14, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -30],
    ])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).astype(np.float64)
    got = np.array([oracle.round_storage(x, "fp16") for x in xs])
    assert np.array_equal(got, want)


def test_round_bf16_matches_torch():
    g = rng(2)
    # fp32-representable inputs, so torch's conversion cannot double-round
    xs = (g.standard_normal(4000) * np.exp(g.uniform(-30, 30, 4000))).astype(np.float32)
    want = torch.from_numpy(xs).to(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([oracle.round_storage(float(x), "bf16") for x in xs])
    assert np.array_equal(got, want)
    # exact ties and a just-above-tie in fp64 (8 significand bits)
    assert oracle.round_storage(1.0 + 2.0 ** -8, "bf16") == 1.0            # tie -> even
    assert oracle.round_storage(1.0 + 3 * 2.0 ** -8, "bf16") == 1.0 + 2.0 ** -6
    assert oracle.round_storage(1.0 + 2.0 ** -8 + 2.0 ** -40, "bf16") == 1.0 + 2.0 ** -7


def test_round_fp32_matches_numpy():
    g = rng(3)
    xs = g.standard_normal(4000) * np.exp(g.uniform(-60, 60, 4000))
    want = xs.astype(np.float32).astype(np.float64)
    got = np.array([oracle.round_storage(x, "fp32") for x in xs])
    assert np.array_equal(got, want)
    assert oracle.round_storage(1.2345678901234567, "fp64") == 1.2345678901234567


# --------------------------------------------------------------------------
# attention: pinned to library softmax (Section III-A definition, III-B scale)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("L,d", [(1, 8), (7, 16), (65, 64), (300, 128)])
def test_attend_matches_library_softmax(L, d):
    g = rng(10 + L)
    q, K, V = g.standard_normal(d), g.standard_normal((L, d)) * 2, g.standard_normal((L, d))
    o, p = oracle.attend(q, K, V)
    p_ref = scipy.special.softmax(K @ q / math.sqrt(d))
    assert np.allclose(p, p_ref, rtol=1e-13, atol=0)
    assert abs(p.sum() - 1) < 1e-14
    tq, tK, tV = (torch.from_numpy(x) for x in (q, K, V))
    o_ref = (torch.softmax(tK @ tq / math.sqrt(d), dim=0) @ tV).numpy()
    assert np.allclose(o, o_ref, rtol=1e-12, atol=1e-14)


def test_attend_is_not_transposed_or_unscaled():
    # a hand-computable case: d=4, two keys; logits (q.k)/2 = 1 and 0
    q = np.array([1.0, 1.0, 0.0, 0.0])
    K = np.array([[2.0, 0.0, 5.0, 5.0], [0.0, 0.0, 7.0, 7.0]])
    V = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0]])
    o, p = oracle.attend(q, K, V)
    e = math.e
    assert np.allclose(p, [e / (1 + e), 1 / (1 + e)], rtol=1e-15)
    assert np.allclose(o, [e / (1 + e), 1 / (1 + e), 0, 0], rtol=1e-15)


def test_budget_at_least_stream_is_full_attention():
    n, U, d = 40, 3, 16
    q, k, v = rand_stream(20, n, U, d)
    orc = oracle.Oracle(U, d, m=n, R=1)
    res = orc.run(q, k, v)
    assert (res["evict_pos"] == -1).all() and (res["evict_slot"] == -1).all()
    for t in range(n):
        for u in range(U):
            K = k[: t + 1, u].astype(np.float64); V = v[: t + 1, u].astype(np.float64)
            p = scipy.special.softmax(K @ q[t, u].astype(np.float64) / math.sqrt(d))
            assert np.allclose(res["out"][t, u], p @ V, rtol=1e-12, atol=1e-14)
    # the score lists of an uncompressed cache: column sums of the causal attention matrix
    st = orc.state(0)
    A = np.zeros((n, n))
    for t in range(n):
        K = k[: t + 1, 0].astype(np.float64)
        A[t, : t + 1] = scipy.special.softmax(K @ q[t, 0].astype(np.float64) / math.sqrt(d))
    assert np.allclose(st["a"], A.sum(0), rtol=1e-12)
    assert np.array_equal(st["n"], n - np.arange(n))


# --------------------------------------------------------------------------
# the paper's worked example (Section IV)
# --------------------------------------------------------------------------
def test_worked_example_weights(golden_dir):
    gold = parse_golden(os.path.join(golden_dir, "worked_example.txt"))
    sj, sr = float(gold["score_evicted"][0]), float(gold["score_neighbour"][0])
    wj, wr = Fraction(gold["weight_evicted"][0]), Fraction(gold["weight_neighbour"][0])
    d = 5
    Vj, Vr = np.eye(d)[0], np.eye(d)[1]          # basis vectors expose the two weights
    merged = oracle.merge_pair(sj, sr, Vj, Vr)
    assert np.allclose(merged[:2], [float(wj), float(wr)], rtol=1e-15)
    assert np.all(merged[2:] == 0)
    # and the selection picks token 2 (index 1) when its score is the lowest
    j, _ = oracle.select(np.array([0.3, sj, sr, 0.2, 0.9]), 0, 4)
    assert j == int(gold["evicted_token"][0]) - 1


def test_worked_example_end_state(golden_dir):
    """What this pins and what it does not.  Section IV states the end of its toy run: after
    step 8 a cache of 4 holds tokens 3, 6, 7, 8, and the first two hold three raw values each.
    The per-step scores are only in the figure, which is not available, so the arg-mins in
    between cannot be replayed: the removal order used here (tokens 2, 1, 4, 5) is one order
    that is consistent with the stated end, imposed through the forced-choice hook.  The test
    therefore pins the STRUCTURE of merge and removal -- folding into the right-hand neighbour,
    counts of folded values, which keys survive -- and says nothing about the selection."""
    gold = parse_golden(os.path.join(golden_dir, "worked_example.txt"))
    m = int(gold["budget"][0])
    n, d = 8, 8
    g = rng(5)
    q = g.standard_normal((n, 1, d)).astype(np.float32)
    k = g.standard_normal((n, 1, d)).astype(np.float32)
    v = np.eye(n, d, dtype=np.float32)[:, None, :]          # one-hot values
    forced = np.full((n, 1), -1, np.int32)
    forced[4:, 0] = [1, 0, 3, 4]                              # 0-based tokens 2, 1, 4, 5
    orc = oracle.Oracle(1, d, m=m, R=1)
    res = orc.run(q, k, v, forced_pos=forced)
    assert list(res["evict_pos"][4:, 0]) == [1, 0, 3, 4]
    st = orc.state(0)
    assert [p + 1 for p in st["pos"]] == [int(x) for x in gold["final_tokens"]]
    assert list(st["nmerged"]) == [int(x) for x in gold["final_merged_counts"]]
    # slot "3" is a convex combination of raw values 1..3, slot "6" of 4..6
    V = st["V"]
    assert np.all(V >= 0) and np.allclose(V.sum(1), 1, rtol=1e-14)
    assert np.all(V[0, 3:] == 0) and np.all(V[0, :3] > 0)
    assert np.all(V[1, :3] == 0) and np.all(V[1, 6:] == 0) and np.all(V[1, 3:6] > 0)


# --------------------------------------------------------------------------
# selection: tie-break, protected regions, closed forms
# --------------------------------------------------------------------------
def test_select_ties_go_to_oldest_and_runner_up():
    j, ru = oracle.select(np.array([0.5, 0.25, 0.25, 0.75]), 0, 4)
    assert (j, ru) == (1, 0.25)
    j, ru = oracle.select(np.array([0.5, 0.25, 0.1, 0.75, 0.01]), 0, 4)   # hi excludes index 4
    assert (j, ru) == (2, 0.25)
    j, ru = oracle.select(np.array([0.0, 0.25, 0.1]), 1, 3)               # lo excludes index 0
    assert (j, ru) == (2, 0.25)
    j, ru = oracle.select(np.array([0.3]), 0, 1)
    assert j == 0 and math.isinf(ru)


@pytest.mark.parametrize("m,R", [(4, 4), (7, 7), (16, 16)])
def test_recent_window_equal_to_budget_is_a_fifo_fold(m, R):
    """R = m leaves logical slot 0 as the only candidate: the choice no longer
    depends on any score.  evict_slot = 0 and evict_pos = t - m for t >= m."""
    n, d = 60, 8
    q, k, v = rand_stream(30 + m, n, 2, d)
    res = oracle.Oracle(2, d, m, R).run(q, k, v)
    t = np.arange(n)[:, None]
    assert np.array_equal(res["evict_slot"], np.where(t >= m, 0, -1) * np.ones((1, 2), int))
    assert np.array_equal(res["evict_pos"], np.where(t >= m, t - m, -1) * np.ones((1, 2), int))


@pytest.mark.parametrize("m,R", [(8, 1), (8, 3), (15, 4), (31, 8)])
def test_zero_query_closed_form(m, R):
    """q = 0 makes every attention row uniform, p_i = 1/L.  Then a token's average
    score strictly decreases with its birth step, so the youngest candidate is
    evicted each time: evict_pos = t - R, evict_slot = m - R, and outputs are the
    plain mean of the slot values."""
    n, d = 3 * m + 5, 8
    _, k, v = rand_stream(40 + m, n, 1, d)
    q = np.zeros_like(k)
    orc = oracle.Oracle(1, d, m, R)
    res = orc.run(q, k, v)
    t = np.arange(n)
    assert np.array_equal(res["evict_pos"][:, 0], np.where(t >= m, t - R, -1))
    assert np.array_equal(res["evict_slot"][:, 0], np.where(t >= m, m - R, -1))
    # closed-form score sums: a token born at b has a = sum_{tau=b}^{t} 1/min(tau+1, m+1)
    st = orc.state(0)
    T = n
    for a, nn, b in zip(st["a"], st["n"], st["pos"]):
        want = sum(Fraction(1, min(tau + 1, m + 1)) for tau in range(b, T))
        assert abs(a - float(want)) < 1e-13
        assert nn == T - b
    # step 0..m-1 outputs: mean of v[0..t]
    for tt in range(m):
        assert np.allclose(res["out"][tt, 0], v[: tt + 1, 0].astype(np.float64).mean(0), rtol=1e-12,
                           atol=1e-14)


def test_recent_window_one_is_algorithm_as_printed():
    """With R = 1 the candidate set is {0..m-1} of the m+1 slots."""
    n, d, m = 50, 8, 6
    q, k, v = rand_stream(50, n, 1, d)
    res = oracle.Oracle(1, d, m, 1).run(q, k, v)
    ev = res["evict_slot"][m:, 0]
    assert ev.min() >= 0 and ev.max() <= m - 1
    assert (res["evict_pos"][m:, 0] < np.arange(m, n)).all()     # never the token just appended


def test_sink_protection():
    n, d, m, R, ns = 80, 8, 10, 3, 4
    q, k, v = rand_stream(51, n, 2, d)
    orc = oracle.Oracle(2, d, m, R, n_sink=ns)
    res = orc.run(q, k, v)
    assert (res["evict_pos"][m:] >= ns).all()
    for u in range(2):
        assert list(orc.state(u)["pos"][:ns]) == list(range(ns))


# --------------------------------------------------------------------------
# invariants that hold for any stream
# --------------------------------------------------------------------------
@pytest.mark.parametrize("m,R,storage", [(5, 1, "fp64"), (9, 4, "fp64"), (12, 12, "fp16"), (6, 2, "bf16")])
def test_invariants(m, R, storage):
    n, U, d = 70, 3, 80          # d >= n so one-hot values expose merge coefficients
    g = rng(60 + m)
    q = g.standard_normal((n, U, d)).astype(np.float32)
    k = g.standard_normal((n, U, d)).astype(np.float32)
    v = np.broadcast_to(np.eye(n, d, dtype=np.float32)[:, None, :], (n, U, d)).copy()
    orc = oracle.Oracle(U, d, m, R, storage=storage)
    evicted_mass = np.zeros(U)
    for t in range(n):                       # one token per call: state visible after every step
        res = orc.run(q[t:t + 1], k[t:t + 1], v[t:t + 1])
        for u in range(U):
            st = orc.state(u)
            T = t + 1
            assert orc.length(u) == min(T, m)                       # cache holds min(T, m) slots
            assert np.all(np.diff(st["pos"]) > 0)                    # order of tokens preserved
            assert st["pos"][-1] == t                                # newest token always kept
            assert np.array_equal(st["n"], T - st["pos"])            # n_i = t - pos_i + 1
            assert st["nmerged"].sum() == T                          # every raw value is somewhere
            if res["evict_pos"][0, u] >= 0:
                evicted_mass[u] += res["evict_score"][0, u] * (T - res["evict_pos"][0, u])
            # every softmax row sums to 1: live + discarded score mass = tokens processed
            assert abs(st["a"].sum() + evicted_mass[u] - T) < 1e-10
            # each slot is a convex combination of the contiguous run of raw values ending at pos
            V = st["V"][:, :n]
            tol = 0 if storage == "fp64" else 2.0 ** -7
            assert np.all(V >= 0)
            assert np.allclose(V.sum(1), 1, rtol=0, atol=max(tol, 1e-14))
            start = 0
            for row, p_, cnt in zip(V, st["pos"], st["nmerged"]):
                assert p_ - cnt + 1 == start
                assert np.all(row[:start] == 0) and np.all(row[p_ + 1:] == 0)
                start = p_ + 1
            # the output is a convex combination of slot values: coefficients sum to 1
            assert abs(res["out"][0, u, :n].sum() - 1) < max(tol, 1e-12)


def test_constant_values_stay_constant():
    n, d, m, R = 64, 8, 7, 2
    q, k, _ = rand_stream(70, n, 2, d)
    c = rng(71).standard_normal(d).astype(np.float32)
    v = np.broadcast_to(c, (n, 2, d)).copy()
    orc = oracle.Oracle(2, d, m, R)
    res = orc.run(q, k, v)
    assert np.allclose(res["out"], c.astype(np.float64), rtol=1e-13, atol=1e-15)
    assert np.allclose(orc.state(1)["V"], c.astype(np.float64), rtol=1e-13, atol=1e-15)


def test_merge_weights_are_the_two_average_scores():
    """First compression of a stream: the merged row must equal
    (abar_j V_j + abar_r V_r) / (abar_j + abar_r) with abar taken from an uncompressed
    run of the same stream (which the full-attention pin already covers)."""
    n, d, m = 9, 16, 8
    q, k, v = rand_stream(80, n, 1, d)
    full = oracle.Oracle(1, d, m=n, R=1); full.run(q, k, v)
    sf = full.state(0)
    abar = sf["a"] / sf["n"]
    j = int(np.argmin(abar[:m]))
    orc = oracle.Oracle(1, d, m, 1)
    res = orc.run(q, k, v)
    assert res["evict_slot"][-1, 0] == j and res["evict_pos"][-1, 0] == j
    assert res["evict_score"][-1, 0] == abar[j]
    st = orc.state(0)
    want = (abar[j] * sf["V"][j] + abar[j + 1] * sf["V"][j + 1]) / (abar[j] + abar[j + 1])
    assert np.allclose(st["V"][j], want, rtol=1e-14)
    lo, hi = np.minimum(sf["V"][j], sf["V"][j + 1]), np.maximum(sf["V"][j], sf["V"][j + 1])
    assert np.all(st["V"][j] >= lo - 1e-15) and np.all(st["V"][j] <= hi + 1e-15)
    # survivor keeps its own key, score sum and count; evicted score is discarded
    assert np.array_equal(st["K"][j], sf["K"][j + 1])
    assert st["a"][j] == sf["a"][j + 1] and st["n"][j] == sf["n"][j + 1]
    assert np.array_equal(np.delete(sf["a"], j), st["a"])


def test_zero_denominator_is_a_reading_and_both_implementations_take_it():
    """Both averages zero: the merge formula of Algorithm 1 is 0/0 there and the paper says nothing.
    The reading taken (weights 1/2, 1/2) is NOT a fact the paper or the mathematics fixes; this test
    only makes sure that the branch does what the reading says, in the C oracle and in the
    separately written simulator alike, and that it is reached the way a real stream reaches it:
    through scores that underflow to exactly 0 (keys that point away from every query)."""
    # the primitive: 0, 0 -> the plain mean; anything positive -> the convex combination
    a, b = np.array([1.0, -2.0, 8.0]), np.array([3.0, 6.0, -8.0])
    assert np.array_equal(oracle.merge_pair(0.0, 0.0, a, b), 0.5 * a + 0.5 * b)
    assert np.array_equal(oracle.merge_pair(0.0, 2.0, a, b), b)
    assert np.allclose(oracle.merge_pair(1.0, 3.0, a, b), 0.25 * a + 0.75 * b, rtol=1e-15)
    # a stream: tokens 1 and 2 carry keys opposite to every query, scaled so that their softmax
    # weights are exp(-1e4) = 0 in fp64 at every step; everything else attends normally
    d, m, T = 8, 5, 9
    g = np.random.default_rng(5)
    base = np.zeros(d); base[0] = 1.0
    q = np.tile(base * 100.0, (T, 1, 1)).astype(np.float64)              # [T, units=1, d]
    k = g.standard_normal((T, 1, d)) * 0.01
    k[:, 0, 0] = np.abs(k[:, 0, 0])
    k[1, 0] = -base * 300.0; k[2, 0] = -base * 300.0                      # logit -30000/sqrt(8) against ~0
    v = g.standard_normal((T, 1, d))
    q, k, v = (x.astype(np.float32) for x in (q, k, v))                  # what both sides are given
    orc = oracle.Oracle(1, d, m, 1)
    res = orc.run(q[:m + 1], k[:m + 1], v[:m + 1])                        # up to and including the first compression
    # token 0 collects all the mass of step 0; tokens 1 and 2 never collect any: average 0, the lowest,
    # ties to the oldest -> token 1 goes first and folds into token 2 with weights 1/2, 1/2
    assert res["evict_pos"][m, 0] == 1 and res["evict_score"][m, 0] == 0.0
    st = orc.state(0)
    assert list(st["pos"]) == [0, 2, 3, 4, 5]
    assert np.array_equal(st["V"][1], 0.5 * v[1, 0].astype(np.float64) + 0.5 * v[2, 0].astype(np.float64))
    assert st["a"][1] == 0.0                                              # the survivor keeps its own (zero) mass
    res2 = orc.run(q[m + 1:], k[m + 1:], v[m + 1:])                       # token 2 goes next, the same way
    assert res2["evict_pos"][0, 0] == 2 and res2["evict_score"][0, 0] == 0.0
    st = orc.state(0)
    from oracle import brute
    sim = brute.BruteUnit(d, m, 1)
    for t in range(T):
        sim.step([float(x) for x in q[t, 0]], [float(x) for x in k[t, 0]], [float(x) for x in v[t, 0]])
    assert list(sim.pos) == list(st["pos"])
    assert np.allclose(np.array(sim.V), st["V"], rtol=1e-12, atol=1e-14)


def test_storage_rounding_of_merged_rows():
    n, d, m = 80, 16, 6
    q, k, v = rand_stream(90, n, 1, d, np.float16)
    q, k, v = (x.astype(np.float32) for x in (q, k, v))
    for storage, conv in (("fp16", lambda x: x.astype(np.float16).astype(np.float64)),
                          ("fp32", lambda x: x.astype(np.float32).astype(np.float64))):
        orc = oracle.Oracle(1, d, m, 2, storage=storage); orc.run(q, k, v)
        V = orc.state(0)["V"]
        assert np.array_equal(conv(V), V)
    exact = oracle.Oracle(1, d, m, 2); exact.run(q, k, v)
    assert not np.array_equal(exact.state(0)["V"].astype(np.float16).astype(np.float64),
                              exact.state(0)["V"])


# --------------------------------------------------------------------------
# brute force on tiny inputs: the list simulator and the C oracle agree exactly
# --------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(4))
def test_c_oracle_equals_list_simulator(seed):
    """Every budget up to 6, every window, with and without a protected first token, for
    WeightedKV (rule 0 with the merge), its eviction-only ablation, and the accumulated-score
    and latest-weight eviction rules of Section II (rules 1 and 2, which never merge)."""
    g = rng(100 + seed)
    cases = 0
    for m in (1, 2, 3, 5, 6):
        for R in range(1, m + 1):
            for ns in (0, 1):
                if ns + R > m:
                    continue
                for rule, merge in ((0, True), (0, False), (1, False), (2, False)):
                    d = int(g.integers(1, 9)); n = int(g.integers(m + 1, 41))
                    q, k, v = (g.standard_normal((n, 1, d)).astype(np.float32) for _ in range(3))
                    orc = oracle.Oracle(1, d, m, R, n_sink=ns, score_mode=rule, merge_mode=0 if merge else 1)
                    res = orc.run(q, k, v)
                    bu = BruteUnit(d, m, R, n_sink=ns, merge=merge, rule=rule)
                    for t in range(n):
                        o, es, ep = bu.step([float(x) for x in q[t, 0]], [float(x) for x in k[t, 0]],
                                            [float(x) for x in v[t, 0]])
                        assert es == res["evict_slot"][t, 0] and ep == res["evict_pos"][t, 0], (m, R, ns, rule, t)
                        assert np.allclose(o, res["out"][t, 0], rtol=1e-12, atol=1e-14)
                    st = orc.state(0)
                    assert list(st["pos"]) == bu.pos and list(st["n"]) == bu.n
                    assert list(st["nmerged"]) == bu.nmerged
                    assert np.allclose(st["a"], bu.a, rtol=1e-12)
                    assert np.allclose(st["V"], np.array(bu.V), rtol=1e-12, atol=1e-14)
                    assert np.array_equal(st["K"], np.array(bu.K))
                    cases += 1
    assert cases == 116


@pytest.mark.parametrize("rule", [1, 2])
def test_eviction_rules_every_step_against_an_uncompressed_run_of_the_survivors(rule):
    """The accumulated-score and latest-weight rules, pinned at EVERY compression of a stream and
    not only the first: whatever was evicted before, the scores of the tokens still alive are
    functions of the keys still alive.  So replay the stream keeping, by hand, exactly the
    oracle's survivors, compute each step's attention row with the library softmax, accumulate
    it per token, and the victim must be the arg-min (ties to the oldest) over the unprotected."""
    n, d, m, R, sink = 60, 8, 7, 2, 1
    q, k, v = rand_stream(410 + rule, n, 1, d)
    res = oracle.Oracle(1, d, m, R, n_sink=sink, score_mode=rule, merge_mode=1).run(q, k, v)
    alive, mass = [], {}
    for t in range(n):
        alive.append(t); mass[t] = 0.0
        p = scipy.special.softmax(k[alive, 0].astype(np.float64) @ q[t, 0].astype(np.float64) / math.sqrt(d))
        for tok, w in zip(alive, p):
            mass[tok] += w
        if len(alive) > m:
            free = alive[sink:len(alive) - R]
            score = {tok: (mass[tok] if rule == 1 else p[alive.index(tok)]) for tok in free}
            expect = min(free, key=lambda tok: (score[tok], tok))
            assert res["evict_pos"][t, 0] == expect, t
            assert math.isclose(res["evict_score"][t, 0], score[expect], rel_tol=1e-12)
            alive.remove(expect)
        else:
            assert res["evict_pos"][t, 0] == -1


def test_list_simulator_storage_rounding_agrees():
    g = rng(200)
    d, m, R, n = 6, 4, 2, 30
    q, k, v = (g.standard_normal((n, 1, d)).astype(np.float16).astype(np.float32) for _ in range(3))
    orc = oracle.Oracle(1, d, m, R, storage="fp16"); res = orc.run(q, k, v)
    bu = BruteUnit(d, m, R, rounder=lambda x: float(np.float16(x)))
    for t in range(n):
        _, es, ep = bu.step(*[[float(x) for x in a[t, 0]] for a in (q, k, v)])
        assert ep == res["evict_pos"][t, 0]
    assert np.array_equal(orc.state(0)["V"], np.array(bu.V))


# --------------------------------------------------------------------------
# forced choices (near-tie classification support)
# --------------------------------------------------------------------------
def test_forced_choice_reports_scores_and_rejects_protected_tokens():
    n, d, m, R = 12, 8, 6, 2
    q, k, v = rand_stream(300, n, 1, d)
    free = oracle.Oracle(1, d, m, R).run(q, k, v)
    t0 = m
    own = free["evict_pos"][t0, 0]
    other = next(p for p in range(0, t0 + 1 - R) if p != own)
    forced = np.full((n, 1), -1, np.int32); forced[t0, 0] = other
    res = oracle.Oracle(1, d, m, R).run(q, k, v, forced_pos=forced)
    assert res["evict_pos"][t0, 0] == other
    assert res["evict_score"][t0, 0] == free["evict_score"][t0, 0]
    assert res["forced_score"][t0, 0] >= res["evict_score"][t0, 0]
    forced[t0, 0] = t0                                    # the token just appended: protected
    with pytest.raises(RuntimeError):
        oracle.Oracle(1, d, m, R).run(q, k, v, forced_pos=forced)


def test_eviction_baseline_variants():
    """merge_mode 1 (the ablation of Section V-B) keeps selection identical as long as
    scores are identical, and leaves values untouched."""
    n, d, m, R = 40, 8, 6, 2
    q, k, v = rand_stream(400, n, 1, d)
    a = oracle.Oracle(1, d, m, R).run(q, k, v)
    orc = oracle.Oracle(1, d, m, R, merge_mode=1)
    b = orc.run(q, k, v)
    assert np.array_equal(a["evict_pos"], b["evict_pos"])      # scores depend on q,K only
    st = orc.state(0)
    assert np.array_equal(st["V"], v[st["pos"], 0].astype(np.float64))
    assert (st["nmerged"] == 1).all()
    with pytest.raises(ValueError):
        oracle.Oracle(1, d, m, R, score_mode=1, merge_mode=0)
    # cumulative-score rule: victim = arg-min of a over candidates of an uncompressed run
    full = oracle.Oracle(1, d, m + 1, 1); full.run(q[: m + 1], k[: m + 1], v[: m + 1])
    h2o = oracle.Oracle(1, d, m, R, score_mode=1, merge_mode=1).run(q[: m + 1], k[: m + 1], v[: m + 1])
    assert h2o["evict_slot"][m, 0] == int(np.argmin(full.state(0)["a"][: m + 1 - R]))
    # last-step rule: victim = arg-min of the current attention row over candidates
    p = scipy.special.softmax(k[: m + 1, 0].astype(np.float64) @ q[m, 0].astype(np.float64) / math.sqrt(d))
    tova = oracle.Oracle(1, d, m, R, score_mode=2, merge_mode=1).run(q[: m + 1], k[: m + 1], v[: m + 1])
    assert tova["evict_slot"][m, 0] == int(np.argmin(p[: m + 1 - R]))


# --------------------------------------------------------------------------
# the ideal-merge identity of Section III-B: an independent check of the attention conventions
# --------------------------------------------------------------------------
@pytest.mark.parametrize("t,d", [(2, 4), (5, 8), (40, 64)])
def test_ideal_merge_leaves_the_output_unchanged(t, d):
    from oracle.ideal import ideal_merge, single_step_merge
    g = rng(500 + t)
    q, K, V = g.standard_normal(d), g.standard_normal((t, d)) * 1.5, g.standard_normal((t, d))
    o_full, _ = oracle.attend(q, K, V)
    v_tilde = ideal_merge(q, K, V)
    o_merged, _ = oracle.attend(q, K[1:], np.vstack([v_tilde[None], V[2:]]))
    assert np.allclose(o_merged, o_full, rtol=1e-11, atol=1e-13)
    # the practical approximation is a convex combination of v_1, v_2 and is *not* exact
    approx = single_step_merge(q, K, V)
    lo, hi = np.minimum(V[0], V[1]), np.maximum(V[0], V[1])
    assert np.all(approx >= lo - 1e-15) and np.all(approx <= hi + 1e-15)
    if t > 2:
        o_approx, _ = oracle.attend(q, K[1:], np.vstack([approx[None], V[2:]]))
        assert not np.allclose(o_approx, o_full, rtol=1e-9, atol=1e-12)


# ---------------------------------------------------------------------------
# bulk prefill (a reading: the paper only streams; see the oracle's comment)
# ---------------------------------------------------------------------------
def _prompt(seed, P, units, d, dtype=np.float16):
    g = rng(seed)
    return tuple(g.standard_normal((P, units, d)).astype(dtype).astype(np.float32) for _ in range(3))


@pytest.mark.parametrize("P,m", [(1, 4), (7, 7), (12, 20), (21, 20)])
def test_prefill_equals_streaming_while_nothing_or_one_token_is_evicted(P, m):
    """For P <= m nothing is compressed; for P = m + 1 the single compression comes after the last
    row's attention in both procedures.  There the bulk reading and Algorithm 1 must agree."""
    q, k, v = _prompt(40 + P, P, 3, 16)
    a = oracle.Oracle(3, 16, m, 2, "fp16"); b = oracle.Oracle(3, 16, m, 2, "fp16")
    ra = a.prefill(q, k, v); rb = b.run(q, k, v)
    np.testing.assert_allclose(ra["out"], rb["out"], rtol=0, atol=1e-13)
    if P > m:
        assert np.array_equal(ra["evict_pos"][0], rb["evict_pos"][-1])
    for u in range(3):
        sa, sb = a.state(u), b.state(u)
        assert a.tokens(u) == b.tokens(u) == P
        for key in ("pos", "n", "nmerged"):
            assert np.array_equal(sa[key], sb[key]), key
        np.testing.assert_allclose(sa["a"], sb["a"], rtol=1e-13)
        np.testing.assert_allclose(sa["V"], sb["V"], rtol=0, atol=1e-13)
        assert np.array_equal(sa["K"], sb["K"])


def test_prefill_rows_are_causal_library_attention_and_scores_are_its_column_sums():
    P, d, m = 37, 32, 64
    q, k, v = _prompt(51, P, 1, d, np.float32)
    o = oracle.Oracle(1, d, m, 1)
    r = o.prefill(q, k, v)
    S = (q[:, 0].astype(np.float64) @ k[:, 0].astype(np.float64).T) / math.sqrt(d)
    S[np.triu_indices(P, 1)] = -np.inf
    A = scipy.special.softmax(S, axis=1)
    np.testing.assert_allclose(r["out"][:, 0], A @ v[:, 0].astype(np.float64), rtol=0, atol=1e-12)
    st = o.state(0)
    np.testing.assert_allclose(st["a"], A.sum(axis=0), rtol=1e-12)
    assert math.isclose(st["a"].sum(), P, rel_tol=1e-12)            # every row sums to one
    assert np.array_equal(st["n"], P - np.arange(P))                 # rows that attended token i
    assert r["evict_pos"].shape == (0, 1)


@pytest.mark.parametrize("rule,merge", [(0, True), (0, False), (1, False)])
@pytest.mark.parametrize("seed,P,m,R,sink,storage", [(0, 30, 8, 2, 0, "fp64"), (1, 45, 11, 1, 0, "fp16"),
                                                      (2, 64, 16, 5, 3, "bf16"), (3, 25, 24, 24, 0, "fp64"),
                                                      (4, 50, 3, 1, 2, "fp16")])
def test_prefill_equals_list_simulator(seed, P, m, R, sink, storage, rule, merge):
    d = 8
    q, k, v = _prompt(60 + seed, P, 1, d)
    o = oracle.Oracle(1, d, m, R, storage, n_sink=sink, score_mode=rule, merge_mode=0 if merge else 1)
    r = o.prefill(q, k, v)
    rounder = None if storage == "fp64" else (lambda x: oracle.round_storage(x, storage))
    b = BruteUnit(d, m, R, n_sink=sink, rounder=rounder, merge=merge, rule=rule)
    outs, removed = b.prefill(q[:, 0].tolist(), k[:, 0].tolist(), v[:, 0].tolist())
    assert r["evict_pos"][:, 0].tolist() == removed
    np.testing.assert_allclose(r["out"][:, 0], np.array(outs), rtol=0, atol=1e-12)
    st = o.state(0)
    assert st["pos"].tolist() == b.pos and st["nmerged"].tolist() == b.nmerged and st["n"].tolist() == b.n
    np.testing.assert_allclose(st["a"], b.a, rtol=1e-12)
    np.testing.assert_allclose(st["V"], np.array(b.V), rtol=0, atol=1e-12)


def test_prefill_with_accumulated_scores_removes_the_lowest_sums():
    """The accumulated-score rule on a prompt: the sums are the column sums of the causal
    attention matrix (library softmax), they do not change during the compression, so the removed
    tokens are the P - m unprotected tokens of smallest (a, token), in that order; the survivors
    keep their raw values (the rule only evicts)."""
    P, d, m, R, sink = 80, 16, 18, 5, 2
    q, k, v = _prompt(73, P, 2, d)
    o = oracle.Oracle(2, d, m, R, n_sink=sink, score_mode=1, merge_mode=1)
    r = o.prefill(q, k, v)
    for u in range(2):
        S = (q[:, u].astype(np.float64) @ k[:, u].astype(np.float64).T) / math.sqrt(d)
        S[np.triu_indices(P, 1)] = -np.inf
        a = scipy.special.softmax(S, axis=1).sum(axis=0)
        expect = sorted(range(sink, P - R), key=lambda i: (a[i], i))[: P - m]
        assert r["evict_pos"][:, u].tolist() == expect
        np.testing.assert_allclose(r["evict_score"][:, u], a[expect], rtol=1e-12)
        kept = o.state(u)
        assert kept["pos"].tolist() == sorted(set(range(P)) - set(expect))
        np.testing.assert_allclose(kept["a"], a[kept["pos"]], rtol=1e-12)
        assert np.array_equal(kept["V"], v[kept["pos"], u].astype(np.float64))
        # the ranking differs from the average-score one on this prompt, so the test tells them apart
        avg = oracle.Oracle(1, d, m, R, n_sink=sink, merge_mode=1)
        ra = avg.prefill(q[:, u:u + 1], k[:, u:u + 1], v[:, u:u + 1])
        assert ra["evict_pos"][:, 0].tolist() != expect


def test_prefill_removes_the_lowest_average_scores_in_ascending_order():
    """Scores do not change between two merges (the survivor keeps its own a and n), and neither
    does the protected set, so the removed tokens are exactly the P - m unprotected tokens with the
    smallest (abar, token) and they leave in that order."""
    P, d, m, R, sink = 90, 16, 20, 6, 2
    q, k, v = _prompt(71, P, 2, d)
    full = oracle.Oracle(2, d, P, 1); full.prefill(q, k, v)
    o = oracle.Oracle(2, d, m, R, n_sink=sink)
    r = o.prefill(q, k, v)
    for u in range(2):
        st = full.state(u)
        abar = st["a"] / st["n"]
        cand = [i for i in range(sink, P - R)]
        expect = sorted(cand, key=lambda i: (abar[i], i))[: P - m]
        assert r["evict_pos"][:, u].tolist() == expect
        assert np.all(np.diff(r["evict_score"][:, u]) >= 0)
        kept = o.state(u)
        assert sorted(set(range(P)) - set(expect)) == kept["pos"].tolist()
        assert kept["nmerged"].sum() == P                              # every raw value sits in exactly one slot
        assert np.array_equal(kept["n"], P - kept["pos"])
        np.testing.assert_allclose(kept["a"], st["a"][kept["pos"]], rtol=1e-13)   # survivors keep their own sums


def test_prefill_without_merging_keeps_the_survivors_values_and_merging_stays_in_the_hull():
    P, d, m = 40, 8, 10
    q, k, v = _prompt(81, P, 1, d)
    ev = oracle.Oracle(1, d, m, 2, merge_mode=1); ev.prefill(q, k, v)
    st = ev.state(0)
    assert np.array_equal(st["V"], v[st["pos"], 0].astype(np.float64))
    assert np.all(st["nmerged"] == 1)
    mg = oracle.Oracle(1, d, m, 2); mg.prefill(q, k, v)
    sm = mg.state(0)
    assert np.array_equal(sm["pos"], st["pos"])                        # same selection, values differ
    lo = 0
    for slot, p_ in enumerate(sm["pos"]):
        block = v[lo:p_ + 1, 0].astype(np.float64)                     # the run of tokens folded into this slot
        assert np.all(sm["V"][slot] >= block.min(axis=0) - 1e-12) and np.all(sm["V"][slot] <= block.max(axis=0) + 1e-12)
        assert sm["nmerged"][slot] == p_ + 1 - lo
        lo = p_ + 1


def test_prefill_refuses_a_used_cache_and_the_last_step_rule():
    q, k, v = _prompt(91, 5, 1, 8)
    o = oracle.Oracle(1, 8, 4, 1)
    o.run(q[:1], k[:1], v[:1])
    with pytest.raises(RuntimeError):
        o.prefill(q, k, v)
    with pytest.raises(ValueError):
        oracle.Oracle(1, 8, 4, 1, score_mode=2, merge_mode=1).prefill(q, k, v)


def test_streaming_after_prefill_continues_from_the_prefilled_state():
    """A decode step after the prompt sees the compressed cache with the prompt's score sums and
    counts: compare with the list simulator doing the same two calls."""
    P, d, m, R = 30, 8, 12, 3
    q, k, v = _prompt(95, P + 6, 1, d)
    o = oracle.Oracle(1, d, m, R, "fp16")
    o.prefill(q[:P], k[:P], v[:P])
    r = o.run(q[P:], k[P:], v[P:])
    b = BruteUnit(d, m, R, rounder=lambda x: oracle.round_storage(x, "fp16"))
    b.prefill(q[:P, 0].tolist(), k[:P, 0].tolist(), v[:P, 0].tolist())
    for t in range(P, P + 6):
        ob, _, ep = b.step(q[t, 0].tolist(), k[t, 0].tolist(), v[t, 0].tolist())
        np.testing.assert_allclose(r["out"][t - P, 0], ob, rtol=0, atol=1e-12)
        assert r["evict_pos"][t - P, 0] == ep
    assert o.state(0)["pos"].tolist() == b.pos and o.state(0)["n"].tolist() == b.n


# ---------------------------------------------------------------------------
# the single-merge perturbation experiment of Section IV (Fig. 2), on a synthetic stack
# ---------------------------------------------------------------------------
def test_single_merge_perturbation_diagnostic():
    """What the mathematics fixes: before the merge the two runs are the same run (similarity 1);
    in the first layer, whose queries and keys do not depend on earlier outputs, removing a key
    rescales the other weights of a row by one common factor, so the similarity stays 1 after
    the merge too; deeper layers see changed inputs and move, a little."""
    from oracle import diagnostic
    res = diagnostic.single_merge_perturbation(d=16, n_layers=3, merge_at=25, follow=90, seed=3)
    for li, r in res.items():
        assert abs(r["before"] - 1.0) <= 4e-16
        assert r["std"] >= 0 and r["min"] <= r["mean"] <= 1.0 + 1e-15
    assert abs(res[0]["mean"] - 1.0) <= 1e-14 and abs(res[0]["min"] - 1.0) <= 1e-14
    for li in (1, 2):
        assert 0.9 < res[li]["min"] < 1.0 - 1e-9          # perturbed, but still the same attention pattern
