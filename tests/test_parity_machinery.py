"""CPU checks of the comparison machinery the GPU parity tests rely on: tolerance
arithmetic and the near-tie rule (a disagreement in the evicted index is accepted
only when the oracle's own scores of the two candidates are within the threshold,
and the comparison then continues from the other side's choice)."""
import numpy as np
import pytest

import oracle
import parity
from paper_2503_01330_amd import synth


def _fake_gpu_run(cfg, deviate_at=None):
    """Plays the GPU's part with the oracle itself; optionally takes the runner-up at one step."""
    q, k, v = (synth.storage_to_f32(x, cfg.dtype) for x in synth.Stream(cfg).steps(0, cfg.steps))
    free = oracle.Oracle(cfg.units, cfg.head_dim, cfg.budget, cfg.recent, storage=cfg.dtype).run(q, k, v)
    forced = None
    if deviate_at is not None:
        t, u = deviate_at
        # runner-up candidate at (t, u): replay to step t and look at the state
        o = oracle.Oracle(cfg.units, cfg.head_dim, cfg.budget, cfg.recent, storage=cfg.dtype)
        o.run(q[:t], k[:t], v[:t])
        st = o.state(u)
        # candidates after the append of token t are the cached entries outside the window
        cand = st["pos"][: cfg.budget + 1 - cfg.recent]
        other = next(int(p) for p in cand if p != free["evict_pos"][t, u])
        forced = np.full((cfg.steps, cfg.units), -1, np.int32)
        forced[t, u] = other
    res = oracle.Oracle(cfg.units, cfg.head_dim, cfg.budget, cfg.recent, storage=cfg.dtype).run(
        q, k, v, forced_pos=forced)
    return dict(out=res["out"], evict_pos=res["evict_pos"], evict_slot=res["evict_slot"], q=q, k=k, v=v,
                sel=np.arange(cfg.units), cache=None)


CFG = synth.StreamConfig("machinery", 4242, 1, 2, 64, "fp32", 60, 8, 2)


def test_identical_runs_compare_clean():
    stats = parity.compare(CFG, _fake_gpu_run(CFG), check_state=False)
    assert stats["near_ties"] == 0 and stats["out_err"] < 1e-12


def test_a_deviation_beyond_the_threshold_fails():
    g = _fake_gpu_run(CFG, deviate_at=(20, 1))
    with pytest.raises(AssertionError, match="beyond near-tie"):
        parity.compare(CFG, g, check_state=False)


def test_a_deviation_within_the_threshold_is_logged_and_followed(monkeypatch):
    g = _fake_gpu_run(CFG, deviate_at=(20, 1))
    monkeypatch.setattr(parity, "NEAR_TIE", 1e9)       # pretend every gap is a near-tie
    lines = []
    stats = parity.compare(CFG, g, check_state=False, log=lines.append)
    assert stats["near_ties"] == 1 and len(lines) == 1 and "step 20 unit 1" in lines[0]
    assert stats["out_err"] < 1e-12                      # after following, everything matches again


def test_output_tolerance_arithmetic():
    ref = np.array([[1.0, 1e-9, -2.0]])
    with pytest.raises(AssertionError):
        parity.check_outputs(ref * (1 + 3e-3), ref, "fp16")
    parity.check_outputs(ref + np.array([[0, 1.5e-5, 0]]), ref, "fp16")     # near-cancelling element
    with pytest.raises(AssertionError):
        parity.check_outputs(ref * (1 + 2e-5), ref, "fp32")
    assert parity.exact_fraction(np.float16(ref).astype(np.float64), ref, "fp16") == 1.0


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_sixteen_bit_results_must_be_the_rounded_reference_or_its_neighbour(dtype):
    g = np.random.default_rng(11)
    # values in the upper half of their binade, where one step of the format is below the relative bar
    ref = (1.5 + 0.45 * g.random((400, 64))) * 2.0 ** g.integers(-3, 4, (400, 1)) * g.choice([-1.0, 1.0], (400, 64))
    r = parity.round_to_storage(ref, dtype)
    step = 2.0 ** (np.floor(np.log2(np.abs(r))) - (10 if dtype == "fp16" else 7))     # spacing at r
    parity.check_outputs(r, ref, dtype)                                  # the rounded reference itself
    near = ref.copy(); near[::100, ::16] = (r + 0.45 * step)[::100, ::16]      # a few references close to a rounding boundary:
    one = r.copy(); one[::100, ::16] += step[::100, ::16]                # the neighbour beyond the boundary is accepted
    parity.check_outputs(one, near, dtype)                               # (an accumulation error can straddle it) ...
    two = r.copy(); two[3, 4] += 2 * step[3, 4]                          # ... two steps off: not
    with pytest.raises(AssertionError):
        parity.check_outputs(two, ref, dtype)
    pick = g.random(r.shape) < 0.01                                      # the same for 1 % of the elements:
    near = np.where(pick, r + 0.45 * step, ref)                          # each within the bar, together below the exactness floor
    with pytest.raises(AssertionError, match="bit-exact"):
        parity.check_outputs(np.where(pick, r + step, r), near, dtype)


def test_rounding_to_storage_is_a_single_rounding():
    """bf16 from fp64 must not round twice (through fp32): values just above a bf16 tie that
    collapse onto the tie in fp32 show the difference.  Pinned to the oracle's own rounding, which
    the oracle pins tie to torch's and numpy's conversions."""
    g = np.random.default_rng(12)
    x = g.standard_normal(5000) * np.exp(g.uniform(-20, 20, 5000))
    tie = (1.0 + 2.0 ** -8) * 2.0 ** g.integers(-10, 10, 200)           # exact bf16 ties ...
    x = np.concatenate([x, tie, tie * (1 + 2.0 ** -40), tie * (1 - 2.0 ** -40)])   # ... and values a hair off them
    for dtype in ("bf16", "fp16", "fp32"):
        want = np.array([oracle.round_storage(float(v), dtype) for v in x])
        got = parity.round_to_storage(x, dtype)
        keep = np.isfinite(want)
        assert np.array_equal(got[keep], want[keep]), dtype


def test_chunked_comparison_follows_the_other_side_and_classifies_disagreements(monkeypatch):
    g = _fake_gpu_run(CFG, deviate_at=(20, 1))
    def run(chunks):
        orc = oracle.Oracle(CFG.units, CFG.head_dim, CFG.budget, CFG.recent, storage=CFG.dtype)
        lines, near = [], 0
        for lo, hi in chunks:
            r = parity.compare_chunk(orc, CFG, lo, g["q"][lo:hi], g["k"][lo:hi], g["v"][lo:hi], g["out"][lo:hi],
                                     g["evict_pos"][lo:hi], g["evict_slot"][lo:hi], log=lines.append)
            near += r["near_ties"]
        return near, lines
    with pytest.raises(AssertionError, match="beyond near-tie"):
        run([(0, 16), (16, 40), (40, 60)])
    monkeypatch.setattr(parity, "NEAR_TIE", 1e9)
    near, lines = run([(0, 16), (16, 40), (40, 60)])
    assert near == 1 and "step 20 unit 1" in lines[0]
    # a reported victim that is protected (the newest token) is refused outright
    bad = dict(g); bad["evict_pos"] = g["evict_pos"].copy(); bad["evict_pos"][30, 0] = 30
    orc = oracle.Oracle(CFG.units, CFG.head_dim, CFG.budget, CFG.recent, storage=CFG.dtype)
    with pytest.raises(AssertionError, match="not a candidate"):
        parity.compare_chunk(orc, CFG, 0, g["q"], g["k"], g["v"], g["out"], bad["evict_pos"], g["evict_slot"])
