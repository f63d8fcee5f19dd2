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
    parity.check_outputs(ref * (1 + 1.9e-3), ref, "fp16")
    with pytest.raises(AssertionError):
        parity.check_outputs(ref * (1 + 3e-3), ref, "fp16")
    parity.check_outputs(ref + np.array([[0, 1.5e-5, 0]]), ref, "fp16")     # near-cancelling element
    with pytest.raises(AssertionError):
        parity.check_outputs(ref * (1 + 2e-5), ref, "fp32")
    assert parity.exact_fraction(np.float16(ref).astype(np.float64), ref, "fp16") == 1.0
