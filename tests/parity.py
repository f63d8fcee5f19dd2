"""Shared machinery of the GPU parity tests: stream a synthetic configuration
through libwkv (via the C ABI binding) and through the CPU oracle, and compare.

Acceptance bars (stated once here, used by every parity test):
  * eviction indices (evicted token, its rank in token order): bit-exact.  A
    disagreement is tolerated only if, in the oracle's own fp64 state, the two
    candidates' scores differ by at most 1e-6 relative; it is then logged and
    the oracle continues from the GPU's choice for that step.
  * retained keys, token positions, counts, merge counts: bit-exact.
  * attention outputs and merged values: |gpu - ref| <= rtol*|ref| + atol_rel*max|ref row|
    with rtol = 2e-3 for fp16 (fp32 accumulation), 2^-8 for bf16 (its unit roundoff, see
    below) and 1e-5 for fp32.  The
    second term covers elements that nearly cancel: the fp32 accumulation error
    is relative to sum_i p_i |V_i|, not to the (possibly tiny) result.
    On top of that, for the 16-bit formats: every element is the reference rounded to the
    format or one of its two neighbours in the format (again up to the cancellation term),
    and, over comparisons of at least 20000 elements, the fraction that equals the rounded
    reference bit for bit is at least EXACT_FLOOR (0.999 for bf16, 0.998 for fp16).
  * score sums a: 1e-9 relative (both sides accumulate in fp64).
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2503_01330_amd import binding as wkv
from paper_2503_01330_amd import synth

# 2e-3 / 1e-5 are the stated targets.  bf16 carries 8 significand bits, so merely
# storing a result in bf16 moves it by up to 2^-8 = 3.9e-3 relative: no bf16 output can
# be within 2e-3 of an unrounded fp64 value element by element.  For bf16 the relative bar is
# therefore the format's own unit roundoff, and what actually constrains a 16-bit result is
# stated in units of the format: it must be the correctly rounded reference or its neighbour
# (the fp32 accumulation error can straddle a rounding boundary, it cannot do more), and the
# share of bit-exact elements has a floor.  Observed shares on an MI355X: bf16 0.99984-0.99992,
# fp16 0.9992-0.9996 (fp16 keeps three more bits, so the same fp32 error straddles a boundary
# eight times as often).
UNIT_ROUNDOFF = {"fp32": 2.0 ** -24, "fp16": 2.0 ** -11, "bf16": 2.0 ** -8}
RTOL = {"fp32": 1e-5, "fp16": 2e-3, "bf16": max(2e-3, 2.0 ** -8)}
ATOL_REL = {"fp32": 1e-6, "fp16": 1e-5, "bf16": 1e-5}
EXACT_FLOOR = {"fp16": 0.998, "bf16": 0.999}
# The bulk prefill forms P.V on the 16-bit matrix cores with the weights cut into 16-bit parts
# (error 2^-22 per weight for fp16, 2^-24 for bf16) instead of fp32 products: a little more of
# its fp16 outputs straddle a rounding boundary (observed 0.9976 on a 4096-token prompt).
PREFILL_EXACT_FLOOR = {"fp16": 0.995, "bf16": 0.999}
EXACT_FLOOR_MIN_ELEMENTS = 20000
NEAR_TIE = 1e-6

_TORCH_VIEW = {"fp32": torch.float32, "fp16": torch.float16, "bf16": torch.bfloat16}


def to_device(x: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(x).cuda()
    return t.view(torch.bfloat16) if dtype == "bf16" else t


def out_to_f64(t: torch.Tensor, dtype: str) -> np.ndarray:
    return t.to(torch.float64).cpu().numpy()


def gpu_stream(cfg, layer=0, units_sel=None, steps=None, progress=None, arrays=None, **create_kw):
    """Stream cfg (or `arrays`: fp32 [steps, units, d] triples made by hand, rounded to storage
    here) through a libwkv handle.  Returns dict(out [T,U',d] f64 for the selected
    units, evict_pos / evict_slot [T, units] i32, cache (open handle), inputs of the
    selected units as exact fp32)."""
    steps = cfg.steps if steps is None else steps
    st = synth.Stream(cfg, layer)
    if arrays is not None:
        stored = [synth.to_storage(np.ascontiguousarray(x, dtype=np.float32), cfg.dtype) for x in arrays]
    # one workgroup per unit unless a test asks otherwise (split=0 lets the library choose, as
    # the benchmark does; split>1 takes the sliced kernel)
    create_kw.setdefault("split", 1)
    cache = wkv.Cache(cfg.batch, cfg.heads, cfg.head_dim, cfg.budget, cfg.recent,
                      synth.DTYPE_CODE[cfg.dtype], **create_kw)
    sel = np.arange(cfg.units) if units_sel is None else np.asarray(units_sel)
    outs, evp, evs, qs, ks, vs = [], [], [], [], [], []
    t = 0
    while t < steps:
        c = t // synth.CHUNK
        q, k, v = st.chunk(c) if arrays is None else (x[t:t + synth.CHUNK] for x in stored)
        n = min(q.shape[0], steps - t)
        q, k, v = q[:n], k[:n], v[:n]
        tq, tk, tv = (to_device(x, cfg.dtype) for x in (q, k, v))
        out = torch.empty_like(tq)
        for i in range(n):
            cache.step(tq[i], tk[i], tv[i], out[i])
        torch.cuda.synchronize()
        p, s = cache.evictions(n)
        evp.append(p); evs.append(s)
        outs.append(out_to_f64(out[:, torch.from_numpy(sel).cuda()], cfg.dtype))
        for dst, src in ((qs, q), (ks, k), (vs, v)):
            dst.append(synth.storage_to_f32(src[:, sel], cfg.dtype))
        t += n
        if progress:
            print(f"  [{progress}] gpu step {t}/{steps}", flush=True)
    return dict(out=np.concatenate(outs), evict_pos=np.concatenate(evp), evict_slot=np.concatenate(evs),
                cache=cache, q=np.concatenate(qs), k=np.concatenate(ks), v=np.concatenate(vs), sel=sel)


def oracle_stream(cfg, g, forced=None, **orc_kw):
    orc = oracle.Oracle(len(g["sel"]), cfg.head_dim, cfg.budget, cfg.recent, storage=cfg.dtype, **orc_kw)
    res = orc.run(g["q"], g["k"], g["v"], forced_pos=forced)
    res["orc"] = orc
    return res


def round_to_storage(ref, dtype):
    """fp64 reference values rounded (nearest even) to the storage format, as fp64."""
    if dtype == "fp16":
        return ref.astype(np.float16).astype(np.float64)
    if dtype == "bf16":
        # fp64 -> fp32 first would round twice; go through round-to-odd on the way down
        f = ref.astype(np.float32)
        back = f.astype(np.float64)
        inexact = back != ref
        bits = f.view(np.uint32).copy()
        toward_zero = inexact & (np.abs(back) > np.abs(ref))
        bits[toward_zero] -= np.uint32(1)
        bits[inexact] |= np.uint32(1)
        return synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(bits.view(np.float32))).astype(np.float64)
    return ref.astype(np.float32).astype(np.float64)


def _format_index(x, dtype):
    """Position of every (representable) value on the format's number line, as an integer:
    neighbours in the format differ by 1."""
    if dtype == "fp16":
        b = x.astype(np.float16).view(np.int16).astype(np.int64)
        return np.where(b < 0, -(b & 0x7FFF), b)
    b = synth.f32_to_bf16_bits(x.astype(np.float32)).astype(np.int64)      # exact: x is representable
    return np.where(b & 0x8000, -(b & 0x7FFF), b)


def check_outputs(got, ref, dtype, what="out", exact_floor=None):
    exact_floor = EXACT_FLOOR if exact_floor is None else exact_floor
    scale = np.abs(ref).max(axis=-1, keepdims=True)
    err = np.abs(got - ref)
    bound = RTOL[dtype] * np.abs(ref) + ATOL_REL[dtype] * scale
    bad = err > bound
    assert not bad.any(), (f"{what}: {bad.sum()} elements out of tolerance, worst error "
                           f"{err.max():.3e} at {np.unravel_index(np.argmax(err - bound), err.shape)}")
    if dtype in EXACT_FLOOR:
        r = round_to_storage(ref, dtype)
        steps = np.abs(_format_index(got, dtype) - _format_index(r, dtype))
        off = (steps > 1) & (err > ATOL_REL[dtype] * scale)
        assert not off.any(), (f"{what}: {off.sum()} elements more than one {dtype} step from the rounded reference, "
                               f"first at {tuple(np.argwhere(off)[0])}")
        if got.size >= EXACT_FLOOR_MIN_ELEMENTS:
            frac = float((got == r).mean())
            assert frac >= exact_floor[dtype], f"{what}: only {frac:.5f} of the {dtype} elements are bit-exact"
    return float((err / np.maximum(scale, 1e-300)).max())


def exact_fraction(got, ref, dtype):
    """Fraction of elements that equal the reference rounded to the storage format."""
    return float((got == round_to_storage(ref, dtype)).mean())


def check_cache_state(cache, orc, sel, cfg, T):
    """The library's cache against the oracle's, unit by unit: token positions, counts, merge counts
    and keys bit-exact, score sums to 1e-9, values within the output tolerance.  Returns the number
    of units whose values are bit-identical."""
    assert cache.tokens == T and cache.length == min(T, cfg.budget)
    K = cache.state(wkv.WKV_K)[sel]; V = cache.state(wkv.WKV_V)[sel]
    a = cache.state(wkv.WKV_SCORE_SUM)[sel]; n = cache.state(wkv.WKV_COUNT)[sel]
    pos = cache.state(wkv.WKV_POS)[sel]; nm = cache.state(wkv.WKV_NMERGED)[sel]
    Kf = synth.storage_to_f32(K, cfg.dtype).astype(np.float64)
    Vf = synth.storage_to_f32(V, cfg.dtype).astype(np.float64)
    v_exact = 0
    for i in range(len(sel)):
        st = orc.state(i)
        assert np.array_equal(pos[i], st["pos"]), f"retained token positions differ (unit {sel[i]})"
        assert np.array_equal(n[i], st["n"]), "counts differ"
        assert np.array_equal(nm[i], st["nmerged"]), "merge counts differ"
        assert np.array_equal(Kf[i], st["K"]), "retained keys differ"
        assert np.allclose(a[i], st["a"], rtol=1e-9, atol=0), "score sums differ"
        check_outputs(Vf[i], st["V"], cfg.dtype, what="merged values")
        v_exact += int(np.array_equal(Vf[i], st["V"]))
    status = cache.state(wkv.WKV_STATUS)
    assert status[1] == 0, "non-finite scores flagged"
    return v_exact


def gpu_prefill(cfg, P, layer=0, units_sel=None, want_out=True, arrays=None, **create_kw):
    """Prefill a fresh handle with the first P tokens of the stream (or of `arrays`, fp32
    [steps, units, d] triples made by hand, rounded to storage here).  Returns dict(out [P,U',d]
    f64, cache, inputs of the selected units as exact fp32, the device tensors of the whole stream)."""
    if arrays is None:
        st = synth.Stream(cfg, layer)
        q, k, v = st.steps(0, cfg.steps)
    else:
        q, k, v = (synth.to_storage(np.ascontiguousarray(x, dtype=np.float32), cfg.dtype) for x in arrays)
    create_kw.setdefault("split", 1)
    cache = wkv.Cache(cfg.batch, cfg.heads, cfg.head_dim, cfg.budget, cfg.recent,
                      synth.DTYPE_CODE[cfg.dtype], **create_kw)
    sel = np.arange(cfg.units) if units_sel is None else np.asarray(units_sel)
    tq, tk, tv = (to_device(x, cfg.dtype) for x in (q, k, v))
    out = torch.zeros_like(tq) if want_out else None
    cache.prefill(tq[:P], tk[:P], tv[:P], None if out is None else out[:P])
    torch.cuda.synchronize()
    f32 = lambda x: synth.storage_to_f32(x[:, sel], cfg.dtype)
    return dict(out=None if out is None else out_to_f64(out[:P][:, torch.from_numpy(sel).cuda()], cfg.dtype),
                cache=cache, q=f32(q), k=f32(k), v=f32(v), sel=sel, dev=(tq, tk, tv, out), P=P)


def compare_prefill(cfg, g, decode_steps=0, **orc_kw):
    """gpu_prefill result against the oracle's prefill, then `decode_steps` streamed tokens on both."""
    P, sel = g["P"], g["sel"]
    orc = oracle.Oracle(len(sel), cfg.head_dim, cfg.budget, cfg.recent, storage=cfg.dtype, **orc_kw)
    ref = orc.prefill(g["q"][:P], g["k"][:P], g["v"][:P])
    stats = {}
    if g["out"] is not None:
        stats["out_err"] = check_outputs(g["out"], ref["out"], cfg.dtype, exact_floor=PREFILL_EXACT_FLOOR)
        stats["out_exact"] = exact_fraction(g["out"], ref["out"], cfg.dtype)
    stats["v_bit_exact_units"] = check_cache_state(g["cache"], orc, sel, cfg, P)
    if ref["evict_score"].size:
        with np.errstate(divide="ignore", invalid="ignore"):   # scores may be exactly 0
            gaps = np.diff(ref["evict_score"], axis=0) / ref["evict_score"][1:]
        stats["min_gap"] = float(gaps.min()) if gaps.size else float("nan")
    if decode_steps:
        tq, tk, tv, out = g["dev"]
        cache = g["cache"]
        for t in range(P, P + decode_steps):
            cache.step(tq[t], tk[t], tv[t], out[t])
        torch.cuda.synchronize()
        gp, _ = cache.evictions(decode_steps)
        r2 = orc.run(g["q"][P:P + decode_steps], g["k"][P:P + decode_steps], g["v"][P:P + decode_steps])
        assert np.array_equal(gp[:, sel], r2["evict_pos"]), "evictions after the prefill differ"
        got = out_to_f64(out[P:P + decode_steps][:, torch.from_numpy(sel).cuda()], cfg.dtype)
        check_outputs(got, r2["out"], cfg.dtype)
        check_cache_state(cache, orc, sel, cfg, P + decode_steps)
    return stats


def compare(cfg, g, check_state=True, log=print, **orc_kw):
    """Full comparison of a gpu_stream result with the oracle on the same inputs."""
    sel = g["sel"]
    gp, gs = g["evict_pos"][:, sel], g["evict_slot"][:, sel]
    ref = oracle_stream(cfg, g, **orc_kw)
    near_ties = 0
    if not np.array_equal(gp, ref["evict_pos"]):
        # classify: rerun the oracle following the GPU's choices, every override must be a near-tie
        forced = np.where(gp >= 0, gp, -1).astype(np.int32)
        ref = oracle_stream(cfg, g, forced=forced, **orc_kw)
        ov = ~np.isnan(ref["forced_score"])
        gap = np.abs(ref["forced_score"][ov] - ref["evict_score"][ov]) / np.abs(ref["evict_score"][ov])
        for (t, u), gv in zip(np.argwhere(ov), gap):
            log(f"near-tie: step {t} unit {sel[u]} relative score gap {gv:.3e}")
        assert (gap <= NEAR_TIE).all(), f"eviction index mismatch beyond near-tie: worst gap {gap.max():.3e}"
        near_ties = int(ov.sum())
    assert np.array_equal(gp, ref["evict_pos"]), "evicted token indices differ"
    assert np.array_equal(gs, ref["evict_slot"]), "evicted slot ranks differ"
    worst = check_outputs(g["out"], ref["out"], cfg.dtype)
    with np.errstate(divide="ignore", invalid="ignore"):       # a victim's score may be exactly 0
        rel_gap = (ref["runner_up"] - ref["evict_score"]) / ref["evict_score"]
    stats = dict(near_ties=near_ties, out_err=worst, out_exact=exact_fraction(g["out"], ref["out"], cfg.dtype),
                 min_gap=float(np.nanmin(rel_gap)) if np.isfinite(ref["evict_score"]).any() else float("nan"))
    if check_state:
        T = g["out"].shape[0]
        stats["v_bit_exact_units"] = check_cache_state(g["cache"], ref["orc"], sel, cfg, T)
    return stats


# --------------------------------------------------------------------------------------------
# comparison chunk by chunk: every unit of a full-size configuration without holding the stream
# --------------------------------------------------------------------------------------------
def compare_chunk(orc, cfg, t0, q, k, v, gpu_out, gpu_pos, gpu_slot, units=None, log=print):
    """One chunk of steps [t0, t0 + n): the oracle `orc` (which has seen steps < t0) is run over
    the chunk FOLLOWING the evictions the other side reports (gpu_pos), so that one pass both
    compares and classifies: wherever the oracle's own arg-min would have been another token,
    it reports the two scores, and the disagreement must be a near-tie by the oracle's scores
    (it is logged, and the comparison goes on from the other side's choice); a reported token
    that is no candidate at all makes the oracle refuse.  Outputs are checked to the stated bar.
    q, k, v: exact fp32 inputs [n, U, d]; gpu_out [n, U, d] f64; gpu_pos, gpu_slot [n, U] i32.
    Returns dict(near_ties, out_err, exact (count of bit-exact output elements), elements, min_gap)."""
    forced = np.where(gpu_pos >= 0, gpu_pos, -1).astype(np.int32)
    try:
        ref = orc.run(q, k, v, forced_pos=forced)
    except RuntimeError as e:
        raise AssertionError(f"steps {t0}..{t0 + len(q) - 1}: an evicted token is not a candidate of the oracle ({e})")
    ov = ~np.isnan(ref["forced_score"])
    near = 0
    if ov.any():
        gap = np.abs(ref["forced_score"][ov] - ref["evict_score"][ov]) / np.abs(ref["evict_score"][ov])
        for (t, u), gv in zip(np.argwhere(ov), gap):
            log(f"near-tie: step {t0 + t} unit {u if units is None else units[u]} relative score gap {gv:.3e}")
        assert (gap <= NEAR_TIE).all(), f"eviction index mismatch beyond near-tie: worst gap {gap.max():.3e}"
        near = int(ov.sum())
    assert np.array_equal(gpu_pos, ref["evict_pos"]), "evicted token indices differ"
    assert np.array_equal(gpu_slot, ref["evict_slot"]), "evicted slot ranks differ"
    worst = check_outputs(gpu_out, ref["out"], cfg.dtype)
    with np.errstate(divide="ignore", invalid="ignore"):
        rel_gap = (ref["runner_up"] - ref["evict_score"]) / ref["evict_score"]
    fin = np.isfinite(rel_gap)
    return dict(near_ties=near, out_err=worst, exact=int((gpu_out == round_to_storage(ref["out"], cfg.dtype)).sum()),
                elements=int(gpu_out.size), min_gap=float(rel_gap[fin].min()) if fin.any() else float("nan"))


def stream_compare(cfg, layer=0, steps=None, progress=None, log=print, **create_kw):
    """EVERY unit of cfg through libwkv and through the oracle, compared chunk by chunk (256 steps
    at a time; nothing of the stream is kept), then the final cache state of every unit.  The
    handle is created as the benchmark creates it unless create_kw says otherwise (split=0: the
    library chooses the kernel)."""
    steps = cfg.steps if steps is None else steps
    st = synth.Stream(cfg, layer)
    create_kw.setdefault("split", 0)
    okw = {k_: create_kw[k_] for k_ in ("n_sink", "score_mode", "merge_mode") if k_ in create_kw}
    cache = wkv.Cache(cfg.batch, cfg.heads, cfg.head_dim, cfg.budget, cfg.recent,
                      synth.DTYPE_CODE[cfg.dtype], **create_kw)
    orc = oracle.Oracle(cfg.units, cfg.head_dim, cfg.budget, cfg.recent, storage=cfg.dtype, **okw)
    tot = dict(near_ties=0, out_err=0.0, exact=0, elements=0, min_gap=float("inf"))
    try:
        t = 0
        while t < steps:
            q, k, v = st.chunk(t // synth.CHUNK)
            n = min(q.shape[0], steps - t)
            q, k, v = q[:n], k[:n], v[:n]
            tq, tk, tv = (to_device(x, cfg.dtype) for x in (q, k, v))
            out = torch.empty_like(tq)
            for i in range(n):
                cache.step(tq[i], tk[i], tv[i], out[i])
            torch.cuda.synchronize()
            gp, gs = cache.evictions(n)
            r = compare_chunk(orc, cfg, t, *(synth.storage_to_f32(x, cfg.dtype) for x in (q, k, v)),
                              out_to_f64(out, cfg.dtype), gp, gs, log=log)
            tot["near_ties"] += r["near_ties"]; tot["exact"] += r["exact"]; tot["elements"] += r["elements"]
            tot["out_err"] = max(tot["out_err"], r["out_err"])
            if r["min_gap"] == r["min_gap"]:
                tot["min_gap"] = min(tot["min_gap"], r["min_gap"])
            t += n
            if progress:
                print(f"  [{progress}] step {t}/{steps} compared, near-ties so far {tot['near_ties']}", flush=True)
        tot["v_bit_exact_units"] = check_cache_state(cache, orc, np.arange(cfg.units), cfg, steps)
        tot["pos"] = cache.state(wkv.WKV_POS)
    finally:
        cache.close()
    tot["out_exact"] = tot["exact"] / max(tot["elements"], 1)
    if cfg.dtype in EXACT_FLOOR and tot["elements"] >= EXACT_FLOOR_MIN_ELEMENTS:
        assert tot["out_exact"] >= EXACT_FLOOR[cfg.dtype], f"bit-exact share of the outputs {tot['out_exact']:.5f}"
    return tot
