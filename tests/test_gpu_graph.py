"""Recorded steps replayed from a HIP graph (handles created with `replayable`): the token index
lives on the device and advances with every replay, so a stack of layers recorded once can be
replayed token after token.  Every replay is compared with a plain, directly enqueued run of the
same stream, bit for bit: outputs, eviction log, final cache state.  Between two replays the test
does ordinary eager work on the same stream (input copies, output copies, a synchronisation).
"""
import numpy as np
import pytest
import torch

from paper_2503_01330_amd import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import parity
    from paper_2503_01330_amd import binding as wkv


def _streams(cfg, layers, T):
    per = []
    for l in range(layers):
        q, k, v = synth.Stream(synth.scaled(cfg, layers=layers), l).steps(0, T)
        per.append(tuple(parity.to_device(x, cfg.dtype) for x in (q, k, v)))
    return per


def _state(c):
    return {w: c.state(w) for w in (wkv.WKV_K, wkv.WKV_V, wkv.WKV_SCORE_SUM, wkv.WKV_POS)}


@pytest.mark.parametrize("name,batch,heads,d,dtype,m,R,kw", [
    ("wide", 2, 4, 128, "fp16", 40, 4, dict(threads=1024)),            # four bookkeeping waves
    ("narrow", 3, 4, 64, "bf16", 70, 9, dict(threads=256)),            # the smaller workgroups
    ("sliced", 1, 2, 128, "fp16", 300, 5, dict(split=4)),              # several workgroups per unit
])
def test_replayed_steps_equal_enqueued_steps(name, batch, heads, d, dtype, m, R, kw):
    layers, T = 3, m + 45                                   # through the fill phase and 45 compressions
    cfg = synth.StreamConfig(f"graph-{name}", 9100 + m, batch, heads, d, dtype, T, m, R, layers=layers)
    code = synth.DTYPE_CODE[dtype]
    data = _streams(cfg, layers, T)
    kw = dict(kw); kw.setdefault("split", 1)

    # reference: every step enqueued directly (ordinary handles)
    ref_out = [torch.empty_like(q) for q, _, _ in data]
    ref = [wkv.Cache(batch, heads, d, m, R, code, **kw) for _ in range(layers)]
    for t in range(T):
        for l, (q, k, v) in enumerate(data):
            ref[l].step(q[t], k[t], v[t], ref_out[l][t])
    torch.cuda.synchronize()

    # recorded once, replayed T - 2 times; the first and the last token are enqueued directly
    caches = [wkv.Cache(batch, heads, d, m, R, code, replayable=1, **kw) for _ in range(layers)]
    try:
        sq, sk, sv, so = ([torch.empty_like(data[l][0][0]) for l in range(layers)] for _ in range(4))
        got = [torch.empty_like(q) for q, _, _ in data]
        for l, (q, k, v) in enumerate(data):
            caches[l].step(q[0], k[0], v[0], got[l][0])
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        for l, (q, k, v) in enumerate(data):               # the recording below executes nothing: stage token 1
            sq[l].copy_(q[1]); sk[l].copy_(k[1]); sv[l].copy_(v[1])
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            for l in range(layers):
                caches[l].step(sq[l], sk[l], sv[l], so[l])
        for t in range(1, T - 1):
            for l, (q, k, v) in enumerate(data):
                sq[l].copy_(q[t]); sk[l].copy_(k[t]); sv[l].copy_(v[t])
            g.replay()
            for l in range(layers):
                got[l][t].copy_(so[l])
            if t % 7 == 0:
                torch.cuda.synchronize()
        for l, (q, k, v) in enumerate(data):
            caches[l].step(q[T - 1], k[T - 1], v[T - 1], got[l][T - 1])
        torch.cuda.synchronize()
        for l in range(layers):
            assert caches[l].tokens == T, "the device-side token index did not follow the replays"
            assert torch.equal(got[l].view(torch.int16) if dtype != "fp32" else got[l],
                               ref_out[l].view(torch.int16) if dtype != "fp32" else ref_out[l]), f"outputs differ (layer {l})"
            n = min(T, 1024)
            gp, gs = caches[l].evictions(n)
            rp, rs = ref[l].evictions(n)
            assert np.array_equal(gp, rp) and np.array_equal(gs, rs), f"eviction logs differ (layer {l})"
            a, b = _state(caches[l]), _state(ref[l])
            for w in a:
                assert np.array_equal(a[w], b[w]), f"cache state item {w} differs (layer {l})"
    finally:
        for c in caches + ref:
            c.close()


def test_replayable_prefill_and_load_set_the_device_index():
    cfg = synth.StreamConfig("graph-prefill", 9200, 1, 4, 128, "fp16", 90, 30, 4)
    code = synth.DTYPE_CODE[cfg.dtype]
    q, k, v = (parity.to_device(x, cfg.dtype) for x in synth.Stream(cfg).steps(0, cfg.steps))
    a = wkv.Cache(1, 4, 128, 30, 4, code, replayable=1)
    b = wkv.Cache(1, 4, 128, 30, 4, code)
    try:
        out_a, out_b = torch.empty_like(q), torch.empty_like(q)
        a.prefill(q[:60], k[:60], v[:60], out_a[:60]); b.prefill(q[:60], k[:60], v[:60], out_b[:60])
        for t in range(60, 90):
            a.step(q[t], k[t], v[t], out_a[t]); b.step(q[t], k[t], v[t], out_b[t])
        torch.cuda.synchronize()
        assert a.tokens == b.tokens == 90
        assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16))
        for w in (wkv.WKV_V, wkv.WKV_SCORE_SUM, wkv.WKV_POS):
            assert np.array_equal(a.state(w), b.state(w))
        # resume a replayable handle from a readback
        c = wkv.Cache(1, 4, 128, 30, 4, code, replayable=1)
        try:
            c.load(90, b.state(wkv.WKV_K), b.state(wkv.WKV_V), b.state(wkv.WKV_SCORE_SUM), b.state(wkv.WKV_POS))
            assert c.tokens == 90
            o1, o2 = torch.empty_like(q[0]), torch.empty_like(q[0])
            c.step(q[5], k[5], v[5], o1); b.step(q[5], k[5], v[5], o2)
            torch.cuda.synchronize()
            assert c.tokens == 91 and np.array_equal(c.evictions(1)[0], b.evictions(1)[0])
        finally:
            c.close()
    finally:
        a.close(); b.close()
