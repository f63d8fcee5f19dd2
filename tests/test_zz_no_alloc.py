"""wkv_prefill_noalloc (the entry point for callers that cannot allocate device memory) against
wkv_prefill: same kernels, the scratch in the library's static device array instead of the
handle's memory.  Two calls in a row, the second with a smaller input, so that the second one
runs over what the first left in the shared array; every output and the whole cache state must
be bit-identical to wkv_prefill's.  Collected last on purpose (the name sorts after the others).
"""
import numpy as np
import pytest
import torch

from paper_2503_01330_amd import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import parity
    from paper_2503_01330_amd import binding as wkv


def _both(cfg, P):
    """The same prompt through both entry points; returns (outputs, cache states) of each."""
    q, k, v = synth.Stream(cfg).steps(0, P)
    tq, tk, tv = (parity.to_device(x, cfg.dtype) for x in (q, k, v))
    res = []
    for noalloc in (False, True):
        cache = wkv.Cache(cfg.batch, cfg.heads, cfg.head_dim, cfg.budget, cfg.recent, synth.DTYPE_CODE[cfg.dtype])
        try:
            out = torch.zeros_like(tq)
            cache.prefill(tq, tk, tv, out, noalloc=noalloc)
            torch.cuda.synchronize()
            assert cache.tokens == P
            state = {w: cache.state(w) for w in (wkv.WKV_K, wkv.WKV_V, wkv.WKV_SCORE_SUM, wkv.WKV_POS, wkv.WKV_NMERGED)}
            res.append((out.view(torch.int16).cpu().numpy(), state, cache.state(wkv.WKV_STATUS)))
        finally:
            cache.close()
    return res


def test_noalloc_prefill_equals_prefill_twice_in_a_row():
    big = synth.StreamConfig("noalloc-big", 8801, 2, 8, 128, "fp16", 700, 96, 8)
    small = synth.StreamConfig("noalloc-small", 8802, 1, 3, 64, "bf16", 150, 40, 4)
    for cfg, P in ((big, 700), (small, 150)):
        (out_a, st_a, status_a), (out_b, st_b, status_b) = _both(cfg, P)
        assert np.array_equal(out_a, out_b), f"{cfg.name}: outputs differ"
        for w in st_a:
            assert np.array_equal(st_a[w], st_b[w]), f"{cfg.name}: cache state item {w} differs"
        assert np.array_equal(status_a, status_b)
    # and against the oracle, through the shared machinery, for the second (smaller) call's shape
    g = parity.gpu_prefill(small, 150)
    g["cache"].close()
    cache = wkv.Cache(small.batch, small.heads, small.head_dim, small.budget, small.recent, synth.DTYPE_CODE[small.dtype])
    tq, tk, tv, out = g["dev"]
    out.zero_()
    cache.prefill(tq[:150], tk[:150], tv[:150], out[:150], noalloc=True)
    torch.cuda.synchronize()
    g["cache"] = cache
    g["out"] = parity.out_to_f64(out[:150], small.dtype)
    try:
        parity.compare_prefill(small, g)
    finally:
        cache.close()


def test_noalloc_prefill_rejects_what_the_static_scratch_cannot_hold():
    # 1024 units x 2048 tokens = 2 Mi entries, twice the array
    cache = wkv.Cache(32, 32, 64, 64, 4, wkv.WKV_FP16)
    try:
        x = torch.zeros(16, dtype=torch.float16, device="cuda")
        with pytest.raises(wkv.WkvError) as e:
            wkv.wkv_prefill_noalloc(cache.h, x.data_ptr(), x.data_ptr(), x.data_ptr(), 0, 2048, 0)
        assert e.value.code == wkv.WKV_ESIZE
        assert cache.tokens == 0
    finally:
        cache.close()
