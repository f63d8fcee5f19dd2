"""TEST INFRASTRUCTURE ONLY -- Python face of the CPU oracle.

`build()` compiles wkv_oracle.c with gcc; `Oracle` wraps it through ctypes.
Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; the product path (paper_2503_01330_amd) never does.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "wkv_oracle.c")
_LIB = os.path.join(_HERE, "libwkv_oracle.so")

STORAGE = {"fp64": -1, "fp32": 0, "fp16": 1, "bf16": 2}


def build(force: bool = True) -> str:
    """gcc -O2 -fopenmp; plain C, no intrinsics, no fast-math."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=gnu99", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(_LIB)
        dp, fp, ip = C.POINTER(C.c_double), C.POINTER(C.c_float), C.POINTER(C.c_int32)
        L.orc_create.restype = C.c_void_p
        L.orc_create.argtypes = [C.c_int] * 8
        L.orc_destroy.argtypes = [C.c_void_p]
        L.orc_run.restype = C.c_int
        L.orc_run.argtypes = [C.c_void_p, C.c_int, fp, fp, fp, dp, ip, ip, dp, dp, ip, dp, C.c_int]
        L.orc_prefill.restype = C.c_int
        L.orc_prefill.argtypes = [C.c_void_p, C.c_int, fp, fp, fp, dp, ip, dp, dp, C.c_int]
        L.orc_len.restype = C.c_int
        L.orc_len.argtypes = [C.c_void_p, C.c_int]
        L.orc_tokens.restype = C.c_int64
        L.orc_tokens.argtypes = [C.c_void_p, C.c_int]
        L.orc_threads.restype = C.c_int
        L.orc_state.argtypes = [C.c_void_p, C.c_int, dp, dp, dp, C.POINTER(C.c_int64), ip, ip]
        L.orc_round_storage.restype = C.c_double
        L.orc_round_storage.argtypes = [C.c_double, C.c_int]
        L.orc_attend.argtypes = [C.c_int, C.c_int, dp, dp, dp, dp, dp, dp]
        L.orc_select.restype = C.c_int
        L.orc_select.argtypes = [dp, C.c_int, C.c_int, dp]
        L.orc_merge_pair.argtypes = [C.c_double, C.c_double, dp, dp, C.c_int, C.c_int, dp]
        _lib = L
    return _lib


def _p(a, ty):
    return None if a is None else a.ctypes.data_as(C.POINTER(ty))


class Oracle:
    """fp64 WeightedKV over `units` independent (sequence, head) units."""

    def __init__(self, units, d, m, R, storage="fp64", n_sink=0, score_mode=0, merge_mode=0):
        self.units, self.d, self.m, self.R = units, d, m, R
        self._h = lib().orc_create(units, d, m, R, STORAGE[storage], n_sink, score_mode, merge_mode)
        if not self._h:
            raise ValueError("oracle: invalid configuration")

    def close(self):
        if self._h:
            lib().orc_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def run(self, q, k, v, want_out=True, forced_pos=None, threads=0):
        """q,k,v: float32 [n, units, d] (exact storage values).  Returns a dict with
        out [n,units,d] f64, evict_slot / evict_pos [n,units] i32, evict_score and
        runner_up [n,units] f64 (NaN where nothing was evicted)."""
        q = np.ascontiguousarray(q, dtype=np.float32)
        k = np.ascontiguousarray(k, dtype=np.float32)
        v = np.ascontiguousarray(v, dtype=np.float32)
        n = q.shape[0]
        assert q.shape == k.shape == v.shape == (n, self.units, self.d)
        out = np.empty((n, self.units, self.d), np.float64) if want_out else None
        es = np.empty((n, self.units), np.int32)
        ep = np.empty((n, self.units), np.int32)
        sc = np.empty((n, self.units), np.float64)
        ru = np.empty((n, self.units), np.float64)
        fs = None
        if forced_pos is not None:
            forced_pos = np.ascontiguousarray(forced_pos, dtype=np.int32)
            assert forced_pos.shape == (n, self.units)
            fs = np.empty((n, self.units), np.float64)
        rc = lib().orc_run(self._h, n, _p(q, C.c_float), _p(k, C.c_float), _p(v, C.c_float),
                           _p(out, C.c_double), _p(es, C.c_int32), _p(ep, C.c_int32),
                           _p(sc, C.c_double), _p(ru, C.c_double),
                           _p(forced_pos, C.c_int32), _p(fs, C.c_double), threads)
        if rc:
            raise RuntimeError(f"oracle: forced token is not a candidate at local step {-rc - 1}")
        return dict(out=out, evict_slot=es, evict_pos=ep, evict_score=sc, runner_up=ru,
                    forced_score=fs)

    def prefill(self, q, k, v, want_out=True, threads=0):
        """Bulk prefill of the (empty) cache with a prompt: q,k,v float32 [P, units, d].  Returns
        out [P,units,d] f64 and the removed tokens in order: evict_pos [max(P-m,0), units] i32,
        evict_score and runner_up (f64)."""
        q = np.ascontiguousarray(q, dtype=np.float32)
        k = np.ascontiguousarray(k, dtype=np.float32)
        v = np.ascontiguousarray(v, dtype=np.float32)
        P = q.shape[0]
        assert q.shape == k.shape == v.shape == (P, self.units, self.d)
        out = np.empty((P, self.units, self.d), np.float64) if want_out else None
        ne = max(P - self.m, 0)
        ep = np.empty((ne, self.units), np.int32)
        sc = np.empty((ne, self.units), np.float64)
        ru = np.empty((ne, self.units), np.float64)
        rc = lib().orc_prefill(self._h, P, _p(q, C.c_float), _p(k, C.c_float), _p(v, C.c_float),
                               _p(out, C.c_double), _p(ep, C.c_int32), _p(sc, C.c_double),
                               _p(ru, C.c_double), threads)
        if rc == -1:
            raise RuntimeError("oracle: prefill needs an empty cache")
        if rc == -2:
            raise ValueError("oracle: the last-step scoring rule is not defined for a prompt")
        return dict(out=out, evict_pos=ep, evict_score=sc, runner_up=ru)

    def length(self, unit=0):
        return lib().orc_len(self._h, unit)

    def tokens(self, unit=0):
        return lib().orc_tokens(self._h, unit)

    def state(self, unit):
        L = self.length(unit)
        K = np.empty((L, self.d)); V = np.empty((L, self.d)); a = np.empty(L)
        n = np.empty(L, np.int64); pos = np.empty(L, np.int32); nm = np.empty(L, np.int32)
        lib().orc_state(self._h, unit, _p(K, C.c_double), _p(V, C.c_double), _p(a, C.c_double),
                        _p(n, C.c_int64), _p(pos, C.c_int32), _p(nm, C.c_int32))
        return dict(K=K, V=V, a=a, n=n, pos=pos, nmerged=nm)


def threads() -> int:
    return lib().orc_threads()


def round_storage(x: float, storage: str) -> float:
    return lib().orc_round_storage(float(x), STORAGE[storage])


def attend(q, K, V):
    """Full softmax attention of one query over L rows; returns (o, p)."""
    q = np.ascontiguousarray(q, np.float64); K = np.ascontiguousarray(K, np.float64)
    V = np.ascontiguousarray(V, np.float64)
    L, d = K.shape
    s = np.empty(L); p = np.empty(L); o = np.empty(d)
    lib().orc_attend(L, d, _p(q, C.c_double), _p(K, C.c_double), _p(V, C.c_double),
                     _p(s, C.c_double), _p(p, C.c_double), _p(o, C.c_double))
    return o, p


def select(score, lo, hi):
    score = np.ascontiguousarray(score, np.float64)
    ru = C.c_double()
    j = lib().orc_select(_p(score, C.c_double), lo, hi, C.byref(ru))
    return j, ru.value


def merge_pair(wj, wr, Vj, Vr, storage="fp64"):
    Vj = np.ascontiguousarray(Vj, np.float64); Vr = np.ascontiguousarray(Vr, np.float64)
    out = np.empty_like(Vj)
    lib().orc_merge_pair(wj, wr, _p(Vj, C.c_double), _p(Vr, C.c_double), Vj.size, STORAGE[storage],
                         _p(out, C.c_double))
    return out
