"""ctypes binding of libwkv (include/wkv.h): argument marshalling only.

Every step of the method runs inside the library's HIP kernels.  There is no
CPU or PyTorch fallback: if the shared library has not been built, importing
this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

# PyTorch ships its own copy of the HIP runtime.  The tensors handed to wkv_step live in that
# runtime's context, so it has to be the one libwkv binds to: load torch first, and the
# dynamic loader resolves libwkv's libamdhip64 dependency to the copy already in the process.
import torch  # noqa: F401  (imported for its side effect on library resolution)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libwkv.so")

WKV_FP32, WKV_FP16, WKV_BF16 = 0, 1, 2
WKV_OK, WKV_EINVAL, WKV_ENOMEM, WKV_EHIP, WKV_ESIZE = 0, -1, -2, -3, -4
WKV_MAX_BUDGET = 4095
WKV_MAX_PROMPT = 4096
WKV_SCORE_AVERAGE, WKV_SCORE_CUMULATIVE, WKV_SCORE_LAST = 0, 1, 2
WKV_MERGE_CONVEX, WKV_MERGE_NONE = 0, 1
WKV_LOADS_AUTO, WKV_LOADS_CACHED, WKV_LOADS_STREAMING = 0, 1, 2
(WKV_STEP, WKV_LEN, WKV_K, WKV_V, WKV_SCORE_SUM, WKV_COUNT, WKV_POS, WKV_NMERGED,
 WKV_EVICT_POS, WKV_EVICT_SLOT, WKV_STATUS) = range(11)

EXPORTS = ("wkv_create", "wkv_create_ex", "wkv_step", "wkv_prefill", "wkv_prefill_noalloc", "wkv_state", "wkv_load", "wkv_destroy",
           "wkv_last_error", "wkv_workspace_bytes", "wkv_step_bytes", "wkv_launch_shape", "wkv_probe_read", "wkv_version")


class wkv_options(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("batch", "heads", "head_dim", "budget", "recent_window",
                                        "dtype", "n_sink", "score_mode", "merge_mode",
                                        "log_capacity", "threads", "split", "streaming", "max_prompt", "replayable")] + [("reserved", C.c_int * 1)]


class WkvError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libwkv error {code}: {msg}")
        self.code = code


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it first (python -c "
                      "'import __graft_entry__ as g; g.build()'); there is no fallback path")

_lib = C.CDLL(LIB_PATH)
_lib.wkv_create.argtypes = [C.POINTER(C.c_void_p)] + [C.c_int] * 6
_lib.wkv_create_ex.argtypes = [C.POINTER(C.c_void_p), C.POINTER(wkv_options)]
_lib.wkv_step.argtypes = [C.c_void_p] * 6
_lib.wkv_prefill.argtypes = [C.c_void_p] * 5 + [C.c_int, C.c_void_p]
_lib.wkv_prefill_noalloc.argtypes = [C.c_void_p] * 5 + [C.c_int, C.c_void_p]
_lib.wkv_state.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_size_t]
_lib.wkv_load.argtypes = [C.c_void_p, C.c_int64, C.c_int] + [C.c_void_p] * 4
_lib.wkv_destroy.argtypes = [C.c_void_p]
_lib.wkv_last_error.restype = C.c_char_p
_lib.wkv_workspace_bytes.restype = C.c_size_t
_lib.wkv_workspace_bytes.argtypes = [C.POINTER(wkv_options)]
_lib.wkv_step_bytes.restype = C.c_size_t
_lib.wkv_step_bytes.argtypes = [C.POINTER(wkv_options)]


_lib.wkv_probe_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]


def wkv_probe_read(src: int, nbytes: int, workgroups: int, threads: int, nontemporal: bool, sink: int = 0,
                   stream: int = 0) -> None:
    """Plain streaming read of device memory with a chosen launch shape (measurement aid)."""
    _check(_lib.wkv_probe_read(src, nbytes, workgroups, threads, int(nontemporal), sink or None, stream))


def wkv_last_error() -> str:
    return _lib.wkv_last_error().decode()


def _check(rc):
    if rc != WKV_OK:
        raise WkvError(rc, wkv_last_error())


def wkv_version() -> int:
    return _lib.wkv_version()


def make_options(batch, heads, head_dim, budget, recent_window, dtype, n_sink=0, score_mode=0,
                 merge_mode=0, log_capacity=0, threads=0, split=0, streaming=0, max_prompt=0,
                 replayable=0) -> wkv_options:
    return wkv_options(batch, heads, head_dim, budget, recent_window, dtype, n_sink, score_mode,
                       merge_mode, log_capacity, threads, split, streaming, max_prompt, replayable)


def wkv_create(batch, heads, head_dim, budget, recent_window, dtype):
    h = C.c_void_p()
    _check(_lib.wkv_create(C.byref(h), batch, heads, head_dim, budget, recent_window, dtype))
    return h


def wkv_create_ex(opt: wkv_options):
    h = C.c_void_p()
    _check(_lib.wkv_create_ex(C.byref(h), C.byref(opt)))
    return h


def wkv_step(h, q: int, k_new: int, v_new: int, out: int, stream: int = 0) -> None:
    """q, k_new, v_new, out: device addresses (tensor.data_ptr()); stream: hipStream_t as int."""
    _check(_lib.wkv_step(h, q, k_new, v_new, out, stream))


def wkv_prefill(h, q: int, k: int, v: int, out: int, n_tokens: int, stream: int = 0) -> None:
    """q, k, v, out: device addresses of [n_tokens, batch, heads, head_dim] arrays (out may be 0)."""
    _check(_lib.wkv_prefill(h, q, k, v, out or None, n_tokens, stream))


def wkv_prefill_noalloc(h, q: int, k: int, v: int, out: int, n_tokens: int, stream: int = 0) -> None:
    """wkv_prefill on the library's static scratch: no device allocation in the call."""
    _check(_lib.wkv_prefill_noalloc(h, q, k, v, out or None, n_tokens, stream))


def wkv_state_raw(h, what: int, dst: np.ndarray) -> None:
    _check(_lib.wkv_state(h, what, dst.ctypes.data_as(C.c_void_p), dst.nbytes))


def wkv_load(h, tokens: int, length: int, K: np.ndarray, V: np.ndarray, score_sum: np.ndarray,
             pos: np.ndarray) -> None:
    """Host arrays in token order, as wkv_state returns them."""
    K, V = np.ascontiguousarray(K), np.ascontiguousarray(V)
    score_sum = np.ascontiguousarray(score_sum, np.float64)
    pos = np.ascontiguousarray(pos, np.int32)
    _check(_lib.wkv_load(h, tokens, length, K.ctypes.data_as(C.c_void_p), V.ctypes.data_as(C.c_void_p),
                         score_sum.ctypes.data_as(C.c_void_p), pos.ctypes.data_as(C.c_void_p)))


def wkv_destroy(h) -> None:
    _check(_lib.wkv_destroy(h))


def wkv_workspace_bytes(opt: wkv_options) -> int:
    return _lib.wkv_workspace_bytes(C.byref(opt))


def wkv_step_bytes(opt: wkv_options) -> int:
    return _lib.wkv_step_bytes(C.byref(opt))


def wkv_launch_shape(opt: wkv_options):
    """(workgroups, threads per workgroup) of a wkv_step launch for these options."""
    g, t = C.c_int(), C.c_int()
    _check(_lib.wkv_launch_shape(C.byref(opt), C.byref(g), C.byref(t)))
    return g.value, t.value


_NP_STORE = {WKV_FP32: np.float32, WKV_FP16: np.float16, WKV_BF16: np.uint16}


class Cache:
    """Owner of one handle; remembers the shape so readbacks can be sized."""

    def __init__(self, batch, heads, head_dim, budget, recent_window, dtype, **kw):
        self.opt = make_options(batch, heads, head_dim, budget, recent_window, dtype, **kw)
        self.units, self.d, self.dtype = batch * heads, head_dim, dtype
        self.h = wkv_create_ex(self.opt)

    def step(self, q, k_new, v_new, out, stream=None):
        """q, k_new, v_new, out: torch tensors on the GPU, contiguous [batch, heads, head_dim]."""
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        wkv_step(self.h, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), out.data_ptr(), stream)

    def prefill(self, q, k, v, out=None, stream=None, noalloc=False):
        """q, k, v (and out, if wanted): torch tensors on the GPU, contiguous [n_tokens, batch, heads, head_dim]
        (or [n_tokens, units, head_dim]); the cache must be empty.  noalloc: through wkv_prefill_noalloc."""
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        (wkv_prefill_noalloc if noalloc else wkv_prefill)(
            self.h, q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr() if out is not None else 0,
            q.shape[0], stream)

    def step_ptr(self, q, k_new, v_new, out, stream=0):
        wkv_step(self.h, q, k_new, v_new, out, stream)

    @property
    def tokens(self) -> int:
        t = np.zeros(1, np.int64)
        wkv_state_raw(self.h, WKV_STEP, t)
        return int(t[0])

    @property
    def length(self) -> int:
        l = np.zeros(1, np.int32)
        wkv_state_raw(self.h, WKV_LEN, l)
        return int(l[0])

    def state(self, what):
        """Slot arrays in token order; K/V in the storage dtype (bf16 as uint16 bit patterns)."""
        L = self.length
        if what in (WKV_K, WKV_V):
            dst = np.empty((self.units, L, self.d), _NP_STORE[self.dtype])
        elif what == WKV_SCORE_SUM:
            dst = np.empty((self.units, L), np.float64)
        elif what in (WKV_COUNT, WKV_POS, WKV_NMERGED):
            dst = np.empty((self.units, L), np.int32)
        elif what == WKV_STATUS:
            dst = np.empty(2, np.int32)
        else:
            raise ValueError("use evictions() / tokens / length for this item")
        if dst.size:
            wkv_state_raw(self.h, what, dst)
        return dst

    def evictions(self, n):
        """(evict_pos, evict_slot) of the last n steps, each int32 [n, units]."""
        pos = np.empty((n, self.units), np.int32)
        slot = np.empty((n, self.units), np.int32)
        if n:
            wkv_state_raw(self.h, WKV_EVICT_POS, pos)
            wkv_state_raw(self.h, WKV_EVICT_SLOT, slot)
        return pos, slot

    def load(self, tokens, K, V, score_sum, pos):
        wkv_load(self.h, tokens, pos.shape[1] if pos.ndim == 2 else 0, K, V, score_sum, pos)

    def step_bytes(self) -> int:
        return wkv_step_bytes(self.opt)

    def close(self):
        if self.h is not None:
            wkv_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
