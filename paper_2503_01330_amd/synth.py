"""Seeded synthetic q/k/v streams for the WeightedKV decode step.

This module only *draws inputs*.  It contains none of the method's arithmetic
(no attention, no scores, no merging) and is the single piece of code that both
the CPU oracle's tests and the HIP path's tests/benchmark consume, so that both
sides read byte-identical inputs.

The paper evaluates on Llama-2-7B (32 layers x 32 heads x 128) over PG19,
OpenWebText2, ProofPile and ArXiv (Section V-A); neither weights nor datasets
are used here.  The streams below take the *shapes* of that workload and the
one distributional fact the paper states about it (Section I, Fig. 1): keys are
strongly low-rank, values are not.  Keys are therefore a low-rank Gaussian
factor product, values are full-rank Gaussian.

Generation is counter based (numpy Philox keyed by (seed, layer, chunk)) and
chunked, so a 32k-token stream never has to exist in memory at once.  Numbers
are drawn in fp32 and rounded once (round-to-nearest-even) to the storage
dtype; both consumers see the rounded values.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import numpy as np

CHUNK = 256  # steps per generation chunk

# dtype codes shared with the C ABI (include/wkv.h) and the oracle
FP32, FP16, BF16 = 0, 1, 2
DTYPE_CODE = {"fp32": FP32, "fp16": FP16, "bf16": BF16}
DTYPE_BYTES = {"fp32": 4, "fp16": 2, "bf16": 2}


@dataclass(frozen=True)
class StreamConfig:
    name: str
    seed: int
    batch: int
    heads: int
    head_dim: int
    dtype: str           # "fp32" | "fp16" | "bf16"
    steps: int           # tokens streamed one at a time (prefill included)
    budget: int          # m: retained slots after every step
    recent: int          # R: newest R tokens are never evicted (counted inside m)
    layers: int = 1
    key_rank: int = 16
    key_noise: float = 0.0      # std of full-rank noise added to the low-rank keys
    sink_tokens: int = 0        # first tokens whose keys are scaled by sink_gain
    sink_gain: float = 1.0
    zipf_heads: bool = False    # per-head key-norm scale min(Zipf(1.1), 8)
    prefill: int = 0            # leading steps that are streamed but not timed

    @property
    def units(self) -> int:
        return self.batch * self.heads


# The five synthetic configurations (shapes of a Llama-2-7B-style workload, see the module docstring).
CONFIGS: Dict[str, StreamConfig] = {
    "cfg1": StreamConfig("cfg1", 1001, 1, 4, 64, "fp32", 512, 64, 16,
                         key_rank=8, key_noise=0.1),
    "cfg2": StreamConfig("cfg2", 1002, 1, 32, 128, "fp16", 4096, 819, 64),
    "cfg3": StreamConfig("cfg3", 1003, 8, 32, 128, "fp16", 4096, 410, 32, layers=32),
    "cfg4": StreamConfig("cfg4", 1004, 4, 32, 128, "fp16", 32768, 2048, 128,
                         sink_tokens=4, sink_gain=8.0),
    "cfg5": StreamConfig("cfg5", 1005, 64, 32, 128, "bf16", 3072, 512, 32,
                         zipf_heads=True, prefill=2048),
}


def scaled(cfg: StreamConfig, **kw) -> StreamConfig:
    """A variant of a configuration (shorter stream, fewer layers, ...)."""
    return replace(cfg, **kw)


# --------------------------------------------------------------------------
# storage-dtype rounding (input preparation only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 array -> storage representation (fp32 / fp16 arrays, uint16 bits for bf16)."""
    if dtype == "fp32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "fp16":
        return x.astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def storage_to_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact fp32 values of a storage array (every storage dtype embeds in fp32)."""
    if dtype == "fp32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "fp16":
        return x.astype(np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(x)
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# the stream
# --------------------------------------------------------------------------
class Stream:
    """q/k/v for one layer of one configuration, produced chunk by chunk.

    chunk(c) returns three storage arrays of shape [n, batch*heads, head_dim]
    for steps c*CHUNK .. c*CHUNK+n-1 (n = CHUNK except for a ragged last chunk).
    Unit index = b*heads + h.
    """

    def __init__(self, cfg: StreamConfig, layer: int = 0):
        if not (0 <= layer < cfg.layers):
            raise ValueError("layer out of range")
        self.cfg = cfg
        self.layer = layer
        g = np.random.Generator(np.random.Philox(key=[cfg.seed, (layer << 32) | 0xFFFFFFFF]))
        # per-(layer, head) mixing matrix of the low-rank keys
        self.W = g.standard_normal((cfg.heads, cfg.key_rank, cfg.head_dim), dtype=np.float32)
        if cfg.zipf_heads:
            z = g.zipf(1.1, size=cfg.heads).astype(np.float64)
            self.head_gain = np.minimum(z, 8.0).astype(np.float32)
        else:
            self.head_gain = np.ones(cfg.heads, dtype=np.float32)

    @property
    def n_chunks(self) -> int:
        return (self.cfg.steps + CHUNK - 1) // CHUNK

    def chunk(self, c: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        cfg = self.cfg
        t0 = c * CHUNK
        n = min(CHUNK, cfg.steps - t0)
        if n <= 0:
            raise IndexError("chunk beyond the stream")
        B, H, d, r = cfg.batch, cfg.heads, cfg.head_dim, cfg.key_rank
        g = np.random.Generator(np.random.Philox(key=[cfg.seed, (self.layer << 32) | c]))
        # always draw a full chunk so a ragged tail reads the same numbers
        q = g.standard_normal((CHUNK, B, H, d), dtype=np.float32)[:n]
        z = g.standard_normal((CHUNK, B, H, r), dtype=np.float32)[:n]
        v = g.standard_normal((CHUNK, B, H, d), dtype=np.float32)[:n]
        # k[t,b,h,:] = z[t,b,h,:] @ W[h] / sqrt(r)
        zh = np.ascontiguousarray(z.transpose(2, 0, 1, 3)).reshape(H, n * B, r)
        kh = np.matmul(zh, self.W) * np.float32(1.0 / np.sqrt(r))
        kh *= self.head_gain[:, None, None]
        k = np.ascontiguousarray(kh.reshape(H, n, B, d).transpose(1, 2, 0, 3))
        if cfg.key_noise:
            k += np.float32(cfg.key_noise) * g.standard_normal((CHUNK, B, H, d), dtype=np.float32)[:n]
        if cfg.sink_tokens and t0 < cfg.sink_tokens:
            k[: cfg.sink_tokens - t0] *= np.float32(cfg.sink_gain)
        shape = (n, B * H, d)
        return (to_storage(q.reshape(shape), cfg.dtype),
                to_storage(k.reshape(shape), cfg.dtype),
                to_storage(v.reshape(shape), cfg.dtype))

    def steps(self, t0: int, t1: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """Storage arrays for steps [t0, t1), assembled from chunks."""
        qs, ks, vs = [], [], []
        for c in range(t0 // CHUNK, (t1 - 1) // CHUNK + 1):
            q, k, v = self.chunk(c)
            lo = max(t0 - c * CHUNK, 0)
            hi = min(t1 - c * CHUNK, q.shape[0])
            qs.append(q[lo:hi]); ks.append(k[lo:hi]); vs.append(v[lo:hi])
        return np.concatenate(qs), np.concatenate(ks), np.concatenate(vs)
