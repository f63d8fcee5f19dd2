"""The CPU side under AddressSanitizer and UndefinedBehaviorSanitizer.

oracle/wkv_oracle.c is compiled, together with the small driver in tests/sanitize/, with
`gcc -O1 -fsanitize=address,undefined` into a stand-alone program (a sanitized shared object
cannot be loaded into an unsanitized Python).  The program runs the cases the pin tests rely on --
random streams in every rule and merge mode with sinks and all storage formats, prompts through
the bulk prefill, a stream with forced choices -- and must finish without a sanitizer report and
with the results of the regular build.
"""
import os
import struct
import subprocess

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def _build(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=gnu99", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-Wall",
           os.path.join(ROOT, "oracle", "wkv_oracle.c"), os.path.join(HERE, "sanitize", "driver.c"),
           "-o", exe, "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 and "asan" in (r.stderr or "").lower() and "cannot find" in r.stderr:
        pytest.skip("the sanitizer runtimes are not installed")
    assert r.returncode == 0, r.stderr
    return exe


def _cases():
    g = np.random.default_rng(77)
    out = []
    for storage in ("fp64", "fp32", "fp16", "bf16"):
        for rule, mm in ((0, 0), (0, 1), (1, 1), (2, 1)):
            units, d = int(g.integers(1, 4)), int(g.integers(1, 17))
            m = int(g.integers(1, 12)); R = int(g.integers(1, m + 1)); ns = int(g.integers(0, m - R + 1))
            n = int(g.integers(1, 60))
            out.append(dict(kind=0, units=units, d=d, m=m, R=R, storage=storage, n_sink=ns, score_mode=rule,
                            merge_mode=mm, n=n))
    for storage, rule, mm, P, m, R, ns in (("fp16", 0, 0, 45, 11, 1, 0), ("bf16", 0, 0, 64, 16, 5, 3),
                                            ("fp64", 1, 1, 30, 8, 2, 0), ("fp16", 0, 1, 9, 20, 4, 2),
                                            ("fp32", 0, 0, 21, 20, 20, 0)):
        out.append(dict(kind=1, units=2, d=8, m=m, R=R, storage=storage, n_sink=ns, score_mode=rule,
                        merge_mode=mm, n=P))
    for c in out:
        shape = (c["n"], c["units"], c["d"])
        c["q"], c["k"], c["v"] = (g.standard_normal(shape).astype(np.float16).astype(np.float32) for _ in range(3))
    # a stream in which every compression is told which token to drop (the near-tie hook): the
    # oldest unprotected one, always a legal choice
    c = dict(kind=0, units=2, d=8, m=6, R=2, storage="fp16", n_sink=1, score_mode=0, merge_mode=0, n=30)
    shape = (c["n"], c["units"], c["d"])
    c["q"], c["k"], c["v"] = (g.standard_normal(shape).astype(np.float16).astype(np.float32) for _ in range(3))
    ref = oracle.Oracle(2, 8, 6, 2, "fp16", n_sink=1)
    forced = np.full((30, 2), -1, np.int32)
    alive = [list(), list()]
    for t in range(30):
        for u in range(2):
            alive[u].append(t)
            if len(alive[u]) > 6:
                forced[t, u] = alive[u][1]          # the oldest token after the protected first one
                alive[u].remove(forced[t, u])
    c["forced"] = forced
    out.append(c)
    return out


def test_oracle_runs_clean_under_the_sanitizers(tmp_path):
    exe = _build(tmp_path)
    cases = _cases()
    with open(tmp_path / "cases.bin", "wb") as f:
        for c in cases:
            forced = c.get("forced")
            f.write(struct.pack("11i", c["kind"], c["units"], c["d"], c["m"], c["R"], oracle.STORAGE[c["storage"]],
                                c["n_sink"], c["score_mode"], c["merge_mode"], c["n"], int(forced is not None)))
            for x in (c["q"], c["k"], c["v"]):
                f.write(np.ascontiguousarray(x, np.float32).tobytes())
            if forced is not None:
                f.write(np.ascontiguousarray(forced, np.int32).tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2")
    r = subprocess.run([exe, str(tmp_path / "cases.bin"), str(tmp_path / "res.bin")], capture_output=True, text=True,
                       env=env, timeout=300)
    if r.returncode != 0 and "LeakSanitizer has encountered a fatal error" in r.stderr:
        env["ASAN_OPTIONS"] = "detect_leaks=0"          # no ptrace here: everything but the leak check
        r = subprocess.run([exe, str(tmp_path / "cases.bin"), str(tmp_path / "res.bin")], capture_output=True,
                           text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    assert r.stdout.strip() == f"{len(cases)} cases"

    # same results as the regular build (same source, other optimisation level: no fast-math, so bit for bit)
    raw = open(tmp_path / "res.bin", "rb").read()
    off = 0

    def take(dtype, count):
        nonlocal off
        a = np.frombuffer(raw, dtype, count, off)
        off += a.nbytes
        return a

    for c in cases:
        o = oracle.Oracle(c["units"], c["d"], c["m"], c["R"], c["storage"], n_sink=c["n_sink"],
                          score_mode=c["score_mode"], merge_mode=c["merge_mode"])
        ref = o.run(c["q"], c["k"], c["v"], forced_pos=c.get("forced")) if c["kind"] == 0 else o.prefill(c["q"], c["k"], c["v"])
        assert take(np.int32, 1)[0] == 0
        assert np.array_equal(take(np.float64, c["q"].size).reshape(c["q"].shape), ref["out"])
        assert np.array_equal(take(np.int32, ref["evict_pos"].size).reshape(ref["evict_pos"].shape), ref["evict_pos"])
        for u in range(c["units"]):
            st = o.state(u)
            L = int(take(np.int32, 1)[0])
            assert L == len(st["pos"])
            assert np.array_equal(take(np.float64, L * c["d"]).reshape(L, c["d"]), st["V"])
            assert np.array_equal(take(np.float64, L), st["a"])
            assert np.array_equal(take(np.int32, L), st["pos"])
    assert off == len(raw)
