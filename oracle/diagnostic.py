"""TEST INFRASTRUCTURE ONLY -- how far the compressed cache's outputs drift from full attention.

Runs the oracle three times over the same synthetic stream: uncompressed (budget >= stream),
WeightedKV (convex merge) and its eviction-only variant (the ablation of Section V-B), and
reports the mean relative output error of the two compressed runs against full attention.
Synthetic data: this shows the *shape* of the paper's ablation, not its perplexity numbers.

    python -m oracle.diagnostic
"""
import numpy as np

import oracle
from paper_2503_01330_amd import synth


def drift(cfg, steps):
    q, k, v = (synth.storage_to_f32(x, cfg.dtype) for x in synth.Stream(cfg).steps(0, steps))
    full = oracle.Oracle(cfg.units, cfg.head_dim, steps, 1).run(q, k, v)["out"]
    res = {}
    for name, mode in (("merge", 0), ("evict", 1)):
        out = oracle.Oracle(cfg.units, cfg.head_dim, cfg.budget, cfg.recent, merge_mode=mode).run(q, k, v)["out"]
        err = np.linalg.norm(out - full, axis=-1) / np.linalg.norm(full, axis=-1)
        res[name] = float(err[cfg.budget:].mean())
    return res


if __name__ == "__main__":
    for name, steps in (("cfg1", 512), ("cfg2", 2048)):
        cfg = synth.CONFIGS[name]
        if name == "cfg2":
            cfg = synth.scaled(cfg, heads=8, budget=410, recent=32)
        r = drift(cfg, steps)
        print(f"{name}: budget {cfg.budget} of {steps} tokens: mean relative output error vs full attention "
              f"merge {r['merge']:.4f}  evict {r['evict']:.4f}")
