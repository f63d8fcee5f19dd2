"""TEST INFRASTRUCTURE ONLY -- two oracle-side diagnostics on synthetic data.

1. `drift`: how far the compressed cache's outputs move from full attention.  Runs the oracle
   three times over the same synthetic stream: uncompressed (budget >= stream), WeightedKV
   (convex merge) and its eviction-only variant (the ablation of Section V-B), and reports the
   mean relative output error of the two compressed runs against full attention.

2. `single_merge_perturbation`: the experiment behind the paper's Fig. 2 (Section IV, first
   paragraphs).  At one generation step the token with the lowest average attention score is
   merged into its right-hand neighbour, once; the attention weights of the following steps are
   then compared with those of a run without the merge, by cosine similarity over the tokens
   both runs still hold, and the mean and standard deviation over the steps are reported.
   In a single attention layer whose queries and keys do not depend on earlier outputs the
   experiment is degenerate: dropping a key rescales every other weight of a row by the same
   factor, so the similarity is 1 whatever is merged.  The perturbation the paper measures
   travels through the model: the merged value changes the layer's later outputs, these feed the
   next layer's queries, keys and values.  The stand-in here is therefore a small stack of
   attention layers with fixed random projections and a residual connection (no trained weights,
   no dataset): the merge is made in every layer at the chosen step, layer 0 must stay at
   similarity 1 (the rescaling argument), deeper layers show the perturbation.

Synthetic Gaussian data shows the *shape* of these experiments, not the paper's numbers: the
paper measures Llama-2-7B on PG19 and calls the similarity "extremely close to 1"; random
projections of Gaussian tokens are no language model, and whatever figure comes out here
(about 0.9999 in the deeper layers of the default setting) says nothing about text.

    python -m oracle.diagnostic
"""
import math

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


class _Layer:
    """One attention layer's cache, uncompressed except for merges asked for explicitly; built on
    the oracle's own attention, selection and merge routines."""

    def __init__(self, d):
        self.d = d
        self.K, self.V = np.empty((0, d)), np.empty((0, d))
        self.a, self.born, self.tok = np.empty(0), np.empty(0, np.int64), np.empty(0, np.int64)

    def step(self, t, q, k, v):
        """Appends (k, v), attends; returns (output, attention weights, token of every weight)."""
        self.K = np.vstack([self.K, k]); self.V = np.vstack([self.V, v])
        self.a = np.append(self.a, 0.0); self.born = np.append(self.born, t); self.tok = np.append(self.tok, t)
        o, p = oracle.attend(q, self.K, self.V)
        self.a = self.a + p                                               # Algorithm 1's bookkeeping
        return o, p, self.tok.copy()

    def merge_lowest(self, t):
        """The token of lowest average score (the newest excluded) is folded into its right-hand
        neighbour: one application of Algorithm 1's selection, merge and removal."""
        abar = self.a / (t - self.born + 1)
        j, _ = oracle.select(abar, 0, len(abar) - 1)
        self.V[j + 1] = oracle.merge_pair(abar[j], abar[j + 1], self.V[j], self.V[j + 1])
        keep = np.arange(len(abar)) != j
        self.K, self.V, self.a = self.K[keep], self.V[keep], self.a[keep]
        self.born, self.tok = self.born[keep], self.tok[keep]
        return j


def _run_stack(x, W, merge_at):
    """x: [T, d] token inputs; W: per layer (Wq, Wk, Wv).  Returns per layer and step the attention
    weights and the tokens they belong to.  merge_at < 0: no merge."""
    T, d = x.shape
    layers = [_Layer(d) for _ in W]
    rows = [[] for _ in W]
    for t in range(T):
        h = x[t]
        for li, (Wq, Wk, Wv) in enumerate(W):
            o, p, tok = layers[li].step(t, Wq @ h, Wk @ h, Wv @ h)
            rows[li].append((p, tok))
            h = h + o                                                     # residual stream
        if t == merge_at:
            for layer in layers:
                layer.merge_lowest(t)
    return rows


def single_merge_perturbation(d=64, n_layers=3, merge_at=100, follow=800, seed=7):
    """Cosine similarity between the attention weights with and without one merge at step
    `merge_at`, over the `follow` steps after it and over the steps before it.
    Returns {layer: dict(mean, std, min, before)}; `before` is the lowest similarity of the steps
    up to and including the merge step (the two runs are identical there)."""
    g = np.random.default_rng(seed)
    T = merge_at + 1 + follow
    x = g.standard_normal((T, d))
    W = [tuple(g.standard_normal((d, d)) / math.sqrt(d) for _ in range(3)) for _ in range(n_layers)]
    plain = _run_stack(x, W, -1)
    merged = _run_stack(x, W, merge_at)
    res = {}
    for li in range(n_layers):
        sims = []
        for (p0, tok0), (p1, tok1) in zip(plain[li], merged[li]):
            both = np.isin(tok0, tok1)                                    # tokens the merged run still holds
            a, b = p0[both], p1
            sims.append(float(a @ b / math.sqrt((a @ a) * (b @ b))))
        sims = np.array(sims)
        after = sims[merge_at + 1:]
        res[li] = dict(mean=float(after.mean()), std=float(after.std()), min=float(after.min()),
                       before=float(sims[:merge_at + 1].min()))
    return res


if __name__ == "__main__":
    for name, steps in (("cfg1", 512), ("cfg2", 2048)):
        cfg = synth.CONFIGS[name]
        if name == "cfg2":
            cfg = synth.scaled(cfg, heads=8, budget=410, recent=32)
        r = drift(cfg, steps)
        print(f"{name}: budget {cfg.budget} of {steps} tokens: mean relative output error vs full attention "
              f"merge {r['merge']:.4f}  evict {r['evict']:.4f}")
    print("one merge at step 100, attention weights of the next 800 steps, cosine similarity with / without it "
          "(3 attention layers, random projections, d = 64):")
    for li, r in single_merge_perturbation().items():
        print(f"  layer {li}: mean {r['mean']:.6f}  std {r['std']:.6f}  min {r['min']:.6f}   (before the merge: {r['before']:.6f})")
