#!/usr/bin/env python3
"""Writes the expected-output fixtures for the full-size configurations by running ONLY the CPU
oracle (oracle/) on the seeded synthetic inputs (synth/).  Nothing here touches the GPU library.

    python tests/golden/make_golden.py C2        # Qwen3-8B-shaped, batch 1, 32 greedy steps

    python tests/golden/make_golden.py C2 f64    # add the fp64 oracle's step-0 samples to C2_greedy.json and
                                                 # write all of its step-0 logits to C2_step0_logits_f64.npy
    python tests/golden/make_golden.py C2 f64 all   # ... and its last-step samples along the fixture's tokens
    python tests/golden/make_golden.py C4        # mixture-of-experts: routing decisions recorded too

Each fixture is a small JSON file: greedy tokens of every step, the top-8 logits (index, value)
of every step, and 512 pseudo-randomly sampled logits of step 0 and of the last step (fp32
oracle for the dense configurations, fp64 for mixture of experts); "samples64_0" holds the same step-0 samples from the oracle built with fp64 arithmetic
(same inputs), which bounds the fp32 oracle's own rounding error.
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import decoder as D  # noqa: E402
from synth import gen as G  # noqa: E402


def sample_indices(vocab, n=512):
    return (G.mix64(99, 77, np.arange(n, dtype=np.uint64)) % np.uint64(vocab)).astype(np.int64)


def add_f64(name):
    s = G.CONFIGS[name]
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"{name}_greedy.json")
    with open(path) as f:
        out = json.load(f)
    o = D.DecoderOracle(s, G.SynthWeights(s, out["seed"], cache=False), "f64")
    tok = np.array(out["start_tokens"], np.int64)
    pos = np.array(out["start_positions"], np.int64)
    idx = np.array(out["sample_indices"])
    lg = o.step(tok, pos)
    out["samples64_0"] = [[float(v) for v in lg[b, idx]] for b in range(s.batch)]
    out["absmax64_0"] = [float(np.abs(lg[b]).max()) for b in range(s.batch)]
    # every logit of step 0 from the fp64 build (stored as float32: 6e-8 relative, far below any
    # bound it is compared at)
    if s.batch == 1:
        np.save(os.path.join(os.path.dirname(path), f"{name}_step0_logits_f64.npy"), lg.astype(np.float32))
    if not s.n_experts and len(sys.argv) > 3 and sys.argv[3] == "all":
        # ... and the fp64 build driven along the fixture's token sequence to the last step, so
        # that later steps, too, are compared with a reference whose own rounding error is nil
        t0 = time.time()
        for i in range(1, out["steps"]):
            tok, pos = np.array(out["tokens"][i - 1], np.int64), pos + 1
            lg = o.step(tok, pos)
            print(f"fp64 step {i} ({time.time() - t0:.0f} s)", flush=True)
        out["samples64_last"] = [[float(v) for v in lg[b, idx]] for b in range(s.batch)]
        out["absmax64_last"] = [float(np.abs(lg[b]).max()) for b in range(s.batch)]
    if s.n_experts:
        # the fp32 oracle's own error on the router outputs, per layer (largest difference to the
        # fp64 oracle over sequences and experts at step 0): a routing decision whose margin is
        # below this scale is not resolved by fp32 arithmetic, whatever the summation order
        rl64 = o.last_moe_logits.astype(np.float64)
        o32 = D.DecoderOracle(s, G.SynthWeights(s, out["seed"], cache=False), "f32")
        lg32 = o32.step(tok, pos)
        out["samples32_0"] = [[float(v) for v in lg32[b, idx]] for b in range(s.batch)]
        out["moe_noise"] = np.abs(o32.last_moe_logits.astype(np.float64) - rl64).max((1, 2)).tolist()
    with open(path, "w") as f:
        json.dump(out, f)
    print("added fp64 step-0 samples to", path)


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "C2"
    if len(sys.argv) > 2 and sys.argv[2] == "f64":
        return add_f64(name)
    steps = int(sys.argv[2]) if len(sys.argv) > 2 else G.CONFIGS[name].steps
    s = G.CONFIGS[name]
    seed = 0
    layer_bytes = sum(rows * cols * 2 for _, rows, cols, _ in G.layer_tensor_shapes(s))
    cache = s.n_layers * layer_bytes < 40e9   # else every step regenerates the layers it visits
    # Top-k routing is discontinuous and the fp32 oracle's own rounding error on the router
    # outputs (1e-4 after 40 layers) is far above the GPU's, so a mixture-of-experts fixture comes
    # from the fp64 build: its decisions are the ones better arithmetic converges to.
    prec = "f64" if s.n_experts else "f32"
    o = D.DecoderOracle(s, G.SynthWeights(s, seed, cache=cache), prec)
    tok, pos = G.tokens(seed, s).astype(np.int64), G.kv_lengths(seed, s).astype(np.int64)
    idx = sample_indices(s.vocab)
    out = {"config": name, "seed": seed, "steps": steps, "start_tokens": tok.tolist(),
           "start_positions": pos.tolist(), "sample_indices": idx.tolist(), "tokens": [],
           "top8": [], "samples": {}, "top2_gap_min": None, "precision": prec}
    if s.n_experts:
        # routing decisions of every step: selected experts [layer][sequence][top_k] and the gap
        # between the top_k-th and the next router output [layer][sequence] (a decision with a
        # tiny gap may legitimately go the other way in another summation order)
        out["moe_sel"], out["moe_gap"] = [], []
    gap = np.inf
    t0 = time.time()
    for i in range(steps):
        lg = o.step(tok, pos)
        nxt = np.array([o.ops.argmax(lg[b]) for b in range(s.batch)], np.int64)
        top = []
        for b in range(s.batch):
            order = np.argsort(-lg[b], kind="stable")[:8]
            top.append([[int(j), float(lg[b, j])] for j in order])
            gap = min(gap, float(lg[b, order[0]] - lg[b, order[1]]))
        out["tokens"].append(nxt.tolist())
        out["top8"].append(top)
        if s.n_experts:
            r = -np.sort(-o.last_moe_logits.astype(np.float64), axis=-1)
            out["moe_sel"].append(o.last_moe_sel.tolist())
            out["moe_gap"].append((r[..., s.top_k - 1] - r[..., s.top_k]).tolist())
        if i in (0, steps - 1):
            out["samples"][str(i)] = [[float(v) for v in lg[b, idx]] for b in range(s.batch)]
            out["absmax_%d" % i] = [float(np.abs(lg[b]).max()) for b in range(s.batch)]
        tok, pos = nxt, pos + 1
        print(f"step {i}: tokens {nxt.tolist()}  ({time.time() - t0:.0f} s)", flush=True)
    out["top2_gap_min"] = gap
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"{name}_greedy.json")
    with open(path, "w") as f:
        json.dump(out, f)
    print("wrote", path)


if __name__ == "__main__":
    main()
