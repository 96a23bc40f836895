"""Writes tests/golden/gpt2medium_stage_G.json from the oracle alone (never from the HIP path).

The accumulated gradient G of ONE full iteration of the GPT-2-medium-shaped benchmark stage (6 blocks, hidden 1024,
16 heads, seq 1024, micro-batch 4, 16 micro-batches, causal; inputs and weights conditioned to bf16-representable
values), as the float64 oracle computes it: per parameter tensor its L2 norm and the values at 48 seeded positions.
The paper prints no numeric example; this is the oracle's own record at a size the GPU tests cannot afford to
recompute (16 micro-batches of float64 numpy: minutes).  Run:  python tests/golden/make_fullsize_golden.py
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import kfkb_synth as synth                      # noqa: E402
from oracle import schedule as sch              # noqa: E402
from oracle import stage_math as sm             # noqa: E402

CASE = dict(L=6, H=1024, heads=16, T=1024, b=4, M=16, dtype="bf16", samples=48, sample_seed=777)


def sample_positions(l, t, n, count, seed):
    """`count` seeded flat positions inside a tensor of n elements (block l, tensor index t)."""
    return (synth.uniform(seed + 101 * l + t, count) * n).astype(np.int64) % n


def compute(progress=True):
    c = CASE
    blocks = synth.stage_weights(c["L"], c["H"], 4 * c["H"], c["dtype"])
    G = [{n: np.zeros_like(v) for n, v in p.items()} for p in blocks]
    for mb in range(c["M"]):                     # ascending micro-batch order: the backward order of every kFkB plan
        t0 = time.time()
        x = synth.microbatch_inputs(mb, c["b"], c["T"], c["H"], c["dtype"])
        dy = synth.microbatch_upstream_grads(mb, c["b"], c["T"], c["H"], c["dtype"])
        _, caches = sm.stage_fwd(x, blocks, c["heads"], True)
        _, grads = sm.stage_bwd(dy, blocks, caches, c["heads"])
        del caches
        for Gl, gl in zip(G, grads):
            for n in Gl:
                Gl[n] += gl[n]
        if progress:
            print("micro-batch %d done in %.1f s" % (mb, time.time() - t0), flush=True)
    out = {"case": c, "tensors": {}}
    for l in range(c["L"]):
        for t, n in enumerate(synth.PARAM_ORDER):
            g = G[l][n].reshape(-1)
            pos = sample_positions(l, t, g.size, c["samples"], c["sample_seed"])
            out["tensors"]["%d.%s" % (l, n)] = {"l2": float(np.linalg.norm(g)), "max_abs": float(np.abs(g).max()),
                                                 "positions": [int(p) for p in pos], "values": [float(g[p]) for p in pos]}
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "gpt2medium_stage_G.json")
    res = compute()
    with open(path, "w") as f:
        json.dump(res, f, indent=0, sort_keys=True)
    print("wrote", path)
