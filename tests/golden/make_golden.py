"""Writes tests/golden/tiny_stage.json from the oracle alone (never from the HIP path).

The paper prints no worked numeric example (its figures carry the timelines), so this
fixture is a regression record of the oracle on one tiny seeded stage: a later edit of the
oracle's arithmetic shows up as a change here.  Run:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import kfkb_synth as synth                      # noqa: E402
from oracle import schedule as sch              # noqa: E402

CASE = dict(L=2, b=2, T=8, H=16, heads=4, F=64, M=4, k=2)


def compute():
    c = CASE
    blocks = synth.stage_weights(c["L"], c["H"], c["F"], "f32")
    xs = [synth.microbatch_inputs(mb, c["b"], c["T"], c["H"], "f32") for mb in range(c["M"])]
    dys = [synth.microbatch_upstream_grads(mb, c["b"], c["T"], c["H"], "f32") for mb in range(c["M"])]
    G, Y, dX, _ = sch.run_iteration(sch.kfkb_order(c["k"], c["M"]), blocks, xs, dys, c["heads"])
    out = {"case": c, "order": ["%s%d" % o for o in sch.kfkb_order(c["k"], c["M"])]}
    out["Y_sum"] = [float(y.sum()) for y in Y]
    out["dX_abs_sum"] = [float(np.abs(d).sum()) for d in dX]
    out["Y0_first4"] = [float(v) for v in Y[0].reshape(-1)[:4]]
    out["G_l2"] = {("%d.%s" % (l, n)): float(np.linalg.norm(G[l][n])) for l in range(c["L"]) for n in synth.PARAM_ORDER}
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_stage.json")
    with open(path, "w") as f:
        json.dump(compute(), f, indent=1, sort_keys=True)
    print("wrote", path)
