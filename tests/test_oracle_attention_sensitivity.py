"""How much bf16 STORAGE of its inputs costs attention, shown with the oracle alone (no GPU): q, k, v and dO are rounded
to bf16, everything else is the float64 oracle.  With weights N(0, 0.02) the logits of the benchmark stages have standard
deviation 0.02^2 * hidden = 0.8, 1.6 and 3.3 (hidden 2048, 4096, 8192); the sharper the softmax, the more it multiplies
relative perturbations of its inputs.  This is the arithmetic behind the bar of the very wide stage's full-size test
(tests/test_gpu_fullsize_large.py): there the inputs of the last block's attention backward already carry 0.5 - 0.65e-2
of storage rounding from the ops before it."""
import numpy as np

import kfkb_synth as synth
from oracle import stage_math as sm


def _errors(sigma, T=1024, d=128, seed=5):
    q, k, v, do = (synth.normal(seed + i, T * d, 0.0, s).reshape(1, 1, T, d) for i, s in enumerate((sigma, sigma, sigma, 1.0)))
    r = lambda a: synth.round_to_bf16(a).astype(np.float64)

    def run(q, k, v, do):
        o, p = sm.attention_fwd(q, k, v, True)
        return (o,) + sm.attention_bwd(do, q, k, v, p)

    exact = run(q, k, v, do)
    stored = run(r(q), r(k), r(v), r(do))
    rel = lambda a, b: np.linalg.norm(a - b) / np.linalg.norm(b)
    storage = np.mean([rel(r(a), a) for a in (q, k, v, do)])
    return storage, rel(stored[0], exact[0]), rel(stored[1], exact[1]), rel(stored[2], exact[2])


def test_sharp_softmax_multiplies_the_storage_rounding_of_its_inputs():
    amp = {}
    for sigma in (0.9, 1.28, 1.81):                              # 0.02 * sqrt(hidden) for hidden 2048, 4096, 8192
        storage, eo, edq, edk = _errors(sigma)
        assert 1.2e-3 < storage < 2.2e-3                         # bf16 keeps 8 significant bits: 2^-9 / sqrt(3) ... 2^-9
        amp[sigma] = (edq / storage, edk / storage)
    # the amplification grows with the logit scale; at the very wide stage's scale it is above three
    assert amp[0.9][0] < amp[1.28][0] < amp[1.81][0] and amp[0.9][1] < amp[1.28][1] < amp[1.81][1]
    assert amp[1.81][0] > 3.0 and amp[1.81][1] > 3.0
    assert amp[0.9][0] < 2.5
