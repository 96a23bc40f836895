"""kfkb_op_colsum_accum_static: the column sum whose scratch is a device array built into the library (for callers
that cannot allocate).  Checked through the C boundary against kfkb_op_colsum_accum (same kernels, so the same bits)
and against the plain column sum, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

import paper_2303_01675_amd as kf
from _util import assert_close, dev, host, rnd

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dt", [kf.F32, kf.BF16, kf.F16])
def test_static_scratch_column_sum_matches_the_allocating_entry_point(dt):
    for seed, rows, N in [(31, 4096, 3072), (32, 333, 136)]:          # two calls in a row, the second smaller
        dy = rnd(seed, (rows, N), dt)
        d = dev(dy, dt)
        ref = torch.full((N,), 3.0, device="cuda")
        scratch = torch.empty(kf.kfkb_op_reduce_scratch_floats(N), device="cuda")
        kf.kfkb_op_colsum_accum(dt, d, ref, scratch, rows, N)
        out = torch.full((N,), 3.0, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        kf.kfkb_op_colsum_accum_static(dt, d, out, rows, N)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(out, ref)                                  # same kernels, same order: bit-identical
        assert_close(host(out) - 3.0, dy.sum(0), kf.F32, "colsum", factor=10)


def test_static_scratch_limits_and_empty_input():
    out = torch.zeros(40000, device="cuda")
    d = torch.zeros(8 * 40000, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(kf.KfkbError) as e:                            # wider than the built-in array: refused, nothing runs
        kf.kfkb_op_colsum_accum_static(kf.BF16, d, out, 8, 40000)
    assert e.value.code == -1
    with pytest.raises(kf.KfkbError) as e:
        kf.kfkb_op_colsum_accum_static(kf.BF16, d, out, 8, 132)
    assert e.value.code == -1
    kf.kfkb_op_colsum_accum_static(kf.BF16, d, out, 0, 128)            # no rows: nothing to add
    kf.kfkb_op_colsum_accum_static(kf.BF16, d, out, 8, 32768)          # the widest case the array holds
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
