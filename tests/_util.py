"""Helpers shared by the GPU parity tests (comparison metrics and host<->device marshalling)."""
import numpy as np
import torch

import kfkb_synth as synth
import paper_2303_01675_amd as kf

# relative tolerances: fp32 and bf16 as the parity bar states them; fp16 carries three more mantissa bits than bf16
# (unit roundoff 2^-11 against 2^-8), its bar is the bf16 one divided by eight
TOL = {kf.F32: 1e-4, kf.BF16: 2e-2, kf.F16: 2.5e-3}
NAME = {kf.F32: "f32", kf.BF16: "bf16", kf.F16: "f16"}


def tdtype(dt):
    return torch.bfloat16 if dt == kf.BF16 else torch.float16 if dt == kf.F16 else torch.float32


def dev(a, dt):
    """numpy (values representable in dt) -> device tensor of storage type dt."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(tdtype(dt)).cuda()


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rnd(seed, shape, dt, std=1.0, mean=0.0):
    """Seeded N(mean, std^2) values, conditioned to be exactly representable in dt (float64 array)."""
    n = int(np.prod(shape))
    v = synth.normal(seed, n, mean, std)
    if dt == kf.BF16:
        v = synth.round_to_bf16(v).astype(np.float64)
    elif dt == kf.F16:
        v = v.astype(np.float32).astype(np.float16).astype(np.float64)
    else:
        v = v.astype(np.float32).astype(np.float64)
    return v.reshape(shape)


def rel_l2(got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return np.linalg.norm(got - ref) / den if den > 0 else np.linalg.norm(got)


def assert_close(got, ref, dt, what="", factor=1.0, max_factor=8.0, floor=0.0):
    """Per tensor: ||got - ref|| / ||ref|| <= tol and max|got - ref| <= tol * max|ref| * max_factor.
    `floor`: magnitude of the terms the result is a sum of; a reference that cancels to (nearly)
    zero is then compared on that scale instead of its own."""
    tol = TOL[dt] * factor
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what + ": non-finite values"
    if not ref.size:
        return
    den = max(np.linalg.norm(ref), floor * np.sqrt(ref.size))
    r = np.linalg.norm(got - ref) / max(den, 1e-300)
    assert r <= tol, "%s: relative L2 error %.3e > %.1e" % (what, r, tol)
    m = np.abs(got - ref).max()
    lim = tol * max(np.abs(ref).max(), floor, 1e-30) * max_factor
    assert m <= lim, "%s: max abs error %.3e > %.3e" % (what, m, lim)
