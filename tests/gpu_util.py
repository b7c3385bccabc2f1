"""Helpers shared by the GPU parity tests (host<->device marshalling, error metric)."""
import numpy as np
import torch

from paper_2502_18394_amd import synth

TOL = {"f32": 1e-5, "bf16": 2e-2}   # relative L2 bars: fp32 I/O, bf16 I/O


def rel_l2(a, b):
    a = np.asarray(a).astype(np.complex128 if np.iscomplexobj(a) or np.iscomplexobj(b) else np.float64)
    b = np.asarray(b).astype(a.dtype)
    return float(np.linalg.norm((a - b).ravel()) / max(np.linalg.norm(b.ravel()), 1e-300))


def assert_close_elementwise(got, want, io, n):
    """Per-element bound on top of the relative-L2 bars, for an n-point transform pair.
    fp32 rows: |got - want| <= 16 * 2^-24 * log2(n) * rms(want): a few times the rounding error that log2(n)
    butterfly stages each way accumulate in fp32 (observed maxima sit near 1 * 2^-24 * log2(n) * rms), so a single
    wrong element far below the whole-tensor bar still fails.
    bf16 rows: one bf16 step of the oracle value (the output rounding) plus the same fp32 term."""
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    rms = float(np.sqrt(np.mean(want ** 2)))
    tol = 16.0 * 2.0 ** -24 * max(np.log2(max(n, 2)), 1.0) * rms
    if io == "bf16":
        tol = np.abs(want) * 2.0 ** -7 + tol
    bad = np.abs(got - want) > tol
    assert not bad.any(), (f"{int(bad.sum())} of {bad.size} elements outside the per-element bound; worst "
                           f"|err| {float(np.abs(got - want).max()):.3e}, rms {rms:.3e}")


def to_device(store, io):
    if io == "bf16":
        return torch.from_numpy(store.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(store).cuda()


def from_device(t):
    if t.dtype == torch.bfloat16:
        return synth.bf16_bits_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16))
    return t.cpu().numpy()


def f64(params):
    def up(v):
        if not isinstance(v, np.ndarray):
            return v
        return v.astype(np.complex128 if np.iscomplexobj(v) else np.float64)
    return {k: up(v) for k, v in params.items()}
