"""Helpers shared by the GPU parity tests (host<->device marshalling, error metric)."""
import numpy as np
import torch

from paper_2502_18394_amd import synth

TOL = {"f32": 1e-5, "bf16": 2e-2}   # relative L2 bars: fp32 I/O, bf16 I/O


def rel_l2(a, b):
    a = np.asarray(a).astype(np.complex128 if np.iscomplexobj(a) or np.iscomplexobj(b) else np.float64)
    b = np.asarray(b).astype(a.dtype)
    return float(np.linalg.norm((a - b).ravel()) / max(np.linalg.norm(b.ravel()), 1e-300))


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
