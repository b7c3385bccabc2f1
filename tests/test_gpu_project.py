"""GPU parity of spectre_project against the fp64 oracle (Sec. 3.2 step 1, Eq. 2, per head)."""
import numpy as np
import pytest
import torch

from gpu_util import TOL, from_device, rel_l2, to_device
from paper_2502_18394_amd import synth

pytestmark = pytest.mark.gpu


def _weights(seed, Hw, d=64, std=0.125):
    rng = np.random.default_rng(seed)
    return ((std * rng.standard_normal((Hw, d, d))).astype(np.float32),
            (std * rng.standard_normal((Hw, d, d))).astype(np.float32))


@pytest.mark.parametrize("B,L,H,io,shared,want_q", [
    (1, 1024, 1, "f32", False, True), (2, 300, 3, "f32", True, False), (1, 8192, 32, "bf16", False, False),
    (3, 1, 2, "f32", False, True), (2, 2500, 5, "bf16", False, True), (4, 196, 12, "f32", False, False)])
def test_project_matches_oracle(oracle, B, L, H, io, shared, want_q):
    from paper_2502_18394_amd import binding
    print(f"case B={B} L={L} H={H} io={io} shared={shared} want_q={want_q}", flush=True)
    vals, store = synth.tokens(80 + L, (B, L, H, 64), io)
    Wq, Wv = _weights(81 + L, 1 if shared else H)
    v, q, sq = binding.project(to_device(store, io), torch.from_numpy(Wq).cuda(), torch.from_numpy(Wv).cuda(), want_q=want_q)
    torch.cuda.synchronize()
    Qo, Vo = oracle.project(vals.astype(np.float64), Wq.astype(np.float64), Wv.astype(np.float64))
    e_v = rel_l2(from_device(v), Vo)
    e_s = rel_l2(sq.cpu().numpy(), oracle.pool_q(Qo))
    print(f"  V {e_v:.3e}  sum_q {e_s:.3e}", flush=True)
    assert e_v <= TOL[io]
    assert e_s <= 1e-5          # pooled in fp64 from exactly represented inputs; weights are fp32
    if want_q:
        assert q is not None and rel_l2(from_device(q), Qo) <= TOL[io]
    else:
        assert q is None


def _seeded_project_cases():
    rng = np.random.default_rng(synth.BASE_SEED + 980)
    return [(int(rng.integers(1, 4)), int(rng.integers(1, 3000)), int(rng.integers(1, 9)),
             "bf16" if rng.integers(0, 2) else "f32", bool(rng.integers(0, 2)), bool(rng.integers(0, 2)))
            for _ in range(10)]


@pytest.mark.parametrize("B,L,H,io,shared,want_q", _seeded_project_cases())
def test_project_seeded_shapes(oracle, B, L, H, io, shared, want_q):
    test_project_matches_oracle(oracle, B, L, H, io, shared, want_q)


def test_projection_feeds_gate_and_mixer(oracle):
    """x -> (V, sum_q) -> gate -> mixer equals the oracle's project -> pool -> gate -> mix."""
    from gpu_util import f64
    from paper_2502_18394_amd import binding
    B, L, H, d = 1, 4096, 4, 64
    vals, store = synth.tokens(90, (B, L, H, d), "f32")
    Wq, Wv = _weights(91, H)
    p = synth.gate_params(92, H, d, L)
    P = binding.GateParams(p)
    v, _, sq = binding.project(to_device(store, "f32"), torch.from_numpy(Wq).cuda(), torch.from_numpy(Wv).cuda())
    g = binding.gate(sq, P, 1.0 / L, pooled=True)
    out = binding.mix_forward(v, g)
    torch.cuda.synchronize()
    Qo, Vo = oracle.project(vals.astype(np.float64), Wq.astype(np.float64), Wv.astype(np.float64))
    want = oracle.mix_forward(Vo, oracle.gate(oracle.pool_q(Qo), 1.0 / L, f64(p), L))
    assert rel_l2(out.cpu().numpy(), want) <= 1e-5
