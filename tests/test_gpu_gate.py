"""GPU parity of spectre_gate against the fp64 oracle (Sec. 3.2 step 3; Sec. 3.5 phase)."""
import numpy as np
import pytest
import torch

from gpu_util import TOL, f64, rel_l2, to_device
from paper_2502_18394_amd import synth

pytestmark = pytest.mark.gpu


def run_gate(oracle, B, L, H, d, dg, n, io, shared=False, modrelu=True, phase=0, seed=1, std=0.02, bias_shift=0.0):
    from paper_2502_18394_amd import binding
    p = synth.gate_params(seed, 1 if shared else H, d, n, d_g=dg, modrelu=modrelu, std=std)
    if bias_shift:
        p["modrelu_bias"] = (p["modrelu_bias"] + np.float32(bias_shift)).astype(np.float32)
    vals, store = synth.tokens(seed + 1, (B, L, H, d), io)
    P = binding.GateParams(p)
    g = binding.gate(to_device(store, io), P, 1.0 / L, phase_pos=phase)
    torch.cuda.synchronize()
    want = oracle.gate(oracle.pool_q(vals.astype(np.float64)), 1.0 / L, f64(p), n, phase)
    return g.cpu().numpy(), want


@pytest.mark.parametrize("B,L,H,d,dg,io,shared", [
    (1, 1024, 1, 64, 64, "f32", False),      # config 1
    (1, 8192, 32, 64, 64, "bf16", False),    # config 2 shape
    (3, 512, 5, 64, 64, "f32", True),        # shared weights, 15 rows on the MFMA column side
    (40, 256, 1, 64, 64, "f32", False),      # more than 32 rows: two row tiles
    (5, 256, 12, 64, 64, "bf16", True),      # shared, 60 rows
    (4, 196, 12, 64, 64, "f32", False),      # ViT length: 2F = 198, ragged last tile
    (2, 300, 3, 32, 48, "f32", False),       # other d, d_g not a multiple of 16, odd chunking
    (1, 7, 2, 8, 5, "f32", False),           # tiny everything, odd n
])
def test_gate_matches_oracle(oracle, B, L, H, d, dg, io, shared):
    print(f"case B={B} L={L} H={H} d={d} dg={dg} io={io} shared={shared}", flush=True)
    got, want = run_gate(oracle, B, L, H, d, dg, L, io, shared=shared)
    err = rel_l2(got, want)
    print(f"  rel_l2={err:.3e}", flush=True)
    assert err <= 1e-5   # the gate is fp32 throughout; bf16 only affects the (exactly represented) inputs


def test_gate_large_std_exercises_modrelu_threshold(oracle):
    got, want = run_gate(oracle, 2, 256, 3, 64, 64, 256, "f32", std=0.5, seed=5, bias_shift=-2.0)
    assert rel_l2(got, want) <= 1e-5
    assert (np.abs(want) == 0).any() and (np.abs(want) > 0).any()
    np.testing.assert_array_equal(np.abs(got) == 0, np.abs(want) == 0)


def test_gate_without_modrelu_and_with_phase(oracle):
    got, want = run_gate(oracle, 2, 512, 2, 64, 64, 512, "f32", modrelu=False, phase=777, seed=9)
    assert rel_l2(got, want) <= 1e-5


def test_gate_from_pooled_sum_decode_form(oracle):
    from paper_2502_18394_amd import binding
    B, H, d, N = 3, 4, 64, 4096
    p = synth.gate_params(11, H, d, N)
    sq = np.random.default_rng(12).standard_normal((B, H, d)) * 40.0
    P = binding.GateParams(p)
    for phase in (0, 4097, 123456789):
        g = binding.gate(torch.from_numpy(sq).cuda(), P, 1.0 / N, pooled=True, phase_pos=phase)
        want = oracle.gate(sq, 1.0 / N, f64(p), N, phase)
        assert rel_l2(g.cpu().numpy(), want) <= 1e-5


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_pooling_kernels_agree_whatever_the_alignment(io):
    """Rows that start on a 16-byte boundary are pooled with 16-byte loads, others pair by pair; both add the rows of
    a channel in the same order, so the gates must be identical bit for bit."""
    from paper_2502_18394_amd import binding
    B, L, H, d = 2, 1000, 3, 64
    P = binding.GateParams(synth.gate_params(31, H, d, L))
    _, store = synth.tokens(32, (B, L, H, d), io)
    q = to_device(store, io)
    shift = 2                                             # elements: 8 bytes (fp32), 4 bytes (bf16)
    flat = torch.empty(q.numel() + shift, dtype=q.dtype, device="cuda")
    q_off = flat[shift:].view(B, L, H, d)
    q_off.copy_(q)
    assert q.data_ptr() % 16 == 0 and q_off.data_ptr() % 16 != 0
    a = binding.gate(q, P, 1.0 / L)
    b = binding.gate(q_off, P, 1.0 / L)
    torch.cuda.synchronize()
    assert torch.equal(torch.view_as_real(a), torch.view_as_real(b))


def test_pooling_of_long_sequence_is_accurate(oracle):
    """128k rows: the pooled mean is ~0.003 and LayerNorm rescales it to O(1), so the sum must be tight."""
    got, want = run_gate(oracle, 1, 131072, 2, 64, 64, 1024, "bf16", seed=21)
    assert rel_l2(got, want) <= 1e-5


@pytest.mark.parametrize("B,L,H,r,shared,modrelu", [(2, 512, 3, 2, False, True), (1, 196, 4, 8, True, True),
                                                     (3, 1024, 2, 0, False, False), (1, 8192, 32, 4, False, True)])
def test_gate_with_toeplitz_update(oracle, B, L, H, r, shared, modrelu):
    """Sec. 3.2 step 3b between the MLP and modReLU."""
    from paper_2502_18394_amd import binding
    d, dg = 64, 64
    Hg = 1 if shared else H
    p = synth.gate_params(50 + r, Hg, d, L, d_g=dg, modrelu=modrelu, std=0.1)
    p["toeplitz"] = synth.toeplitz_taps(60 + r, Hg, r, std=0.3)
    vals, store = synth.tokens(70 + r, (B, L, H, d), "f32")
    P = binding.GateParams(p)
    g = binding.gate(to_device(store, "f32"), P, 1.0 / L, phase_pos=5 if r == 2 else 0)
    torch.cuda.synchronize()
    p64 = f64(p)
    p64["toeplitz"] = p["toeplitz"].astype(np.complex128)
    want = oracle.gate(oracle.pool_q(vals.astype(np.float64)), 1.0 / L, p64, L, 5 if r == 2 else 0)
    err = rel_l2(g.cpu().numpy(), want)
    print(f"  r={r} rel_l2={err:.3e}", flush=True)
    assert err <= 1e-5
    # and it does something: differs from the gate without taps
    p_plain = {k: v for k, v in p64.items() if k != "toeplitz"}
    plain = oracle.gate(oracle.pool_q(vals.astype(np.float64)), 1.0 / L, p_plain, L, 5 if r == 2 else 0)
    assert rel_l2(want, plain) > 1e-3


def _seeded_gate_cases():
    rng = np.random.default_rng(synth.BASE_SEED + 950)
    cases = []
    for _ in range(14):
        B = int(rng.integers(1, 70))
        H = int(rng.integers(1, 6))
        L = int(rng.integers(1, 700))
        d = 2 * int(rng.integers(1, 129))                     # 2 .. 256, even
        dg = int(rng.integers(1, 257))
        n = int(rng.integers(2, 3000))                        # transform length of the gate (even or odd)
        cases.append((B, L, H, d, dg, n, "bf16" if rng.integers(0, 2) else "f32", bool(rng.integers(0, 2)),
                      bool(rng.integers(0, 2)), int(rng.integers(0, 5000)) if rng.integers(0, 2) else 0))
    return cases


@pytest.mark.parametrize("B,L,H,d,dg,n,io,shared,modrelu,phase", _seeded_gate_cases())
def test_gate_seeded_shapes(oracle, B, L, H, d, dg, n, io, shared, modrelu, phase):
    """Channel counts, hidden widths, row counts and transform lengths drawn at random (seeded): every tiling tail of
    the pooling, hidden and output kernels."""
    print(f"case B={B} L={L} H={H} d={d} dg={dg} n={n} io={io} shared={shared} modrelu={modrelu} phase={phase}", flush=True)
    got, want = run_gate(oracle, B, L, H, d, dg, n, io, shared=shared, modrelu=modrelu, phase=phase, seed=960 + B + L)
    err = rel_l2(got, want)
    print(f"  rel_l2={err:.3e}", flush=True)
    assert err <= 1e-5
