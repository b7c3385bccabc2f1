"""spectre_layer_forward (projection, pooled query, gate, mixer and the optional wavelet refinement in one call)
against the oracle's functions chained, Sec. 3.2 steps 1-4 and Sec. 3.5, and against the library's own separate calls.

On the four-step route with bf16 rows the call projects inside the row transforms (V never exists in memory) and
feeds the refinement from block sums the mixer emits; every other shape runs the separate kernels with V in the
workspace.  The oracle side adds no arithmetic: project -> pool -> gate -> mix -> level gates -> refinement."""
import numpy as np
import pytest
import torch

from gpu_util import TOL, f64, from_device, rel_l2, to_device
from paper_2502_18394_amd import synth

pytestmark = pytest.mark.gpu


def oracle_chain(oracle, x, Wq, Wv, p, wp, J):
    B, L, H, d = x.shape
    Q, V = oracle.project(x, Wq, Wv)
    sum_q = oracle.pool_q(Q)
    g = oracle.gate(sum_q, 1.0 / L, p, L, 0)
    out = oracle.mix_forward(V, g)
    if wp is not None:
        out = oracle.wrm_apply(out, oracle.wrm_gates(sum_q, 1.0 / L, wp, J), J)
    return out


def run_layer(oracle, B, L, H, io, J, seed, Hw=None):
    from paper_2502_18394_amd import binding
    d = 64
    Hw = H if Hw is None else Hw
    vals, store = synth.tokens(seed, (B, L, H, d), io)
    rng = np.random.default_rng(seed + 1)
    Wq = (0.125 * rng.standard_normal((Hw, d, d))).astype(np.float32)
    Wv = (0.125 * rng.standard_normal((Hw, d, d))).astype(np.float32)
    p = synth.gate_params(seed + 2, H, d, L)
    wp = synth.wrm_params(seed + 3, H, d, J) if J is not None else None
    P = binding.GateParams(p)
    W = binding.WrmParams(wp) if wp is not None else None
    x_d = to_device(store, io)
    Wq_d, Wv_d = torch.from_numpy(Wq).cuda(), torch.from_numpy(Wv).cuda()
    out = binding.layer_forward(x_d, Wq_d, Wv_d, P, W)
    # the same chain through the separate entry points
    v, _, sq = binding.project(x_d, Wq_d, Wv_d)
    g = binding.gate(sq, P, 1.0 / L, pooled=True)
    ref = binding.mix_forward(v, g)
    if W is not None:
        ref = binding.wrm_apply(ref, binding.wrm_gates(sq, W, 1.0 / L, pooled=True))
    torch.cuda.synchronize()
    bq = Wq if Hw == H else np.broadcast_to(Wq, (H, d, d))
    bv = Wv if Hw == H else np.broadcast_to(Wv, (H, d, d))
    want = oracle_chain(oracle, vals.astype(np.float64), bq.astype(np.float64), bv.astype(np.float64), f64(p),
                        f64(wp) if wp is not None else None, J)
    return from_device(out), from_device(ref), want


# four-step lengths, bf16 rows: the fused route.  N1 = 256 and 4096, even and odd N2 (3 * 256: 48 tile rows, a ragged
# last group of the matrix-core prologue), one and several head groups, shared projection weights, refinement depths
# below and above the 8 levels a tile holds.
@pytest.mark.parametrize("B,L,H,J,Hw", [(1, 8192, 8, None, None), (2, 8192, 3, 13, None), (1, 16384, 5, 6, None),
                                         (1, 768, 2, 8, None), (1, 12288, 2, 12, 1), (1, 32768, 4, 15, None),
                                         (1, 131072, 2, 17, None), (3, 2560, 2, 9, None), (1, 7168, 1, None, 1)])
def test_fused_layer_matches_oracle_chain_bf16(oracle, B, L, H, J, Hw):
    print(f"case B={B} L={L} H={H} J={J} Hw={Hw}", flush=True)
    got, ref, want = run_layer(oracle, B, L, H, "bf16", J, seed=synth.BASE_SEED + 500 + L + H, Hw=Hw)
    err, e_ref = rel_l2(got, want), rel_l2(got, ref)
    print(f"  vs oracle chain {err:.3e}  vs separate calls {e_ref:.3e}  differing {np.mean(got != ref):.2e}", flush=True)
    assert err <= TOL["bf16"]
    # same V bits, same kernels behind; the pooled query is summed in another order (1e-7 on the gate), and the
    # refinement's coarse sums are added in another order: a bf16 step here and there
    assert e_ref <= 2e-3 and np.mean(got != ref) < 2e-2


# every other shape runs the separate kernels inside the call: fp32 rows, the in-LDS lengths, 4096, padded lengths
@pytest.mark.parametrize("B,L,H,io,J", [(1, 8192, 2, "f32", 13), (2, 196, 3, "f32", 2), (2, 196, 3, "bf16", None),
                                        (1, 4096, 4, "bf16", 12), (1, 1000, 2, "bf16", 3), (1, 1024, 1, "f32", None),
                                        (1, 512, 32, "bf16", 9)])
def test_layer_on_the_other_routes_matches_oracle_chain(oracle, B, L, H, io, J):
    print(f"case B={B} L={L} H={H} io={io} J={J}", flush=True)
    got, ref, want = run_layer(oracle, B, L, H, io, J, seed=synth.BASE_SEED + 600 + L + H)
    err = rel_l2(got, want)
    print(f"  vs oracle chain {err:.3e}  identical to separate calls {np.array_equal(got, ref)}", flush=True)
    assert err <= (TOL["bf16"] if io == "bf16" else 2e-5)     # fp32: the gate's 1e-5 bar and the mixer's, chained
    assert np.array_equal(got, ref)                           # the very same kernels in the same order


def test_layer_rejects_bad_arguments():
    from paper_2502_18394_amd import binding
    d = 64
    x = torch.zeros((1, 1024, 2, d), device="cuda")
    Wm = torch.zeros((2, d, d), device="cuda")
    P_wrong = binding.GateParams(synth.gate_params(1, 2, d, 512))
    with pytest.raises(binding.SpectreError) as e:
        binding.layer_forward(x, Wm, Wm, P_wrong)              # gate built for another length
    assert e.value.code in (binding.EINVAL, binding.EUNSUPPORTED)
    P = binding.GateParams(synth.gate_params(1, 2, d, 1024))
    W_bad = binding.WrmParams(synth.wrm_params(2, 2, d, 11))   # 2^11 does not divide 1024
    with pytest.raises(binding.SpectreError):
        binding.layer_forward(x, Wm, Wm, P, W_bad)
    with pytest.raises(binding.SpectreError) as e:
        binding.layer_forward(x, Wm, Wm, P, out=x)             # out overlaps x
    assert e.value.code == binding.EINVAL
