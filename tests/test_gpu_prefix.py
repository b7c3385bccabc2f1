"""GPU parity of the Prefix-FFT cache entry points against the fp64 oracle (Sec. 3.3, Alg. 1)."""
import numpy as np
import pytest
import torch

from gpu_util import TOL, f64, from_device, rel_l2, to_device
from paper_2502_18394_amd import synth

pytestmark = pytest.mark.gpu


def _state_errors(c, oc):
    spec = c.prefix_fft.cpu().numpy()
    return dict(spec=rel_l2(spec, oc.spec), sum_q=rel_l2(c.sum_q.cpu().numpy(), oc.sum_q),
                v_buf=float(np.abs(c.v_buf.cpu().numpy() - oc.v_buf).max()),
                q_buf=float(np.abs(c.q_buf.cpu().numpy() - oc.q_buf).max()))


def _assert_state(c, oc, tag):
    e = _state_errors(c, oc)
    print(f"  {tag}: t={c.t} {e}", flush=True)
    assert c.t == oc.t
    assert e["spec"] <= 1e-5 and e["sum_q"] <= 1e-12 and e["v_buf"] == 0 and e["q_buf"] == 0


@pytest.mark.parametrize("N,T0,steps,io", [(256, 100, 560, "f32"), (256, 0, 300, "bf16"), (512, 512, 40, "f32"),
                                           (768, 500, 300, "f32"), (12288, 12000, 300, "bf16"),
                                           (4096, 1000, 20, "bf16"), (16384, 16384, 6, "f32")])
def test_prefill_then_updates_track_the_oracle(oracle, N, T0, steps, io):
    from paper_2502_18394_amd import binding
    B, H, d = 2, 2, 64
    print(f"case N={N} T0={T0} steps={steps} io={io}", flush=True)
    c = binding.PrefixCache(B, H, d, N)
    oc = oracle.PrefixCache(B, H, d, N)
    seed = synth.BASE_SEED + N
    if T0:
        v, vs = synth.tokens(seed, (B, T0, H, d), io)
        q, qs = synth.tokens(seed + 1, (B, T0, H, d), io)
        c.update(to_device(vs, io), to_device(qs, io))
        oc.prefill(v.astype(np.float64), q.astype(np.float64))
        _assert_state(c, oc, "prefill")
    v, vs = synth.tokens(seed + 2, (B, steps, H, d), io)
    q, qs = synth.tokens(seed + 3, (B, steps, H, d), io)
    checkpoints = {0, 1, steps // 2, steps - 1}
    for i in range(steps):
        c.update(to_device(np.ascontiguousarray(vs[:, i:i + 1]), io), to_device(np.ascontiguousarray(qs[:, i:i + 1]), io))
        oc.update(v[:, i:i + 1].astype(np.float64), q[:, i:i + 1].astype(np.float64))
        if i in checkpoints:
            _assert_state(c, oc, f"step {i}")


def test_multi_token_append_equals_single_steps(oracle):
    from paper_2502_18394_amd import binding
    B, H, d, N = 1, 3, 64, 256
    v, vs = synth.tokens(5, (B, 300, H, d), "f32")
    q, qs = synth.tokens(6, (B, 300, H, d), "f32")
    c = binding.PrefixCache(B, H, d, N)
    oc = oracle.PrefixCache(B, H, d, N)
    c.update(to_device(np.ascontiguousarray(vs[:, :1]), "f32"), to_device(np.ascontiguousarray(qs[:, :1]), "f32"))
    c.update(to_device(np.ascontiguousarray(vs[:, 1:]), "f32"), to_device(np.ascontiguousarray(qs[:, 1:]), "f32"))
    for i in range(300):
        oc.update(v[:, i:i + 1].astype(np.float64), q[:, i:i + 1].astype(np.float64))
    _assert_state(c, oc, "after 1 + 299 tokens")


@pytest.mark.parametrize("N,T0,appends,io", [
    (512, 500, (2, 31, 32, 33, 64, 5), "f32"),      # batches of every size around the 32 tokens one sweep takes
    (768, 700, (100, 7), "bf16"),                   # window length with an odd factor, wraps and evicts
    (4096, 0, (1, 40, 3), "f32"),                   # from an empty cache: a single token first, then batches
    (512, 500, (200, 512, 160, 3, 159), "f32"),     # 160 tokens or more: ring buffers in one pass, window re-transformed
    (768, 100, (300, 768, 33), "bf16"),             # the same on a window with an odd factor, up to the ring capacity
    (256, 200, (300,), "f32"),                      # more tokens than the ring holds: 32 per sweep again
])
def test_appends_of_several_tokens_go_in_with_one_sweep_per_32(oracle, N, T0, appends, io):
    """Eq. 5 for T tokens at once (after the pre-fill): the library applies up to 32 rank-one terms per sweep over
    the cache, or, from 160 tokens on, updates the ring buffers in one pass and transforms the window afresh; the
    oracle applies the tokens one by one."""
    from paper_2502_18394_amd import binding
    B, H, d = 2, 2, 64
    print(f"case N={N} T0={T0} appends={appends} io={io}", flush=True)
    c = binding.PrefixCache(B, H, d, N)
    oc = oracle.PrefixCache(B, H, d, N)
    if T0:
        v, vs = synth.tokens(40, (B, T0, H, d), io)
        q, qs = synth.tokens(41, (B, T0, H, d), io)
        c.update(to_device(vs, io), to_device(qs, io))
        oc.prefill(v.astype(np.float64), q.astype(np.float64))
    for j, T in enumerate(appends):
        v, vs = synth.tokens(42 + 2 * j, (B, T, H, d), io)
        q, qs = synth.tokens(43 + 2 * j, (B, T, H, d), io)
        c.update(to_device(vs, io), to_device(qs, io))
        for i in range(T):
            oc.update(v[:, i:i + 1].astype(np.float64), q[:, i:i + 1].astype(np.float64))
        _assert_state(c, oc, f"after an append of {T}")


@pytest.mark.parametrize("N,T,io", [(256, 90, "f32"), (256, 700, "f32"), (1024, 1024, "bf16"), (16384, 300, "f32"),
                                    (1280, 1500, "f32"), (7168, 7000, "bf16")])
def test_readouts_match_oracle(oracle, N, T, io):
    from paper_2502_18394_amd import binding
    B, H, d = 2, 3, 64
    print(f"case N={N} T={T} io={io}", flush=True)
    c = binding.PrefixCache(B, H, d, N)
    oc = oracle.PrefixCache(B, H, d, N)
    T0 = min(T, N)
    v, vs = synth.tokens(31, (B, T, H, d), "f32")
    q, qs = synth.tokens(32, (B, T, H, d), "f32")
    c.update(to_device(np.ascontiguousarray(vs[:, :T0]), "f32"), to_device(np.ascontiguousarray(qs[:, :T0]), "f32"))
    oc.prefill(v[:, :T0].astype(np.float64), q[:, :T0].astype(np.float64))
    if T > T0:
        c.update(to_device(np.ascontiguousarray(vs[:, T0:]), "f32"), to_device(np.ascontiguousarray(qs[:, T0:]), "f32"))
        for i in range(T0, T):
            oc.update(v[:, i:i + 1].astype(np.float64), q[:, i:i + 1].astype(np.float64))
    p = synth.gate_params(33, H, d, N)
    P = binding.GateParams(p)
    dt = torch.float32 if io == "f32" else torch.bfloat16
    # NEWEST with the un-phased decode gate
    g0 = binding.gate(c.sum_q, P, 1.0 / N, pooled=True)
    og0 = oracle.gate(oc.sum_q, 1.0 / N, f64(p), N, 0)
    got = from_device(c.readout(g0, binding.READ_NEWEST, dt))
    want = oc.readout_newest(og0)
    e1 = rel_l2(got, want)
    # WINDOW with phase p = t
    g1 = binding.gate(c.sum_q, P, 1.0 / N, pooled=True, phase_pos=c.t)
    og1 = oracle.gate(oc.sum_q, 1.0 / N, f64(p), N, oc.t)
    gotw = from_device(c.readout(g1, binding.READ_WINDOW, dt))
    wantw = oc.readout_window(og1)
    e2 = rel_l2(gotw, wantw)
    print(f"  newest {e1:.3e}  window {e2:.3e}", flush=True)
    assert gotw.shape == wantw.shape == (B, min(T, N), H, d)
    assert e1 <= TOL[io] and e2 <= TOL[io]
    # last window row is the newest row
    assert rel_l2(gotw[:, -1], got[:, 0]) <= (1e-5 if io == "f32" else 2e-2)


@pytest.mark.parametrize("N,T0,steps,io", [(256, 200, 120, "f32"), (2048, 2048, 24, "bf16")])
def test_fused_step_matches_update_gate_readout(oracle, N, T0, steps, io):
    from paper_2502_18394_amd import binding
    B, H, d = 2, 4, 64
    c = binding.PrefixCache(B, H, d, N)
    oc = oracle.PrefixCache(B, H, d, N)
    v, vs = synth.tokens(41, (B, T0, H, d), io)
    q, qs = synth.tokens(42, (B, T0, H, d), io)
    c.update(to_device(vs, io), to_device(qs, io))
    oc.prefill(v.astype(np.float64), q.astype(np.float64))
    p = synth.gate_params(43, H, d, N)
    P = binding.GateParams(p)
    v, vs = synth.tokens(44, (B, steps, H, d), io)
    q, qs = synth.tokens(45, (B, steps, H, d), io)
    worst = 0.0
    for i in range(steps):
        out = c.step(to_device(np.ascontiguousarray(vs[:, i:i + 1]), io), to_device(np.ascontiguousarray(qs[:, i:i + 1]), io), P)
        oc.update(v[:, i:i + 1].astype(np.float64), q[:, i:i + 1].astype(np.float64))
        want = oc.readout_newest(oracle.gate(oc.sum_q, 1.0 / N, f64(p), N, 0))
        worst = max(worst, rel_l2(from_device(out), want))
    print(f"  worst step error {worst:.3e}", flush=True)
    assert worst <= TOL[io]
    _assert_state(c, oc, "after fused steps")
