"""GPU parity of the persistent memory extension of the Prefix-FFT cache (Sec. 3.4) against the fp64 oracle."""
import numpy as np
import pytest
import torch

from gpu_util import TOL, f64, from_device, rel_l2, to_device
from paper_2502_18394_amd import synth

pytestmark = pytest.mark.gpu


def _memory(seed, Bm, H, N_mem, d=64):
    return np.random.default_rng(seed).standard_normal((Bm, H, N_mem, d)).astype(np.float32)


def _assert_state(c, oc, tag):
    spec = rel_l2(c.prefix_fft.cpu().numpy(), oc.spec)
    sq = rel_l2(c.sum_q.cpu().numpy(), oc.sum_q) if np.abs(oc.sum_q).max() > 0 else float(np.abs(c.sum_q.cpu().numpy()).max())
    vb = float(np.abs(c.v_buf.cpu().numpy() - oc.v_buf).max())
    qb = float(np.abs(c.q_buf.cpu().numpy() - oc.q_buf).max())
    print(f"  {tag}: t={c.t} spec={spec:.3e} sum_q={sq:.3e} v_buf={vb} q_buf={qb}", flush=True)
    assert c.t == oc.t and spec <= 1e-5 and sq <= 1e-12 and vb == 0 and qb == 0


@pytest.mark.parametrize("N_mem,N_max,T0,steps,io,shared", [(16, 240, 100, 520, "f32", False), (64, 960, 0, 60, "bf16", True),
                                                             (32, 480, 480, 30, "f32", True), (64, 4032, 1000, 12, "bf16", False),
                                                             (255, 1, 0, 6, "f32", False), (0, 256, 100, 300, "f32", True)])
def test_memory_cache_tracks_the_oracle(oracle, N_mem, N_max, T0, steps, io, shared):
    from paper_2502_18394_amd import binding
    B, H, d = 2, 2, 64
    print(f"case N_mem={N_mem} N_max={N_max} T0={T0} steps={steps} io={io} shared={shared}", flush=True)
    M = _memory(500 + N_mem, 1 if shared else B, H, N_mem)
    Mfull = np.broadcast_to(M, (B, H, N_mem, d)).astype(np.float64)
    c = binding.PrefixCache(B, H, d, N_max, N_mem=N_mem)
    if N_mem:                                   # N_mem = 0: the plain cache through the same code path
        c.set_memory(torch.from_numpy(M).cuda())
    oc = oracle.MemoryPrefixCache(B, H, d, N_mem, N_max)
    seed = 510 + N_max
    if T0:
        v, vs = synth.tokens(seed, (B, T0, H, d), io)
        q, qs = synth.tokens(seed + 1, (B, T0, H, d), io)
        c.update(to_device(vs, io), to_device(qs, io))
        oc.prefill(Mfull, v.astype(np.float64), q.astype(np.float64))
    else:
        oc.prefill(Mfull)
    _assert_state(c, oc, "set-up")
    v, vs = synth.tokens(seed + 2, (B, steps, H, d), io)
    q, qs = synth.tokens(seed + 3, (B, steps, H, d), io)
    checkpoints = {0, 1, steps // 2, steps - 1}
    for i in range(steps):
        c.update(to_device(np.ascontiguousarray(vs[:, i:i + 1]), io), to_device(np.ascontiguousarray(qs[:, i:i + 1]), io))
        oc.update(v[:, i:i + 1].astype(np.float64), q[:, i:i + 1].astype(np.float64))
        if i in checkpoints:
            _assert_state(c, oc, f"step {i}")
    assert np.array_equal(c.v_buf.cpu().numpy()[:, :, :N_mem], np.broadcast_to(M, (B, H, N_mem, d)))


@pytest.mark.parametrize("N_mem,N_max,T,io", [(16, 240, 90, "f32"), (16, 240, 700, "f32"), (64, 960, 960, "bf16"),
                                              (32, 16352, 300, "f32"),
                                              (255, 1, 40, "f32"),     # 39 appended tokens that all hit the one ring slot
                                              (16, 240, 440, "f32")])   # 200 appended at once: window re-transformed
def test_memory_readouts_match_oracle(oracle, N_mem, N_max, T, io):
    from paper_2502_18394_amd import binding
    B, H, d = 2, 3, 64
    print(f"case N_mem={N_mem} N_max={N_max} T={T} io={io}", flush=True)
    M = _memory(520 + N_mem, B, H, N_mem)
    c = binding.PrefixCache(B, H, d, N_max, N_mem=N_mem)
    c.set_memory(torch.from_numpy(M).cuda())
    oc = oracle.MemoryPrefixCache(B, H, d, N_mem, N_max)
    T0 = min(T, N_max)
    v, vs = synth.tokens(521, (B, T, H, d), "f32")
    q, qs = synth.tokens(522, (B, T, H, d), "f32")
    c.update(to_device(np.ascontiguousarray(vs[:, :T0]), "f32"), to_device(np.ascontiguousarray(qs[:, :T0]), "f32"))
    oc.prefill(M.astype(np.float64), v[:, :T0].astype(np.float64), q[:, :T0].astype(np.float64))
    if T > T0:
        c.update(to_device(np.ascontiguousarray(vs[:, T0:]), "f32"), to_device(np.ascontiguousarray(qs[:, T0:]), "f32"))
        for i in range(T0, T):
            oc.update(v[:, i:i + 1].astype(np.float64), q[:, i:i + 1].astype(np.float64))
    n = N_mem + N_max
    g = synth.random_gate(523, B, H, n)
    gd = torch.from_numpy(g).cuda()
    dt = torch.bfloat16 if io == "bf16" else torch.float32
    new = from_device(c.readout(gd, binding.READ_NEWEST, dtype=dt))
    win = from_device(c.readout(gd, binding.READ_WINDOW, dtype=dt))
    torch.cuda.synchronize()
    want_new = oc.readout_newest(g.astype(np.complex128))
    want_win = oc.readout_window(g.astype(np.complex128))
    e1, e2 = rel_l2(new, want_new), rel_l2(win, want_win)
    print(f"  newest {e1:.3e}  window {e2:.3e} rows {win.shape[1]}", flush=True)
    assert win.shape == want_win.shape
    assert e1 <= TOL[io] and e2 <= TOL[io]
    if io == "f32":
        assert rel_l2(win[:, -1:], new) <= 1e-5          # the window's last row is the newest token's row


def test_memory_fused_step_matches_unfused_and_oracle(oracle):
    from paper_2502_18394_amd import binding
    B, H, d, N_mem, N_max = 2, 2, 64, 32, 480
    n = N_mem + N_max
    M = _memory(530, 1, H, N_mem)
    p = synth.gate_params(531, H, d, n)
    P = binding.GateParams(p)
    c = binding.PrefixCache(B, H, d, N_max, N_mem=N_mem)
    c.set_memory(torch.from_numpy(M).cuda())
    oc = oracle.MemoryPrefixCache(B, H, d, N_mem, N_max)
    oc.prefill(np.broadcast_to(M, (B, H, N_mem, d)).astype(np.float64))
    v, vs = synth.tokens(532, (B, 520, H, d), "f32")
    q, qs = synth.tokens(533, (B, 520, H, d), "f32")
    worst = 0.0
    for i in range(520):
        out = c.step(to_device(np.ascontiguousarray(vs[:, i:i + 1]), "f32"), to_device(np.ascontiguousarray(qs[:, i:i + 1]), "f32"), P)
        oc.update(v[:, i:i + 1].astype(np.float64), q[:, i:i + 1].astype(np.float64))
        if i in (0, 1, 100, 479, 480, 481, 519):
            g = oracle.gate(oc.sum_q, 1.0 / N_max, f64(p), n, 0)           # divisor stays 1/N_max
            want = oc.readout_newest(g)
            err = rel_l2(from_device(out), want)
            worst = max(worst, err)
            print(f"  step {i}: {err:.3e}", flush=True)
    assert worst <= 1e-5
    assert rel_l2(c.prefix_fft.cpu().numpy(), oc.spec) <= 1e-5


def test_memory_argument_checks():
    from paper_2502_18394_amd import binding
    with pytest.raises(binding.SpectreError) as e:
        binding.PrefixCache(1, 1, 64, 250, N_mem=16)                      # 266 is not a supported window
    assert e.value.code == binding.EUNSUPPORTED
    c = binding.PrefixCache(1, 2, 64, 256)                                # no memory rows
    with pytest.raises(binding.SpectreError) as e:
        c.set_memory(torch.zeros((1, 2, 0, 64), device="cuda"))
    assert e.value.code == binding.EINVAL
    c = binding.PrefixCache(1, 2, 64, 240, N_mem=16)
    x = torch.zeros((1, 1, 2, 64), device="cuda")
    c.update(x, x)
    with pytest.raises(binding.SpectreError) as e:                         # not after tokens have been appended
        c.set_memory(torch.zeros((1, 2, 16, 64), device="cuda"))
    assert e.value.code == binding.EINVAL
    c = binding.PrefixCache(1, 2, 64, 240, N_mem=16)
    with pytest.raises(binding.SpectreError) as e:                         # prompt longer than the ring
        c.update(torch.zeros((1, 241, 2, 64), device="cuda"), torch.zeros((1, 241, 2, 64), device="cuda"))
    assert e.value.code == binding.EINVAL
