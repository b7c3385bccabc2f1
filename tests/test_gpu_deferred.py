"""GPU parity of the fused decode step with deferred rank-one updates (Eq. 5 is linear: pending updates are
accounted for at readout through the gate's convolution kernel and applied to the cache every few steps).
Every step's output is compared with the oracle, which applies Eq. 5 at every token as Algorithm 1 prints it."""
import numpy as np
import pytest
import torch

from gpu_util import TOL, f64, from_device, rel_l2, to_device
from paper_2502_18394_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N_mem,N_max,T0,steps,defer,io", [
    (0, 256, 200, 130, 16, "f32"),      # fills up, wraps, evicts; 8 flushes
    (0, 256, 0, 40, 5, "f32"),          # from an empty cache, odd capacity
    (0, 1024, 1024, 70, 32, "bf16"),    # largest capacity, every step evicts
    (16, 240, 100, 300, 7, "f32"),      # memory rows in front of the ring
    (0, 768, 700, 100, 16, "f32"),      # window length with an odd factor (64-bit index walk)
    (255, 1, 0, 9, 4, "f32"),           # ring of a single slot: every pending token hits the same row
    (0, 256, 100, 20, 1, "f32"),        # capacity 1: every step flushes
    (0, 4096, 4000, 120, 16, "f32"),    # 17 chunks of bins: three workgroups per head in the flush, the last ragged
    (0, 12288, 12280, 30, 8, "bf16"),   # 49 chunks, window length with an odd factor
])
def test_deferred_steps_match_the_oracle_at_every_token(oracle, N_mem, N_max, T0, steps, defer, io):
    from paper_2502_18394_amd import binding
    B, H, d = 2, 3, 64
    n = N_mem + N_max
    print(f"case N_mem={N_mem} N_max={N_max} T0={T0} steps={steps} defer={defer} io={io}", flush=True)
    c = binding.PrefixCache(B, H, d, N_max, N_mem=N_mem, defer=defer)
    oc = oracle.MemoryPrefixCache(B, H, d, N_mem, N_max)
    M = np.random.default_rng(600 + N_mem).standard_normal((B, H, N_mem, d)).astype(np.float32)
    if N_mem:
        c.set_memory(torch.from_numpy(M).cuda())
    if T0:
        v, vs = synth.tokens(601, (B, T0, H, d), io)
        q, qs = synth.tokens(602, (B, T0, H, d), io)
        c.update(to_device(vs, io), to_device(qs, io))
        oc.prefill(M.astype(np.float64), v.astype(np.float64), q.astype(np.float64))
    else:
        oc.prefill(M.astype(np.float64))
    p = synth.gate_params(603, H, d, n)
    P = binding.GateParams(p)
    v, vs = synth.tokens(604, (B, steps, H, d), io)
    q, qs = synth.tokens(605, (B, steps, H, d), io)
    worst, seen_pending = 0.0, set()
    for i in range(steps):
        out = c.step(to_device(np.ascontiguousarray(vs[:, i:i + 1]), io), to_device(np.ascontiguousarray(qs[:, i:i + 1]), io), P)
        oc.update(v[:, i:i + 1].astype(np.float64), q[:, i:i + 1].astype(np.float64))
        want = oc.readout_newest(oracle.gate(oc.sum_q, 1.0 / N_max, f64(p), n, 0))
        err = rel_l2(from_device(out), want)
        worst = max(worst, err)
        seen_pending.add(c.n_pending)
        assert c.n_pending == (i + 1) % defer and c.t == oc.t
    print(f"  worst step error {worst:.3e}; pending counts seen {sorted(seen_pending)}", flush=True)
    assert worst <= TOL[io]
    c.flush()
    assert c.n_pending == 0
    torch.cuda.synchronize()
    assert rel_l2(c.prefix_fft.cpu().numpy(), oc.spec) <= 1e-5
    assert np.array_equal(c.v_buf.cpu().numpy(), oc.v_buf.astype(np.float32))
    assert rel_l2(c.sum_q.cpu().numpy(), oc.sum_q) <= 1e-12


def test_deferred_and_eager_steps_agree_and_other_calls_flush(oracle):
    from paper_2502_18394_amd import binding
    B, H, d, N = 2, 2, 64, 512
    p = synth.gate_params(610, H, d, N)
    P = binding.GateParams(p)
    _, vs = synth.tokens(611, (B, 300, H, d), "f32")
    _, qs = synth.tokens(612, (B, 300, H, d), "f32")
    a, b = binding.PrefixCache(B, H, d, N), binding.PrefixCache(B, H, d, N, defer=16)
    for c in (a, b):
        c.update(to_device(np.ascontiguousarray(vs[:, :200]), "f32"), to_device(np.ascontiguousarray(qs[:, :200]), "f32"))
    for i in range(200, 221):
        x, y = to_device(np.ascontiguousarray(vs[:, i:i + 1]), "f32"), to_device(np.ascontiguousarray(qs[:, i:i + 1]), "f32")
        oa, ob = a.step(x, y, P), b.step(x, y, P)
        assert rel_l2(ob.cpu().numpy(), oa.cpu().numpy()) <= 2e-6
    assert b.n_pending == 21 - 16
    g = torch.from_numpy(synth.random_gate(613, B, H, N)).cuda()
    with pytest.raises(binding.SpectreError) as e:              # a const readout cannot flush
        b.readout(g)
    assert e.value.code == binding.EINVAL and b.n_pending == 5
    b.update(to_device(np.ascontiguousarray(vs[:, 221:230]), "f32"), to_device(np.ascontiguousarray(qs[:, 221:230]), "f32"))
    a.update(to_device(np.ascontiguousarray(vs[:, 221:230]), "f32"), to_device(np.ascontiguousarray(qs[:, 221:230]), "f32"))
    assert b.n_pending == 0 and a.t == b.t                      # an append flushes first
    torch.cuda.synchronize()
    assert rel_l2(b.prefix_fft.cpu().numpy(), a.prefix_fft.cpu().numpy()) <= 2e-6
    for mode in (binding.READ_NEWEST, binding.READ_WINDOW):
        assert rel_l2(b.readout(g, mode).cpu().numpy(), a.readout(g, mode).cpu().numpy()) <= 2e-6


def test_deferred_argument_checks():
    from paper_2502_18394_amd import binding
    c = binding.PrefixCache(1, 1, 64, 256, defer=4)
    c.c.pending_cap = 33
    x = torch.zeros((1, 1, 1, 64), device="cuda")
    with pytest.raises(binding.SpectreError) as e:
        c.update(x, x)
    assert e.value.code == binding.EINVAL
    c.c.pending_cap = 4
    c.c.n_pending = 5
    with pytest.raises(binding.SpectreError) as e:
        c.flush()
    assert e.value.code == binding.EINVAL


@pytest.mark.parametrize("seed,N_mem,N_max,defer", [(0, 0, 256, 0), (1, 0, 256, 16), (2, 16, 240, 5), (3, 0, 768, 32),
                                                     (4, 32, 480, 16), (5, 0, 512, 7)])
def test_random_sequences_of_operations_track_the_oracle(oracle, seed, N_mem, N_max, defer):
    """A seeded mix of everything the cache can be asked to do - fused steps (eager or deferred), appends of 1 to
    N_max tokens (one sweep per token, 32 per sweep, window re-transformed), explicit flushes, both readouts - with
    the oracle applying Eq. 5 token by token beside it; state and outputs are compared after every operation."""
    from paper_2502_18394_amd import binding
    B, H, d = 2, 2, 64
    n = N_mem + N_max
    rng = np.random.default_rng(700 + seed)
    c = binding.PrefixCache(B, H, d, N_max, N_mem=N_mem, defer=defer)
    oc = oracle.MemoryPrefixCache(B, H, d, N_mem, N_max)
    M = rng.standard_normal((B, H, N_mem, d)).astype(np.float32)
    if N_mem:
        c.set_memory(torch.from_numpy(M).cuda())
    oc.prefill(M.astype(np.float64))
    p = synth.gate_params(710 + seed, H, d, n)
    P = binding.GateParams(p)

    def tokens(T):
        v = rng.standard_normal((B, T, H, d)).astype(np.float32)
        q = rng.standard_normal((B, T, H, d)).astype(np.float32)
        return v, q

    def check_state(tag):
        c.flush()
        torch.cuda.synchronize()
        spec = rel_l2(c.prefix_fft.cpu().numpy(), oc.spec)
        sq = rel_l2(c.sum_q.cpu().numpy(), oc.sum_q)
        assert c.t == oc.t and spec <= 1e-5 and sq <= 1e-12, (tag, c.t, oc.t, spec, sq)
        assert np.array_equal(c.v_buf.cpu().numpy(), oc.v_buf.astype(np.float32)), tag

    sizes = [1, 2, 7, 31, 32, 33, 70, 160, 200, N_max]
    log = []
    for i in range(40):
        op = rng.choice(["step", "step", "step", "append", "flush", "newest", "window"])
        if oc.t == 0 and op in ("newest", "window"):
            op = "step"
        log.append(op)
        if op == "step":
            v, q = tokens(1)
            out = c.step(torch.from_numpy(v).cuda(), torch.from_numpy(q).cuda(), P)
            oc.update(v.astype(np.float64), q.astype(np.float64))
            want = oc.readout_newest(oracle.gate(oc.sum_q, 1.0 / N_max, f64(p), n, 0))
            assert rel_l2(from_device(out), want) <= 1e-5, (i, log)
        elif op == "append":
            T = int(rng.choice(sizes))
            v, q = tokens(T)
            c.update(torch.from_numpy(v).cuda(), torch.from_numpy(q).cuda())
            for j in range(T):                  # also where the library pre-fills: the two are the same state
                oc.update(v[:, j:j + 1].astype(np.float64), q[:, j:j + 1].astype(np.float64))
            log[-1] = f"append{T}"
            check_state((i, log))
        elif op == "flush":
            check_state((i, log))
        else:
            c.flush()
            g = synth.random_gate(720 + i, B, H, n)
            mode = binding.READ_NEWEST if op == "newest" else binding.READ_WINDOW
            got = from_device(c.readout(torch.from_numpy(g).cuda(), mode))
            if op == "newest":
                want = oc.readout_newest(g.astype(np.complex128))
            elif N_mem:
                want = oc.readout_window(g.astype(np.complex128))          # live ring slots, oldest first
            else:                                                          # plain cache: the last L' rows of the inverse
                Lw = min(oc.t, N_max)
                want = np.stack([oc.readout_row(g.astype(np.complex128), m) for m in range(n - Lw, n)], axis=1)
            assert got.shape == want.shape and rel_l2(got, want) <= 1e-5, (i, log)
    check_state(("end", log))
    print(f"  operations: {' '.join(log)}", flush=True)
