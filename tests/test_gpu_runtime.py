"""Runtime behaviour of the library on the GPU: streams, determinism, table cache, error paths."""
import ctypes

import numpy as np
import pytest
import torch

from gpu_util import rel_l2, to_device
from paper_2502_18394_amd import synth

pytestmark = pytest.mark.gpu


def test_calls_follow_the_callers_stream(oracle):
    """Work is enqueued on the stream passed in, not on the default one."""
    from paper_2502_18394_amd import binding
    B, L, H, d = 1, 2048, 2, 64
    vals, store = synth.tokens(1, (B, L, H, d), "f32")
    g = synth.random_gate(2, B, H, L)
    s = torch.cuda.Stream()
    v = to_device(store, "f32")
    gd = torch.from_numpy(g).cuda()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        out = binding.mix_forward(v, gd, stream=s)
    s.synchronize()
    want = oracle.mix_forward(vals.astype(np.float64), g.astype(np.complex128))
    assert rel_l2(out.cpu().numpy(), want) <= 1e-5


def test_decode_step_is_bitwise_reproducible():
    from paper_2502_18394_amd import binding
    B, H, d, N = 2, 3, 64, 1024
    p = synth.gate_params(3, H, d, N)
    P = binding.GateParams(p)
    _, v0 = synth.tokens(4, (B, N, H, d), "f32")
    _, q0 = synth.tokens(5, (B, N, H, d), "f32")
    _, vt = synth.tokens(6, (B, 8, H, d), "f32")
    _, qt = synth.tokens(7, (B, 8, H, d), "f32")
    runs = []
    for _ in range(2):
        c = binding.PrefixCache(B, H, d, N)
        c.update(to_device(v0, "f32"), to_device(q0, "f32"))
        outs = [c.step(to_device(np.ascontiguousarray(vt[:, i:i + 1]), "f32"),
                       to_device(np.ascontiguousarray(qt[:, i:i + 1]), "f32"), P).clone() for i in range(8)]
        torch.cuda.synchronize()
        runs.append((torch.stack(outs), c.prefix_fft.clone()))
    assert torch.equal(runs[0][0], runs[1][0]) and torch.equal(runs[0][1].view(torch.float32), runs[1][1].view(torch.float32))


def test_shutdown_frees_tables_and_library_recovers(oracle):
    """After spectre_shutdown a length is unprepared again: the C entry point says so and launches nothing (the output
    keeps its sentinel), spectre_prepare brings it back, and the rows are the same bits as before."""
    from paper_2502_18394_amd import binding
    vals, store = synth.tokens(8, (1, 512, 1, 64), "f32")
    g = torch.from_numpy(synth.random_gate(9, 1, 1, 512)).cuda()
    v = to_device(store, "f32")
    a = binding.mix_forward(v, g).cpu()
    torch.cuda.synchronize()
    binding.shutdown()
    binding.shutdown()
    out = torch.full_like(v, 7.0)
    ws = torch.empty(512, dtype=torch.uint8, device="cuda")
    off = (-ws.data_ptr()) % 256
    L = binding.lib()
    rc = L.spectre_mix_forward(ctypes.c_void_p(v.data_ptr()), ctypes.c_void_p(g.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                               1, 512, 1, 64, 0, ctypes.c_void_p(ws.data_ptr() + off), ctypes.c_size_t(256), None)
    torch.cuda.synchronize()
    assert rc == binding.ENOTREADY and b"spectre_prepare" in L.spectre_last_error()
    assert bool((out == 7.0).all())
    b = binding.mix_forward(v, g).cpu()                  # the binding prepares the length again
    assert torch.equal(a, b)


def test_error_paths_launch_nothing():
    from paper_2502_18394_amd import binding
    v = torch.zeros((1, 8192, 1, 64), device="cuda")
    g = torch.zeros((1, 1, 4097), dtype=torch.complex64, device="cuda")
    L = binding.lib()
    small = torch.empty(512, dtype=torch.uint8, device="cuda")
    off = (-small.data_ptr()) % 256
    rc = L.spectre_mix_forward(ctypes.c_void_p(v.data_ptr()), ctypes.c_void_p(g.data_ptr()), ctypes.c_void_p(v.data_ptr()),
                               1, 8192, 1, 64, 0, ctypes.c_void_p(small.data_ptr() + off), ctypes.c_size_t(256), None)
    assert rc == binding.EINVAL                                  # out overlaps v
    out = torch.empty_like(v)
    rc = L.spectre_mix_forward(ctypes.c_void_p(v.data_ptr()), ctypes.c_void_p(g.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                               1, 8192, 1, 64, 0, ctypes.c_void_p(small.data_ptr() + off), ctypes.c_size_t(256), None)
    assert rc == binding.EWORKSPACE and b"workspace" in L.spectre_last_error()
    c = binding.PrefixCache(1, 1, 64, 256)
    with pytest.raises(binding.SpectreError) as e:
        c.readout(torch.zeros((1, 1, 129), dtype=torch.complex64, device="cuda"))
    assert e.value.code == binding.EINVAL                        # empty cache
    big = torch.zeros((1, 300, 1, 64), device="cuda")
    with pytest.raises(binding.SpectreError) as e:
        c.update(big, big)
    assert e.value.code == binding.EINVAL and c.t == 0           # prompt longer than the window
    with pytest.raises(binding.SpectreError):
        binding.PrefixCache(1, 1, 64, 1000)                      # window length without a plan


def test_prefix_update_with_a_short_workspace_launches_nothing():
    """A cache with deferred updates pending: spectre_prefix_update checks its workspace before it flushes them, so an
    EWORKSPACE return leaves the spectrum, the pending list and the token counter exactly as they were."""
    from paper_2502_18394_amd import binding
    B, H, d, N = 1, 2, 64, 1024
    P = binding.GateParams(synth.gate_params(80, H, d, N))
    c = binding.PrefixCache(B, H, d, N, defer=8)
    _, v0 = synth.tokens(81, (B, 700, H, d), "f32")
    _, q0 = synth.tokens(82, (B, 700, H, d), "f32")
    c.update(to_device(v0, "f32"), to_device(q0, "f32"))
    for i in range(3):
        _, vt = synth.tokens(83 + i, (B, 1, H, d), "f32")
        c.step(to_device(vt, "f32"), to_device(vt, "f32"), P)
    torch.cuda.synchronize()
    assert c.n_pending == 3
    before = c.prefix_fft.clone()
    _, v2 = synth.tokens(90, (B, 4, H, d), "f32")
    v2d = to_device(v2, "f32")
    ws = torch.empty(1024, dtype=torch.uint8, device="cuda")
    off = (-ws.data_ptr()) % 256
    rc = binding.lib().spectre_prefix_update(ctypes.byref(c.c), ctypes.c_void_p(v2d.data_ptr()), ctypes.c_void_p(v2d.data_ptr()),
                                             4, 0, ctypes.c_void_p(ws.data_ptr() + off), ctypes.c_size_t(256), None)
    torch.cuda.synchronize()
    assert rc == binding.EWORKSPACE
    assert c.n_pending == 3 and c.t == 703
    assert torch.equal(before.view(torch.float32), c.prefix_fft.view(torch.float32))
    c.update(v2d, v2d)                                        # the same call with its workspace goes through
    assert c.n_pending == 0 and c.t == 707


@pytest.mark.parametrize("L,H", [(4096, 4), (32768, 32)])
def test_forward_path_replays_from_a_hip_graph(oracle, L, H):
    """gate -> mixer -> level gates -> refinement captured once in a HIP graph and replayed on fresh inputs, with
    eager work and synchronisations between the replays; every replay must equal the eager result bit for bit.
    The capture is the first thing these lengths see after a shutdown: only spectre_prepare ran before it, no eager
    call (compute calls neither allocate nor synchronise).  The larger case runs its head groups on two streams
    (fork and join are captured as graph edges)."""
    from paper_2502_18394_amd import binding
    B, d = 1, 64
    J = synth.max_wavelet_levels(L)
    binding.shutdown()
    binding.prepare(L, d)
    P = binding.GateParams(synth.gate_params(40, H, d, L))
    W = binding.WrmParams(synth.wrm_params(41, H, d, J))

    def inputs(seed):
        _, vs = synth.tokens(seed, (B, L, H, d), "bf16")
        _, qs = synth.tokens(seed + 1, (B, L, H, d), "bf16")
        return to_device(vs, "bf16"), to_device(qs, "bf16")

    def eager(v, q):
        g = binding.gate(q, P, 1.0 / L)
        return binding.wrm_apply(binding.mix_forward(v, g), binding.wrm_gates(q, W, 1.0 / L))

    v0, q0 = inputs(42)
    v_s, q_s = v0.clone(), q0.clone()                   # static graph inputs
    g_s = torch.empty((B, H, L // 2 + 1), dtype=torch.complex64, device="cuda")
    s_s = torch.empty((B, H, J + 1, d), dtype=torch.float32, device="cuda")
    mix_s, out_s = torch.empty_like(v_s), torch.empty_like(v_s)
    ws = [torch.empty(n + 256, dtype=torch.uint8, device="cuda")
          for n in (binding.gate_workspace_bytes(B, L, H, P), binding.mix_workspace_bytes(B, L, H, d, binding.BF16),
                    binding.gate_workspace_bytes(B, L, H, P), binding.wrm_apply_workspace_bytes(B, L, H, d, J))]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.gate(q_s, P, 1.0 / L, g_out=g_s, ws=ws[0])
        binding.mix_forward(v_s, g_s, out=mix_s, ws=ws[1])
        binding.wrm_gates(q_s, W, 1.0 / L, s_out=s_s, ws=ws[2])
        binding.wrm_apply(mix_s, s_s, out=out_s, ws=ws[3])
    want0 = eager(v0, q0).clone()
    torch.cuda.synchronize()
    for r, seed in enumerate((42, 50, 60)):
        v, q = inputs(seed)
        want = eager(v, q).clone()                      # eager work between replays
        torch.cuda.synchronize()
        v_s.copy_(v)
        q_s.copy_(q)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_s.view(torch.int16), want.view(torch.int16)), f"replay {r}"
        if r == 0:
            assert torch.equal(out_s.view(torch.int16), want0.view(torch.int16))


def test_two_stream_call_is_ordered_on_the_callers_stream():
    """A long call runs half of its head groups on the library's helper stream; work enqueued on the
    caller's stream right before and right after it must still see it as one ordered step."""
    from paper_2502_18394_amd import binding
    B, L, H, d = 1, 32768, 32, 64
    _, store = synth.tokens(70, (B, L, H, d), "bf16")
    g = torch.from_numpy(synth.random_gate(71, B, H, L)).cuda()
    v_src = to_device(store, "bf16")
    ref = binding.mix_forward(v_src, g).clone()
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    v = torch.zeros_like(v_src)
    out = torch.zeros_like(v_src)
    with torch.cuda.stream(s):
        for _ in range(3):
            v.copy_(v_src, non_blocking=True)          # producer on the caller's stream, just before the call
            binding.mix_forward(v, g, out=out, stream=s)
            snap = out.clone()                         # consumer on the caller's stream, just after the call
            v.zero_()                                  # and a writer of the input, which must wait for the call
            out.zero_()
    s.synchronize()
    assert torch.equal(snap.view(torch.int16), ref.view(torch.int16))
