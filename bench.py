#!/usr/bin/env python3
"""Benchmark of the SPECTRE hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-decode] [--no-cpu]

One step = one pass of the whole hot path over one batch of synthetic input:
spectre_gate (pool the query rows, LayerNorm, MLP on the matrix cores, modReLU) followed
by spectre_mix_forward (rfft -> gate -> irfft) on the Llama-3.2-1B head shape at L = 131072.
The decode half of the path (one fused Prefix-FFT step per new token, B = 8, N_max = 32768)
is timed in the same run and reported under "decode".  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line.
"""
import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
# L2<->fabric bytes per spectre_mix_forward call at llama1b_128k and per decode sweep come from separate rocprofv3
# FETCH_SIZE and WRITE_SIZE passes over this same script (scaled by what the counters read for a plain 1 GiB copy);
# the figures are read from the tracked summary of those passes, lines of the form `name = bytes`
TRAFFIC_FILE = os.path.join("profiles", "traffic_llama1b_128k_and_decode_32k.txt")
# lane-instructions per complex point (one channel pair at one position) of the three transform kernels at
# L = 131072, counted in the ISA of the built library: 84 (column kernel) + 37 + 37 (row kernels)
COUNTED_LANE_INSTR_PER_POINT_128K = 158
# fp32 vector peak without packed math: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions/s
VALU_PEAK_GINSTR = 256 * 4 * 16 * 2.4


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama1b_128k")
    ap.add_argument("--L", type=int, default=0, help="override the sequence length of the workload")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the per-configuration mixer rows")
    ap.add_argument("--lanes", type=int, default=0,
                    help="1: keep every head group of a long mixer call on one stream (so that a profiler's per-kernel "
                         "durations add up); default: the library's own choice")
    ap.add_argument("--decode-steps", type=int, default=256,
                    help="decode steps timed (the baseline's configuration appends 256 tokens, each a fresh random one)")
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip the secondary decode row (window of 65536 slots), e.g. under a profiler so that every\n"
                         "cache kernel in the trace belongs to the decode_32k workload")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the headline line, print one JSON line per configuration (mixer only): the "
                         "length sweep at the Llama head shape, config 1 and the ViT shape")
    ap.add_argument("--only", default="",
                    help="with --sweep: only the configurations whose name contains this text (e.g. L8192), so that a "
                         "profiler run covers one shape")
    ap.add_argument("--copy-calib", action="store_true",
                    help="also run a plain 1 GiB device copy 5 times (reference for scaling hardware byte counters)")
    return ap.parse_args()


def traffic_figures():
    """{name: bytes} from the tracked counter summary, or {} if it is missing."""
    out = {}
    try:
        with open(os.path.join(ROOT, TRAFFIC_FILE)) as f:
            for line in f:
                if "=" in line and not line.lstrip().startswith("#"):
                    k, v = line.split("=", 1)
                    try:
                        out[k.strip()] = float(v.split()[0])
                    except (ValueError, IndexError):
                        pass
    except OSError:
        pass
    return out


def time_loop(fn, steps, warmup):
    """Average milliseconds per call between HIP events on the current stream."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def time_each(fn, n):
    """(median, min) milliseconds of n calls timed one by one with their own HIP event pairs."""
    import torch
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    t = sorted(a.elapsed_time(b) for a, b in ev)
    return t[len(t) // 2], t[0]


def device_tokens(shape, seed, dtype):
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    return torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).to(dtype)


def device_gate_params(seed, Hg, d, n_fft, d_g, binding):
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    F = n_fft // 2 + 1

    def nrm(*s):
        return 0.02 * torch.randn(s, generator=gen, device="cuda", dtype=torch.float32)
    p = dict(n_fft=n_fft, ln_eps=1e-5, ln_gamma=1.0 + nrm(Hg, d), ln_beta=nrm(Hg, d), W1=nrm(Hg, d, d_g),
             b1=nrm(Hg, d_g), W2=nrm(Hg, d_g, 2 * F), b2=nrm(Hg, 2 * F), modrelu_bias=nrm(Hg, F))
    return binding.GateParams(p)


def cpu_baseline(cfg, L):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload (whole heads)."""
    import numpy as np
    import oracle
    from paper_2502_18394_amd import synth
    oracle.build()
    H, d = cfg["H"], cfg["d"]
    Hs = H                                           # the whole workload: about 6 s at 128k on 16 threads
    vals, _ = synth.tokens(synth.BASE_SEED, (1, L, Hs, d), cfg["io"])
    qv, _ = synth.tokens(synth.BASE_SEED + 1, (1, L, Hs, d), cfg["io"])
    p = synth.gate_params(synth.BASE_SEED + 2, Hs, d, L)
    p64 = {k: (np.asarray(v, np.float64) if isinstance(v, np.ndarray) else v) for k, v in p.items()}
    V, Q = vals.astype(np.float64), qv.astype(np.float64)
    t0 = time.time()
    g = oracle.gate(oracle.pool_q(Q), 1.0 / L, p64, L, 0)
    oracle.mix_forward(V, g)
    dt = time.time() - t0
    return {"value": cfg["B"] * L / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"gate+mix_forward of all {cfg['B'] * H} heads at L={L} (the whole workload, one pass): {dt:.2f} s"}


def mix_case(name, c, steps, graph=False, with_gate=False):
    """Timing of one configuration: the mixer alone and, with_gate, the gate alone and gate + mixer.  A working set
    below the memory-side cache is rotated over enough buffers (> 512 MB in total) that the figure is not a
    cache-resident one; the mixer's cache-resident time rides along."""
    import torch
    from paper_2502_18394_amd import binding, synth
    B, H, L, d = c["B"], c["H"], c["L"], c["d"]
    dtype = torch.bfloat16 if c["io"] == "bf16" else torch.float32
    esize = 2 if c["io"] == "bf16" else 4
    nbytes = B * L * H * d * esize
    nbuf = max(1, min(64, (512 << 20) // (2 * nbytes) + 1))
    Vs = [device_tokens((B, L, H, d), synth.BASE_SEED + i, dtype) for i in range(nbuf)]
    outs = [torch.empty_like(Vs[0]) for _ in range(nbuf)]
    g = torch.from_numpy(synth.random_gate(synth.BASE_SEED, B, H, L)).cuda()
    ws = torch.empty(binding.mix_workspace_bytes(B, L, H, d, binding._dtype_code(Vs[0])) + 256, dtype=torch.uint8, device="cuda")
    it = [0]

    def call():
        i = it[0] % nbuf
        binding.mix_forward(Vs[i], g, out=outs[i], ws=ws)
        it[0] += 1
    reps = max(steps, min(200, int(2e9 // max(nbytes, 1)) + 1))
    # the cache-resident loop first (it also brings the clocks up), then the rotated one with every buffer touched
    ms_hot = time_loop(lambda: binding.mix_forward(Vs[0], g, out=outs[0], ws=ws), reps, 3)
    ms = time_loop(call, reps, max(3, nbuf))
    ms_graph = None
    if graph and nbytes <= (64 << 20):     # launch-bound sizes: the same call replayed from a HIP graph
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            for i in range(min(nbuf, 8)):
                binding.mix_forward(Vs[i], g, out=outs[i], ws=ws)
        ms_graph = time_loop(gr.replay, max(reps // 8, 5), 2) / min(nbuf, 8)
        del gr
    F = L // 2 + 1
    alg = 2 * nbytes + B * H * F * 8
    # share of the fp32 vector peak (157.3 TFLOP/s, which counts packed FMAs) with the usual flop count of the
    # transform pair and the gate product: 4 log2 L + 3 flop per real element
    flops = B * L * H * d * (4.0 * math.log2(L) + 3.0)
    row = {"workload": name, "B": B, "H": H, "L": L, "d": d, "io": c["io"], "ms": ms,
           "tokens_per_s": B * L / (ms * 1e-3), "algorithmic_bytes": alg,
           "hbm_frac": alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "valu_frac": flops / (ms * 1e-3) / 157.3e12,
           "buffers_rotated": nbuf, "ms_cache_resident": ms_hot}
    if graph:
        row["ms_hip_graph"] = ms_graph
    if with_gate:
        # rows (ii) and (iii) of the configuration: the gate from the query rows (per-head weights), and gate + mixer
        P = device_gate_params(synth.BASE_SEED + 2, H, d, L, synth.D_GATE, binding)
        ws_gate = torch.empty(binding.gate_workspace_bytes(B, L, H, P) + 256, dtype=torch.uint8, device="cuda")
        gg = torch.empty((B, H, F), dtype=torch.complex64, device="cuda")
        jt = [0]

        def gate_call():
            i = jt[0] % nbuf
            binding.gate(Vs[i], P, 1.0 / L, g_out=gg, ws=ws_gate)
            jt[0] += 1

        def both():
            i = jt[0] % nbuf
            binding.gate(Vs[(i + 1) % nbuf], P, 1.0 / L, g_out=gg, ws=ws_gate)
            binding.mix_forward(Vs[i], gg, out=outs[i], ws=ws)
            jt[0] += 1
        ms_g = time_loop(gate_call, reps, max(3, nbuf))
        ms_e = time_loop(both, reps, max(3, nbuf))
        gate_bytes = nbytes + P.Hg * P.d_g * 2 * F * 4 + B * H * F * 8
        e2e_bytes = alg + gate_bytes - B * H * F * 8
        row.update({"gate_ms": ms_g, "gate_algorithmic_bytes": gate_bytes,
                    "gate_hbm_frac": gate_bytes / (ms_g * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "end_to_end_ms": ms_e, "end_to_end_algorithmic_bytes": e2e_bytes,
                    "end_to_end_hbm_frac": e2e_bytes / (ms_e * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "end_to_end_tokens_per_s": B * L / (ms_e * 1e-3)})
        del P, ws_gate, gg
    del Vs, outs, g, ws
    torch.cuda.empty_cache()
    return row


def copy_calibration():
    """A plain 1 GiB device-to-device copy, five times: what a hardware byte counter reads for a known size."""
    import torch
    src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB read + 1 GiB written per copy
    dst = torch.empty_like(src)
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst
    torch.cuda.empty_cache()


def config_cases():
    """Every mixer configuration the baseline names: config 1, config 2 (= the 8192 point of the sweep), the length
    sweep of config 3 and the ViT shape of config 5."""
    from paper_2502_18394_amd import synth
    cases = [("config1_single_head_1k", synth.CONFIGS["single_head_1k"])]
    for L in synth.SWEEP_L:
        tag = "config2_and_3" if L == 8192 else "config3"
        cases.append((f"{tag}_llama1b_L{L}", dict(B=1, H=32, L=L, d=64, io="bf16")))
    cases.append(("config5_vit_196", synth.CONFIGS["vit_196"]))
    return cases


def sweep(args):
    """One JSON line per configuration (mixer only), then lengths outside the baseline's list."""
    cases = config_cases()
    # four-step lengths with an odd factor (3 * 4096, 24 * 4096), then lengths with no plan of their own
    # (padded power-of-two convolution)
    cases += [(f"llama1b_L{L}", dict(B=1, H=32, L=L, d=64, io="bf16")) for L in (12288, 98304)]
    cases += [("vit_197_cls", dict(B=256, H=12, L=197, d=64, io="f32"))]
    cases += [(f"llama1b_L{L}", dict(B=1, H=32, L=L, d=64, io="bf16")) for L in (1000, 50000)]
    for name, c in cases:
        if args.only and args.only not in name:
            continue
        print(json.dumps(mix_case(name, c, args.steps, graph=not args.only, with_gate=not args.only)), flush=True)
    if args.copy_calib:
        copy_calibration()


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is a single-GPU kernel path; run with --gpus 1 (no multi-GPU figure exists).",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2502_18394_amd import binding, synth
    if args.sweep:
        torch.cuda.set_device(0)
        binding.lib()
        sweep(args)
        return

    cfg = dict(synth.CONFIGS[args.workload])
    if args.L:
        cfg["L"] = args.L
    B, H, L, d = cfg["B"], cfg["H"], cfg["L"], cfg["d"]
    dtype = torch.bfloat16 if cfg["io"] == "bf16" else torch.float32
    esize = 2 if cfg["io"] == "bf16" else 4
    torch.cuda.set_device(0)
    binding.lib()   # raises if the HIP library is missing: there is no other path
    if args.lanes:
        binding.set_option(binding.OPT_LANES, args.lanes)

    V = device_tokens((B, L, H, d), synth.BASE_SEED, dtype)
    Q = device_tokens((B, L, H, d), synth.BASE_SEED + 1, dtype)
    P = device_gate_params(synth.BASE_SEED + 2, H, d, L, synth.D_GATE, binding)
    out = torch.empty_like(V)
    g = torch.empty((B, H, L // 2 + 1), dtype=torch.complex64, device="cuda")
    ws_mix = torch.empty(binding.mix_workspace_bytes(B, L, H, d, binding._dtype_code(V)) + 256, dtype=torch.uint8, device="cuda")
    ws_gate = torch.empty(binding.gate_workspace_bytes(B, L, H, P) + 256, dtype=torch.uint8, device="cuda")

    def step():
        binding.gate(Q, P, 1.0 / L, g_out=g, ws=ws_gate)
        binding.mix_forward(V, g, out=out, ws=ws_mix)

    def mix_only():
        binding.mix_forward(V, g, out=out, ws=ws_mix)

    def gate_only():
        binding.gate(Q, P, 1.0 / L, g_out=g, ws=ws_gate)

    # whole step: barrier-free single process; synchronize on both sides of the timed region
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps

    ms_mix = time_loop(mix_only, args.steps, 2)
    ms_gate = time_loop(gate_only, args.steps, 2)
    mix_med, mix_min = time_each(mix_only, max(args.steps, 50))

    tokens = B * L
    F = L // 2 + 1
    mix_bytes = 2 * tokens * H * d * esize + B * H * F * 8                # read V, write out, read g
    gate_bytes = tokens * H * d * esize + P.Hg * P.d_g * 2 * F * 4 + B * H * F * 8   # read Q, read W2, write g
    headline = (args.workload == "llama1b_128k" and not args.L)
    traffic = traffic_figures() if headline else {}
    if headline:      # counted in the ISA; other lengths: 3.5 per point per radix-2 stage each way + 6 for the gate
        instr_per_point, instr_src = COUNTED_LANE_INSTR_PER_POINT_128K, "counted in the ISA of the three transform kernels"
    else:
        instr_per_point, instr_src = 2 * 3.5 * (L.bit_length() - 1) + 6, "model: 3.5 per point and radix-2 stage each way + 6"
    mix_flops_instr = tokens * H * (d // 2) * instr_per_point
    e2e_bytes = mix_bytes + gate_bytes - B * H * F * 8        # Q, V in; out; W2; g written once and read once
    res = {
        "metric": "mixer tokens/sec at L=128k (H=32,d=64) + % HBM roofline; decode tokens/sec",
        "value": tokens / (ms_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "io_dtype": cfg["io"], "data": "synthetic",
        "config": {"workload": f"{args.workload}: gate+mix_forward B={B} H={H} d={d} L={L} {cfg['io']} I/O, fp32 spectra",
                   "global_batch": B, "seq_len": L, "parallelism": "single GPU"},
        "roofline": {"bound": "hbm", "kernel": "spectre_mix_forward (gate_expand + per head group: small_fwd, big, small_inv)",
                     "achieved": mix_bytes / (ms_mix * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": mix_bytes / (ms_mix * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": traffic.get("mix_forward_bytes_per_call"),
                     "traffic_source": TRAFFIC_FILE if "mix_forward_bytes_per_call" in traffic else None,
                     "algorithmic_bytes": mix_bytes, "ms": ms_mix},
        "roofline_alu": {"bound": "alu", "achieved": mix_flops_instr / (ms_mix * 1e-3) / 1e9, "peak": VALU_PEAK_GINSTR,
                         "unit": "G lane-instr/s", "frac": mix_flops_instr / (ms_mix * 1e-3) / 1e9 / VALU_PEAK_GINSTR,
                         "lane_instr_per_point": instr_per_point, "lane_instr_source": instr_src},
        "end_to_end": {"what": "gate from the query rows + mixer (the timed step)", "ms": ms_step,
                       "algorithmic_bytes": e2e_bytes, "hbm_frac": e2e_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "mix_only": {"tokens_per_s": tokens / (ms_mix * 1e-3), "ms": ms_mix, "ms_median_of_single_calls": mix_med,
                     "ms_min_of_single_calls": mix_min},
        "gate_only": {"ms": ms_gate, "algorithmic_bytes": gate_bytes,
                      "hbm_frac": gate_bytes / (ms_gate * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    # token projection (next-row item): X -> V and the pooled query, X read once
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.BASE_SEED + 8)
    Wq = 0.125 * torch.randn((H, d, d), generator=gen, device="cuda", dtype=torch.float32)
    Wv = 0.125 * torch.randn((H, d, d), generator=gen, device="cuda", dtype=torch.float32)
    ws_proj = torch.empty(int(binding.lib().spectre_project_workspace_bytes(B, L, H, d)) + 256, dtype=torch.uint8, device="cuda")
    ms_proj = time_loop(lambda: binding.project(Q, Wq, Wv, ws=ws_proj), args.steps, 2)
    proj_bytes = 2 * tokens * H * d * esize
    proj_flops = 2.0 * tokens * H * d * d
    res["project"] = {"ms": ms_proj, "algorithmic_bytes": proj_bytes,
                      "hbm_frac": proj_bytes / (ms_proj * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      "tflops": proj_flops / (ms_proj * 1e-3) / 1e12,
                      "what": "spectre_project: V = X W_v per head + pooled query in one pass over X (bf16 rows: "
                              "32x32x16 bf16 MFMA with two-term weights; fp32 rows: the same instruction on three-term splits); includes "
                              "allocating the outputs"}
    # wavelet refinement (next-row item) applied to the mixer's output, full depth
    J = synth.max_wavelet_levels(L)
    s_lv = torch.randn((B, H, J + 1, d), generator=gen, device="cuda", dtype=torch.float32)
    ws_wrm = torch.empty(binding.wrm_apply_workspace_bytes(B, L, H, d, J) + 256, dtype=torch.uint8, device="cuda")
    wrm_out = torch.empty_like(out)
    ms_wrm = time_loop(lambda: binding.wrm_apply(out, s_lv, out=wrm_out, ws=ws_wrm), args.steps, 2)
    wrm_bytes = 2 * tokens * H * d * esize
    res["wrm"] = {"ms": ms_wrm, "levels": J, "algorithmic_bytes": wrm_bytes,
                  "hbm_frac": wrm_bytes / (ms_wrm * 1e-3) / 1e9 / HBM_PEAK_GBS,
                  "what": "spectre_wrm_apply: V + iDWT(s * DWT(V)), Haar, one gate per band and channel"}
    # the same module with one gate per wavelet coefficient and channel (gates: one more fp32 tensor to read)
    s_co = torch.randn((B, H, L, d), generator=gen, device="cuda", dtype=torch.float32)
    ms_wco = time_loop(lambda: binding.wrm_apply_coeff(out, s_co, J, out=wrm_out, ws=ws_wrm), args.steps, 2)
    wco_bytes = wrm_bytes + tokens * H * d * 4
    res["wrm_coeff"] = {"ms": ms_wco, "levels": J, "algorithmic_bytes": wco_bytes,
                        "hbm_frac": wco_bytes / (ms_wco * 1e-3) / 1e9 / HBM_PEAK_GBS,
                        "what": "spectre_wrm_apply_coeff: one gate per coefficient and channel, s [B,H,L,d] fp32"}
    del s_co
    # the whole layer in one call: X -> projection -> pooled query -> gate -> mixer (-> refinement), against the same
    # chain as separate calls.  Algorithmic bytes: X in, out, W2, and g written and read once.
    layer_bytes = 2 * tokens * H * d * esize + P.Hg * P.d_g * 2 * F * 4 + 2 * B * H * F * 8
    Wp = binding.WrmParams(synth.wrm_params(synth.BASE_SEED + 14, H, d, J))
    res["layer"] = {"algorithmic_bytes": layer_bytes}
    for tag, wp in (("", None), ("_with_refinement", Wp)):
        need = int(binding.lib().spectre_layer_workspace_bytes(B, L, H, d, binding._dtype_code(V), ctypes.byref(P.c),
                                                               ctypes.byref(wp.c) if wp is not None else None))
        ws_layer = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
        ms_layer = time_loop(lambda: binding.layer_forward(Q, Wq, Wv, P, wp, out=out, ws=ws_layer), args.steps, 2)
        del ws_layer

        def chain():
            v, _, sq = binding.project(Q, Wq, Wv, ws=ws_proj)
            binding.gate(sq, P, 1.0 / L, pooled=True, g_out=g, ws=ws_gate)
            binding.mix_forward(v, g, out=out, ws=ws_mix)
            if wp is not None:
                binding.wrm_apply(out, binding.wrm_gates(sq, wp, 1.0 / L, pooled=True), out=out, ws=ws_wrm)
        ms_chain = time_loop(chain, args.steps, 2)
        res["layer"]["ms" + tag] = ms_layer
        res["layer"]["ms_separate_calls" + tag] = ms_chain
        res["layer"]["tokens_per_s" + tag] = tokens / (ms_layer * 1e-3)
        res["layer"]["hbm_frac" + tag] = (layer_bytes + (0 if wp is None else 0)) / (ms_layer * 1e-3) / 1e9 / HBM_PEAK_GBS
    res["layer"]["what"] = ("spectre_layer_forward: projection inside the row transforms (V never in memory), gate from "
                            "the pooled query, mixer; with refinement: Haar level gates, coarse levels from block sums "
                            "the mixer's store phase emits")
    del Wp
    if cfg["io"] == "bf16" and not args.no_secondary and binding.mix_workspace_bytes(B, L, H, d, binding.BF16) > 256:
        # opt-in variant, reported beside the default and never as `value`: bfloat16 pairs between the three kernels
        ms16 = time_loop(lambda: binding.mix_forward(V, g, out=out, ws=ws_mix, flags=binding.MIX_BF16_SCRATCH),
                         args.steps, 2)
        res["mix_only_bf16_scratch"] = {"ms": ms16, "tokens_per_s": tokens / (ms16 * 1e-3),
                                        "hbm_frac": mix_bytes / (ms16 * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                        "what": "flag SPECTRE_MIX_BF16_SCRATCH: same call, fp32 arithmetic, the two exchanges "
                                                "between the kernels in bfloat16 (rel-L2 2.9e-3 instead of 1.7e-3)"}
    del V, Q, out, g, ws_mix, ws_gate, P, Wq, Wv, ws_proj, s_lv, ws_wrm, wrm_out
    torch.cuda.empty_cache()

    if args.copy_calib:
        copy_calibration()

    if not args.no_decode:
        dc = synth.CONFIGS["decode_32k"]
        Bd, Hd, N, dd = dc["B"], dc["H"], dc["N_max"], dc["d"]
        cache = binding.PrefixCache(Bd, Hd, dd, N)
        Pd = device_gate_params(synth.BASE_SEED + 3, Hd, dd, N, synth.D_GATE, binding)
        cache.update(device_tokens((Bd, N, Hd, dd), synth.BASE_SEED + 4, torch.float32),
                     device_tokens((Bd, N, Hd, dd), synth.BASE_SEED + 5, torch.float32))
        # one fresh random token per step (drawn before the timed region, resident in HBM)
        nrot = max(args.decode_steps + 8, 64)
        vts = device_tokens((nrot, Bd, 1, Hd, dd), synth.BASE_SEED + 6, torch.float32)
        qts = device_tokens((nrot, Bd, 1, Hd, dd), synth.BASE_SEED + 7, torch.float32)
        vt, qt = vts[0], qts[0]
        od = torch.empty_like(vt)
        k = [0]

        def decode_step():
            i = k[0] % nrot
            cache.step(vts[i], qts[i], Pd, out=od)
            k[0] += 1
        ms_dec = time_loop(decode_step, args.decode_steps, 3)
        Fd = N // 2 + 1
        sweep_bytes = 2 * 8 * Bd * Hd * Fd * dd
        res["decode"] = {"workload": f"decode_32k: fused Prefix-FFT step B={Bd} H={Hd} d={dd} N_max={N}, cache full (eviction branch), fp32",
                         "tokens_per_s": Bd / (ms_dec * 1e-3), "ms_per_step": ms_dec, "steps": args.decode_steps,
                         "roofline": {"bound": "hbm", "kernel": "k_sweep<update,read>", "achieved": sweep_bytes / (ms_dec * 1e-3) / 1e9,
                                      "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": sweep_bytes / (ms_dec * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                      "traffic": traffic_figures().get("decode_sweep_bytes_per_step"),
                                      "traffic_source": TRAFFIC_FILE, "algorithmic_bytes": sweep_bytes}}
        # one-time rows of the same cache: pre-fill from 32768 tokens (Alg. 1 PreFill) and the literal full-window
        # readout (inverse transform of the gated cache, all live rows)
        Vp = device_tokens((Bd, N, Hd, dd), synth.BASE_SEED + 4, torch.float32)
        Qp = device_tokens((Bd, N, Hd, dd), synth.BASE_SEED + 5, torch.float32)

        def timed(fn, prep, n):
            ts = []
            for _ in range(n):
                prep()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                fn()
                b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b))
            return min(ts)
        ms_pre = timed(lambda: cache.update(Vp, Qp), cache.reset, 3)
        pre_bytes = 5 * 4 * Bd * Hd * N * dd                    # V, Q in; two ring buffers and the spectrum out
        gw = binding.gate(cache.sum_q, Pd, 1.0 / N, pooled=True, phase_pos=cache.t)
        ms_win = timed(lambda: cache.readout(gw, binding.READ_WINDOW), lambda: None, 3)
        win_bytes = 8 * Bd * Hd * Fd * dd + 4 * Bd * Hd * N * dd
        res["decode"]["prefill"] = {"ms": ms_pre, "tokens": Bd * N, "tokens_per_s": Bd * N / (ms_pre * 1e-3),
                                    "algorithmic_bytes": pre_bytes,
                                    "hbm_frac": pre_bytes / (ms_pre * 1e-3) / 1e9 / HBM_PEAK_GBS}
        res["decode"]["readout_window"] = {"ms": ms_win, "rows": N, "algorithmic_bytes": win_bytes,
                                           "hbm_frac": win_bytes / (ms_win * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                           "what": "full inverse of the gated cache, all 32768 live rows, fp32 (output allocated by the call)"}
        # Eq. 5 for 32 tokens appended at once (chunked prefill, speculative verification): one sweep over the cache
        v32 = device_tokens((Bd, 32, Hd, dd), synth.BASE_SEED + 10, torch.float32)
        q32 = device_tokens((Bd, 32, Hd, dd), synth.BASE_SEED + 11, torch.float32)
        ms_app = time_loop(lambda: cache.update(v32, q32), 5, 1)
        res["decode"]["append_32_tokens"] = {"ms": ms_app, "tokens_per_s": Bd * 32 / (ms_app * 1e-3),
                                             "algorithmic_bytes": sweep_bytes,
                                             "hbm_frac": sweep_bytes / (ms_app * 1e-3) / 1e9 / HBM_PEAK_GBS}
        # and for 4096 tokens at once: ring buffers brought up to date in one pass, window transformed afresh
        v4k = device_tokens((Bd, 4096, Hd, dd), synth.BASE_SEED + 12, torch.float32)
        q4k = device_tokens((Bd, 4096, Hd, dd), synth.BASE_SEED + 13, torch.float32)
        ms_app4k = time_loop(lambda: cache.update(v4k, q4k), 3, 1)
        res["decode"]["append_4096_tokens"] = {"ms": ms_app4k, "tokens_per_s": Bd * 4096 / (ms_app4k * 1e-3)}
        del cache, Vp, Qp, gw, v32, q32, v4k, q4k
        torch.cuda.empty_cache()
        # the same steps with deferred updates: the cache is only read, every `cap` steps one sweep applies the
        # pending rank-one updates (same outputs up to fp32 rounding; prefix_fft lags until the flush)
        res["decode_deferred"] = {}
        for cap in (16, 32):
            cache = binding.PrefixCache(Bd, Hd, dd, N, defer=cap)
            cache.update(device_tokens((Bd, N, Hd, dd), synth.BASE_SEED + 4, torch.float32),
                         device_tokens((Bd, N, Hd, dd), synth.BASE_SEED + 5, torch.float32))
            nsteps = max(cap, (min(args.decode_steps, 64) // cap) * cap)          # whole flush periods
            ms_def = time_loop(decode_step, nsteps, cap)
            own_bytes = 8 * Bd * Hd * Fd * dd * (1.0 + 1.0 / cap)    # cap - 1 reads, one read + write
            res["decode_deferred"][f"cap{cap}"] = {
                "tokens_per_s": Bd / (ms_def * 1e-3), "ms_per_step": ms_def, "steps": nsteps,
                "bytes_per_step_of_this_schedule": own_bytes,
                "hbm_frac_of_this_schedule": own_bytes / (ms_def * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "hbm_frac_vs_update_every_step": sweep_bytes / (ms_def * 1e-3) / 1e9 / HBM_PEAK_GBS}
            del cache
            torch.cuda.empty_cache()
        # headline of the decode path as shipped: Alg. 1 with an update at every token (`tokens_per_s` above) and the
        # same outputs with deferred updates
        res["decode"]["tokens_per_s_deferred_cap16"] = res["decode_deferred"]["cap16"]["tokens_per_s"]
        del Pd
        torch.cuda.empty_cache()
        if not args.no_secondary:
            # secondary row: a window of 65536 slots holding the same 32768 tokens, so the steps take the branch of
            # Eq. 5 without eviction; twice the cache bytes per step
            N2w = 2 * N
            cache = binding.PrefixCache(Bd, Hd, dd, N2w)
            Pw = device_gate_params(synth.BASE_SEED + 9, Hd, dd, N2w, synth.D_GATE, binding)
            cache.update(device_tokens((Bd, N, Hd, dd), synth.BASE_SEED + 4, torch.float32),
                         device_tokens((Bd, N, Hd, dd), synth.BASE_SEED + 5, torch.float32))
            nst = max(4, min(args.decode_steps, 32) // 2)
            ms_w = time_loop(lambda: cache.step(vt, qt, Pw, out=od), nst, 2)
            wbytes = 2 * 8 * Bd * Hd * (N2w // 2 + 1) * dd
            res["decode_no_eviction"] = {
                "workload": f"fused Prefix-FFT step B={Bd} H={Hd} d={dd} N_max={N2w}, {N} tokens live (no eviction), fp32",
                "tokens_per_s": Bd / (ms_w * 1e-3), "ms_per_step": ms_w, "steps": nst, "algorithmic_bytes": wbytes,
                "hbm_frac": wbytes / (ms_w * 1e-3) / 1e9 / HBM_PEAK_GBS}
            del cache, Pw
            torch.cuda.empty_cache()

    if not args.no_configs:
        # every configuration the baseline names: the mixer call alone, the gate alone, gate + mixer (config 4 is the
        # decode row above)
        res["configs"] = [mix_case(name, c, args.steps, with_gate=True) for name, c in config_cases()]
        if "decode" in res:
            res["configs"].append({"workload": "config4_decode_32k", "ms": res["decode"]["ms_per_step"],
                                   "tokens_per_s": res["decode"]["tokens_per_s"],
                                   "algorithmic_bytes": res["decode"]["roofline"]["algorithmic_bytes"],
                                   "hbm_frac": res["decode"]["roofline"]["frac"]})
    if not args.no_cpu:
        res["cpu_baseline"] = cpu_baseline(cfg, L)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
