"""Thin Python binding of the C ABI in ``include/spectre.h``.

Argument marshalling only: torch supplies device memory and the current stream,
every step of the computation runs in the HIP library.  There is no fallback: if
``libspectre_hip.so`` has not been built (``python -m paper_2502_18394_amd.build``)
the first call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspectre_hip.so")

F32, BF16 = 0, 1
READ_NEWEST, READ_WINDOW = 0, 1
OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP, ENOTREADY = 0, 1, 2, 3, 4, 5
OPT_LANES, OPT_SCRATCH_MB, OPT_FUSED_4096, OPT_SLAB_COMPILE_TIME, OPT_HEAD_AFFINE, OPT_GROUPS, OPT_LANE_SHUFFLES = 0, 1, 2, 3, 4, 5, 6
MIX_BF16_SCRATCH = 1

_lib = None


class SpectreError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"spectre status {code}: {msg}")
        self.code = code


class GateParamsC(ctypes.Structure):
    _fields_ = [("Hg", ctypes.c_int), ("d", ctypes.c_int), ("d_g", ctypes.c_int), ("n_fft", ctypes.c_int),
                ("ln_gamma", ctypes.c_void_p), ("ln_beta", ctypes.c_void_p), ("ln_eps", ctypes.c_float),
                ("W1", ctypes.c_void_p), ("b1", ctypes.c_void_p), ("W2", ctypes.c_void_p), ("b2", ctypes.c_void_p),
                ("modrelu_bias", ctypes.c_void_p), ("toeplitz", ctypes.c_void_p), ("toeplitz_r", ctypes.c_int)]


class WrmParamsC(ctypes.Structure):
    _fields_ = [("Hg", ctypes.c_int), ("d", ctypes.c_int), ("d_w", ctypes.c_int), ("levels", ctypes.c_int),
                ("ln_gamma", ctypes.c_void_p), ("ln_beta", ctypes.c_void_p), ("ln_eps", ctypes.c_float),
                ("W1", ctypes.c_void_p), ("b1", ctypes.c_void_p), ("W2", ctypes.c_void_p), ("b2", ctypes.c_void_p)]


class PrefixCacheC(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int), ("H", ctypes.c_int), ("d", ctypes.c_int), ("N_max", ctypes.c_int),
                ("N_mem", ctypes.c_int), ("t", ctypes.c_longlong),
                ("prefix_fft", ctypes.c_void_p), ("v_buf", ctypes.c_void_p), ("q_buf", ctypes.c_void_p),
                ("sum_q", ctypes.c_void_p), ("twiddle", ctypes.c_void_p),
                ("pending", ctypes.c_void_p), ("pending_cap", ctypes.c_int), ("n_pending", ctypes.c_int),
                ("pending_slot", ctypes.c_int * 32)]


def lib():
    """The loaded C library; raises if it is missing (never falls back to another path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2502_18394_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        L.spectre_last_error.restype = ctypes.c_char_p
        for name in ("spectre_gate_workspace_bytes", "spectre_mix_workspace_bytes", "spectre_prefix_bytes",
                     "spectre_project_workspace_bytes", "spectre_wrm_gates_workspace_bytes",
                     "spectre_wrm_apply_workspace_bytes",
                     "spectre_prefix_update_workspace_bytes", "spectre_prefix_readout_workspace_bytes",
                     "spectre_prefix_step_workspace_bytes", "spectre_prefix_set_memory_workspace_bytes",
                     "spectre_mix_static_bytes", "spectre_layer_workspace_bytes"):
            getattr(L, name).restype = ctypes.c_size_t
        L.spectre_get_option.restype = ctypes.c_long
        _lib = L
    return _lib


def _check(rc):
    if rc != OK:
        raise SpectreError(rc, lib().spectre_last_error().decode())


def _dtype_code(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev(t, name):
    if not (t.is_cuda and t.is_contiguous()):
        raise ValueError(f"{name} must be a contiguous device tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _workspace(nbytes, device, ws):
    nbytes = max(int(nbytes), 256)
    if ws is None or ws.numel() * ws.element_size() < nbytes:
        ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
    off = (-ws.data_ptr()) % 256
    return ws, ctypes.c_void_p(ws.data_ptr() + off), ctypes.c_size_t(ws.numel() * ws.element_size() - off)


def version():
    return int(lib().spectre_version())


def length_supported(n, d):
    return bool(lib().spectre_length_supported(ctypes.c_int(n), ctypes.c_int(d)))


_prepared = set()


def prepare(n, d=64):
    """Set-up for transform length n on the current device (tables, helper stream): the library's one call that
    allocates and synchronises.  The functions below call it the first time they see a length."""
    key = (torch.cuda.current_device(), int(n), int(d))
    if key not in _prepared:
        _check(lib().spectre_prepare(ctypes.c_int(n), ctypes.c_int(d)))
        _prepared.add(key)


def shutdown():
    """Free the library's tables and helper streams; lengths are prepared again on their next use."""
    lib().spectre_shutdown()
    _prepared.clear()


def set_option(which, value):
    """Tuning switch `which` (one of the OPT_* constants) := value; value < 0 restores the default."""
    _check(lib().spectre_set_option(ctypes.c_int(which), ctypes.c_long(value)))


def get_option(which):
    return int(lib().spectre_get_option(ctypes.c_int(which)))


def mix_workspace_bytes(B, L, H, d, io):
    return int(lib().spectre_mix_workspace_bytes(ctypes.c_int(B), ctypes.c_int(L), ctypes.c_int(H),
                                                 ctypes.c_int(d), ctypes.c_int(io)))


def mix_forward(v, g, out=None, ws=None, stream=None, flags=0):
    """out[b,:,h,c] = irfft_L(g[b,h,:] * rfft_L(v[b,:,h,c])); v [B,L,H,d] f32/bf16, g complex64 [B,H,L//2+1].
    flags: 0 or MIX_BF16_SCRATCH (see spectre_mix_forward_ex)."""
    B, L, H, d = v.shape
    prepare(L, d)
    io = _dtype_code(v)
    if g.dtype != torch.complex64 or tuple(g.shape) != (B, H, L // 2 + 1):
        raise ValueError("g must be complex64 [B,H,L//2+1]")
    if out is None:
        out = torch.empty_like(v)
    ws, wsp, wsn = _workspace(mix_workspace_bytes(B, L, H, d, io), v.device, ws)
    _check(lib().spectre_mix_forward_ex(_dev(v, "v"), _dev(g, "g"), _dev(out, "out"), ctypes.c_int(B), ctypes.c_int(L),
                                        ctypes.c_int(H), ctypes.c_int(d), ctypes.c_int(io), ctypes.c_uint(flags),
                                        wsp, wsn, _stream(stream)))
    return out


def mix_forward_static(v, g, out=None, stream=None):
    """mix_forward on the library's built-in scratch array: no workspace, no allocation inside the call
    (spectre_mix_forward_static; four-step lengths, B*H*L <= 4 Mi)."""
    B, L, H, d = v.shape
    if g.dtype != torch.complex64 or tuple(g.shape) != (B, H, L // 2 + 1):
        raise ValueError("g must be complex64 [B,H,L//2+1]")
    if out is None:
        out = torch.empty_like(v)
    _check(lib().spectre_mix_forward_static(_dev(v, "v"), _dev(g, "g"), _dev(out, "out"), ctypes.c_int(B),
                                            ctypes.c_int(L), ctypes.c_int(H), ctypes.c_int(d),
                                            ctypes.c_int(_dtype_code(v)), _stream(stream)))
    return out


def project(x, Wq, Wv, want_q=False, want_sum_q=True, ws=None, stream=None):
    """Per-head token projection (Eq. 2).  x [B,L,H,64] f32/bf16; Wq, Wv float32 [Hw,64,64] (Hw = H or 1).
    Returns (v, q or None, sum_q float64 [B,H,64] or None)."""
    B, L, H, d = x.shape
    io = _dtype_code(x)
    for w in (Wq, Wv):
        if w.dtype != torch.float32 or tuple(w.shape[1:]) != (d, d) or w.shape[0] != Wq.shape[0]:
            raise ValueError("Wq, Wv must be float32 [Hw,d,d]")
    v = torch.empty_like(x)
    q = torch.empty_like(x) if want_q else None
    sq = torch.empty((B, H, d), dtype=torch.float64, device=x.device) if want_sum_q else None
    need = lib().spectre_project_workspace_bytes(ctypes.c_int(B), ctypes.c_int(L), ctypes.c_int(H), ctypes.c_int(d))
    ws, wsp, wsn = _workspace(need, x.device, ws)
    _check(lib().spectre_project(_dev(x, "x"), _dev(Wq, "Wq"), _dev(Wv, "Wv"), ctypes.c_int(Wq.shape[0]),
                                 ctypes.c_int(B), ctypes.c_int(L), ctypes.c_int(H), ctypes.c_int(d), ctypes.c_int(io),
                                 _dev(v, "v"), None if q is None else _dev(q, "q"),
                                 None if sq is None else _dev(sq, "sum_q"), wsp, wsn, _stream(stream)))
    return v, q, sq


class GateParams:
    """Device copies of the gate parameters plus the C parameter block.

    ``params`` uses the paper's row-vector convention (hid = qbar W1, u = hid W2) with
    W1 [Hg,d,d_g] and W2 [Hg,d_g,2F]; the library wants W2 output-major, [Hg,2F,d_g], so it is
    transposed once here while it is copied to the device."""

    def __init__(self, params, device="cuda"):
        def dev(a):
            return None if a is None else torch.as_tensor(a, dtype=torch.float32).to(device).contiguous()
        self.t = {k: dev(params[k]) for k in ("ln_gamma", "ln_beta", "W1", "b1", "b2")}
        self.t["modrelu_bias"] = dev(params.get("modrelu_bias"))
        Hg, d, d_g = self.t["W1"].shape
        self.n_fft = int(params["n_fft"])
        F = self.n_fft // 2 + 1
        w2 = torch.as_tensor(params["W2"], dtype=torch.float32).to(device)
        assert tuple(w2.shape) == (Hg, d_g, 2 * F)
        self.t["W2"] = w2.transpose(1, 2).contiguous()
        del w2
        self.Hg, self.d, self.d_g, self.F = Hg, d, d_g, F
        taps = params.get("toeplitz")
        self.t["toeplitz"], r = None, 0
        if taps is not None:
            taps = torch.as_tensor(taps).to(torch.complex64).to(device).contiguous()
            assert taps.ndim == 2 and taps.shape[0] == Hg and taps.shape[1] % 2 == 1
            self.t["toeplitz"], r = taps, taps.shape[1] // 2
        p = lambda k: None if self.t[k] is None else ctypes.c_void_p(self.t[k].data_ptr())
        self.c = GateParamsC(Hg, d, d_g, self.n_fft, p("ln_gamma"), p("ln_beta"), float(params["ln_eps"]),
                             p("W1"), p("b1"), p("W2"), p("b2"), p("modrelu_bias"), p("toeplitz"), r)


def gate_workspace_bytes(B, L, H, P):
    return int(lib().spectre_gate_workspace_bytes(ctypes.c_int(B), ctypes.c_int(L), ctypes.c_int(H), ctypes.byref(P.c)))


def gate(q, P, inv_count, pooled=False, phase_pos=0, g_out=None, ws=None, stream=None):
    """Spectral gate complex64 [B,H,F].  q: query rows [B,L,H,d] (f32/bf16), or with pooled=True
    their sum over positions as float64 [B,H,d]."""
    if pooled:
        if q.dtype != torch.float64:
            raise TypeError("pooled q must be float64 [B,H,d]")
        B, H, d = q.shape
        L, code = 1, F32
    else:
        B, L, H, d = q.shape
        code = _dtype_code(q)
    if d != P.d:
        raise ValueError("d mismatch")
    if g_out is None:
        g_out = torch.empty((B, H, P.F), dtype=torch.complex64, device=q.device)
    ws, wsp, wsn = _workspace(gate_workspace_bytes(B, L, H, P), q.device, ws)
    _check(lib().spectre_gate(_dev(q, "q"), ctypes.c_int(1 if pooled else 0), ctypes.c_int(code),
                              ctypes.c_double(inv_count), ctypes.byref(P.c), ctypes.c_int(B), ctypes.c_int(L),
                              ctypes.c_int(H), ctypes.c_longlong(int(phase_pos)), _dev(g_out, "g_out"),
                              wsp, wsn, _stream(stream)))
    return g_out


class WrmParams:
    """Device copies of the wavelet-refinement MLP (Sec. 3.5 step b) plus the C parameter block.
    W1 [Hg,d,d_w], b1 [Hg,d_w], W2 [Hg,d_w,(levels+1)*d], b2 [Hg,(levels+1)*d]."""

    def __init__(self, params, device="cuda"):
        self.t = {k: torch.as_tensor(params[k], dtype=torch.float32).to(device).contiguous()
                  for k in ("ln_gamma", "ln_beta", "W1", "b1", "W2", "b2")}
        Hg, d, d_w = self.t["W1"].shape
        self.levels = int(params["levels"])
        assert tuple(self.t["W2"].shape) == (Hg, d_w, (self.levels + 1) * d)
        self.Hg, self.d, self.d_w = Hg, d, d_w
        p = lambda k: ctypes.c_void_p(self.t[k].data_ptr())
        self.c = WrmParamsC(Hg, d, d_w, self.levels, p("ln_gamma"), p("ln_beta"), float(params["ln_eps"]),
                            p("W1"), p("b1"), p("W2"), p("b2"))


def wrm_gates(q, P, inv_count, pooled=False, s_out=None, ws=None, stream=None):
    """Level gates float32 [B,H,levels+1,d] from query rows [B,L,H,d] or (pooled=True) their float64 sum [B,H,d]."""
    if pooled:
        if q.dtype != torch.float64:
            raise TypeError("pooled q must be float64 [B,H,d]")
        B, H, d = q.shape
        L, code = 1, F32
    else:
        B, L, H, d = q.shape
        code = _dtype_code(q)
    if d != P.d:
        raise ValueError("d mismatch")
    if s_out is None:
        s_out = torch.empty((B, H, P.levels + 1, d), dtype=torch.float32, device=q.device)
    need = lib().spectre_wrm_gates_workspace_bytes(ctypes.c_int(B), ctypes.c_int(L), ctypes.c_int(H), ctypes.byref(P.c))
    ws, wsp, wsn = _workspace(need, q.device, ws)
    _check(lib().spectre_wrm_gates(_dev(q, "q"), ctypes.c_int(1 if pooled else 0), ctypes.c_int(code),
                                   ctypes.c_double(inv_count), ctypes.byref(P.c), ctypes.c_int(B), ctypes.c_int(L),
                                   ctypes.c_int(H), _dev(s_out, "s_out"), wsp, wsn, _stream(stream)))
    return s_out


def wrm_apply_workspace_bytes(B, L, H, d, levels):
    return int(lib().spectre_wrm_apply_workspace_bytes(ctypes.c_int(B), ctypes.c_int(L), ctypes.c_int(H),
                                                       ctypes.c_int(d), ctypes.c_int(levels)))


def wrm_apply(v, s, out=None, ws=None, stream=None):
    """v + iDWT(s * DWT(v)) along the sequence axis (Sec. 3.5 steps a, c, d); v [B,L,H,d] f32/bf16,
    s float32 [B,H,levels+1,d].  Pass out=v for in-place operation."""
    B, L, H, d = v.shape
    if s.dtype != torch.float32 or s.ndim != 4 or tuple(s.shape[:2]) != (B, H) or s.shape[3] != d:
        raise ValueError("s must be float32 [B,H,levels+1,d]")
    levels = s.shape[2] - 1
    if out is None:
        out = torch.empty_like(v)
    ws, wsp, wsn = _workspace(wrm_apply_workspace_bytes(B, L, H, d, levels), v.device, ws)
    _check(lib().spectre_wrm_apply(_dev(v, "v"), _dev(s, "s"), _dev(out, "out"), ctypes.c_int(B), ctypes.c_int(L),
                                   ctypes.c_int(H), ctypes.c_int(d), ctypes.c_int(levels),
                                   ctypes.c_int(_dtype_code(v)), wsp, wsn, _stream(stream)))
    return out


def wrm_apply_coeff(v, s, levels, out=None, ws=None, stream=None):
    """v + iDWT(s * DWT(v)) with one gate per wavelet coefficient and channel: v [B,L,H,d] f32/bf16,
    s float32 [B,H,L,d] in the analysis' coefficient order [a_J | d_J | ... | d_1]."""
    B, L, H, d = v.shape
    if s.dtype != torch.float32 or tuple(s.shape) != (B, H, L, d):
        raise ValueError("s must be float32 [B,H,L,d]")
    if out is None:
        out = torch.empty_like(v)
    ws, wsp, wsn = _workspace(wrm_apply_workspace_bytes(B, L, H, d, levels), v.device, ws)
    _check(lib().spectre_wrm_apply_coeff(_dev(v, "v"), _dev(s, "s"), _dev(out, "out"), ctypes.c_int(B), ctypes.c_int(L),
                                         ctypes.c_int(H), ctypes.c_int(d), ctypes.c_int(levels),
                                         ctypes.c_int(_dtype_code(v)), wsp, wsn, _stream(stream)))
    return out


def layer_forward(x, Wq, Wv, P, W=None, out=None, ws=None, stream=None):
    """The whole layer in one call (spectre_layer_forward): projection, pooled query, gate, mixer and, with W (a
    WrmParams), the wavelet refinement.  x [B,L,H,64] f32/bf16; Wq, Wv float32 [Hw,64,64]; P a GateParams for L."""
    B, L, H, d = x.shape
    io = _dtype_code(x)
    prepare(L, d)
    if out is None:
        out = torch.empty_like(x)
    wc = ctypes.byref(W.c) if W is not None else None
    need = lib().spectre_layer_workspace_bytes(ctypes.c_int(B), ctypes.c_int(L), ctypes.c_int(H), ctypes.c_int(d),
                                               ctypes.c_int(io), ctypes.byref(P.c), wc)
    if need == 0:
        raise SpectreError(EUNSUPPORTED, lib().spectre_last_error().decode())
    ws, wsp, wsn = _workspace(need, x.device, ws)
    _check(lib().spectre_layer_forward(_dev(x, "x"), _dev(Wq, "Wq"), _dev(Wv, "Wv"), ctypes.c_int(Wq.shape[0]),
                                       ctypes.byref(P.c), wc, _dev(out, "out"), ctypes.c_int(B), ctypes.c_int(L),
                                       ctypes.c_int(H), ctypes.c_int(d), ctypes.c_int(io), wsp, wsn, _stream(stream)))
    return out


class PrefixCache:
    """Caller-owned Prefix-FFT cache state (Algorithm 1) in device memory."""

    def __init__(self, B, H, d, N_max, N_mem=0, defer=0, device="cuda"):
        """N_max = ring capacity; N_mem = persistent memory rows (Sec. 3.4); n = N_mem + N_max is the transform length.
        defer > 0: step() leaves up to `defer` rank-one updates pending and only reads the cache (see spectre.h)."""
        L = lib()
        n = N_max + N_mem
        self.B, self.H, self.d, self.N, self.N_mem, self.n = B, H, d, N_max, N_mem, n
        self.F = n // 2 + 1
        nb = [int(L.spectre_prefix_bytes(ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(d), ctypes.c_int(n),
                                         ctypes.c_int(w))) for w in range(5)]
        if min(nb) == 0:
            raise SpectreError(EUNSUPPORTED, f"no prefix cache for B={B} H={H} d={d} N_mem+N_max={n}")
        self.prefix_fft = torch.empty((B, H, self.F, d), dtype=torch.complex64, device=device)
        self.v_buf = torch.empty((B, H, n, d), dtype=torch.float32, device=device)
        self.q_buf = torch.empty((B, H, n, d), dtype=torch.float32, device=device)
        self.sum_q = torch.empty((B, H, d), dtype=torch.float64, device=device)
        self.twiddle = torch.empty((n,), dtype=torch.complex64, device=device)
        for t, nbytes in zip((self.prefix_fft, self.v_buf, self.q_buf, self.sum_q, self.twiddle), nb):
            assert t.numel() * t.element_size() == nbytes, (t.shape, nbytes)
        self.pending = torch.zeros((defer, B, H, d), dtype=torch.float32, device=device) if defer > 0 else None
        self.c = PrefixCacheC(B, H, d, N_max, N_mem, 0, self.prefix_fft.data_ptr(), self.v_buf.data_ptr(),
                              self.q_buf.data_ptr(), self.sum_q.data_ptr(), self.twiddle.data_ptr(),
                              self.pending.data_ptr() if defer > 0 else None, defer, 0)
        self._ws = None
        _check(L.spectre_prefix_init(ctypes.byref(self.c), _stream(None)))

    def reset(self, stream=None):
        """Back to the empty cache (t = 0, zero state); memory rows, if any, must be set again."""
        self.c.n_pending = 0
        _check(lib().spectre_prefix_init(ctypes.byref(self.c), _stream(stream)))

    def set_memory(self, mem, stream=None):
        """mem float32 [1 or B, H, N_mem, d]: the persistent memory rows; call once, before any token."""
        if mem.dtype != torch.float32 or mem.ndim != 4 or tuple(mem.shape[1:]) != (self.H, self.N_mem, self.d):
            raise ValueError("mem must be float32 [1 or B, H, N_mem, d]")
        prepare(self.n, self.d)
        need = lib().spectre_prefix_set_memory_workspace_bytes(ctypes.byref(self.c))
        self._ws, wsp, wsn = _workspace(need, mem.device, self._ws)
        _check(lib().spectre_prefix_set_memory(ctypes.byref(self.c), _dev(mem, "mem"), ctypes.c_int(mem.shape[0]),
                                               wsp, wsn, _stream(stream)))

    @property
    def t(self):
        return int(self.c.t)

    @property
    def n_pending(self):
        return int(self.c.n_pending)

    def flush(self, stream=None):
        """Apply the pending deferred updates to prefix_fft."""
        _check(lib().spectre_prefix_flush(ctypes.byref(self.c), _stream(stream)))

    def update(self, v_new, q_new, stream=None):
        B, T, H, d = v_new.shape
        assert (B, H, d) == (self.B, self.H, self.d) and q_new.shape == v_new.shape and q_new.dtype == v_new.dtype
        io = _dtype_code(v_new)
        prepare(self.n, self.d)
        need = lib().spectre_prefix_update_workspace_bytes(ctypes.byref(self.c), ctypes.c_int(T), ctypes.c_int(io))
        self._ws, wsp, wsn = _workspace(need, v_new.device, self._ws)
        _check(lib().spectre_prefix_update(ctypes.byref(self.c), _dev(v_new, "v_new"), _dev(q_new, "q_new"),
                                           ctypes.c_int(T), ctypes.c_int(io), wsp, wsn, _stream(stream)))

    def readout(self, g, mode=READ_NEWEST, dtype=torch.float32, stream=None):
        io = F32 if dtype == torch.float32 else BF16
        prepare(self.n, self.d)
        rows = 1 if mode == READ_NEWEST else min(self.t, self.N)
        out = torch.empty((self.B, rows, self.H, self.d), dtype=dtype, device=g.device)
        need = lib().spectre_prefix_readout_workspace_bytes(ctypes.byref(self.c), ctypes.c_int(mode), ctypes.c_int(io))
        self._ws, wsp, wsn = _workspace(need, g.device, self._ws)
        _check(lib().spectre_prefix_readout(ctypes.byref(self.c), _dev(g, "g"), ctypes.c_int(mode), _dev(out, "out"),
                                            ctypes.c_int(io), wsp, wsn, _stream(stream)))
        return out

    def step(self, v_t, q_t, P, out=None, stream=None):
        io = _dtype_code(v_t)
        if out is None:
            out = torch.empty((self.B, 1, self.H, self.d), dtype=v_t.dtype, device=v_t.device)
        need = lib().spectre_prefix_step_workspace_bytes(ctypes.byref(self.c), ctypes.byref(P.c))
        self._ws, wsp, wsn = _workspace(need, v_t.device, self._ws)
        _check(lib().spectre_prefix_step(ctypes.byref(self.c), _dev(v_t, "v_t"), _dev(q_t, "q_t"), ctypes.byref(P.c),
                                         _dev(out, "out"), ctypes.c_int(io), wsp, wsn, _stream(stream)))
        return out
