"""numpy front end of the fp64 C oracle (``spectre_oracle.c``).

TEST INFRASTRUCTURE ONLY (see the C file's header).  Argument marshalling and
nothing else: every number is produced by the C code.  All arrays are float64 /
complex128, C-contiguous; shapes follow the paper's notation:

    V, Q       [B, L, H, d]      value / query rows per head (Sec. 3.2 Eq. 2)
    g          [B, H, F]         complex gate, F = L//2 + 1   (Sec. 3.2 step 3)
    spec       [B, H, F, d]      Prefix-FFT cache             (Sec. 3.3, Alg. 1)
    v_buf,q_buf[B, H, N, d]      ring buffers
    sum_q      [B, H, d]         running query sum
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# The two variables let the planted-mistake test point a child test run at a deliberately wrong copy of the source.
_SRC = os.environ.get("SPECTRE_ORACLE_SOURCE", os.path.join(_HERE, "spectre_oracle.c"))
_LIB = os.environ.get("SPECTRE_ORACLE_LIBRARY", os.path.join(_HERE, "libspectre_oracle.so"))

NAIVE = 0   # the O(n^2) sums exactly as printed
FAST = 1    # radix-2 FFT (Bluestein for other lengths)


def build(force=False):
    """Compile the C oracle with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _c128(a):
    return np.ascontiguousarray(a, dtype=np.complex128)


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def num_threads():
    return int(_L().so_num_threads())


def dft_naive(x, sign=-1):
    x = _c128(x)
    out = np.empty_like(x)
    _L().so_dft_naive(ctypes.c_int(x.shape[0]), ctypes.c_int(sign), _p(x), _p(out))
    return out


def fft(x, sign=-1):
    x = _c128(x)
    out = np.empty_like(x)
    rc = _L().so_fft(ctypes.c_int(x.shape[0]), ctypes.c_int(sign), _p(x), _p(out))
    if rc:
        raise RuntimeError(f"so_fft rc={rc}")
    return out


def rfft(x, method=FAST):
    x = _f64(x)
    n = x.shape[0]
    out = np.empty(n // 2 + 1, dtype=np.complex128)
    rc = _L().so_rfft(ctypes.c_int(n), _p(x), _p(out), ctypes.c_int(method))
    if rc:
        raise RuntimeError(f"so_rfft rc={rc}")
    return out


def irfft(Y, n, method=FAST):
    Y = _c128(Y)
    assert Y.shape[0] == n // 2 + 1
    out = np.empty(n, dtype=np.float64)
    rc = _L().so_irfft(ctypes.c_int(n), _p(Y), _p(out), ctypes.c_int(method))
    if rc:
        raise RuntimeError(f"so_irfft rc={rc}")
    return out


def project(X, Wq, Wv):
    """Q = X W^(q), V = X W^(v) per head (Eq. 2); X [B,L,H,d], Wq/Wv [Hw,d,d]."""
    X, Wq, Wv = _f64(X), _f64(Wq), _f64(Wv)
    B, L, H, d = X.shape
    Hw = Wq.shape[0]
    assert Wq.shape == (Hw, d, d) and Wv.shape == (Hw, d, d)
    Q, V = np.empty_like(X), np.empty_like(X)
    rc = _L().so_project(ctypes.c_int(B), ctypes.c_int(L), ctypes.c_int(H), ctypes.c_int(d), ctypes.c_int(Hw),
                         _p(X), _p(Wq), _p(Wv), _p(Q), _p(V))
    if rc:
        raise RuntimeError(f"so_project rc={rc}")
    return Q, V


def pool_q(Q):
    Q = _f64(Q)
    B, L, H, d = Q.shape
    out = np.empty((B, H, d), dtype=np.float64)
    _L().so_pool_q(ctypes.c_int(B), ctypes.c_int(L), ctypes.c_int(H), ctypes.c_int(d), _p(Q), _p(out))
    return out


def gate(sum_q, inv_count, params, n, phase_pos=0):
    """Gate from a pooled query sum.  ``params`` is a dict with ln_gamma, ln_beta
    [Hg,d], ln_eps, W1 [Hg,d,dg], b1 [Hg,dg], W2 [Hg,dg,2F], b2 [Hg,2F],
    modrelu_bias [Hg,F] or None, toeplitz [Hg,2r+1] complex or None (tap m at index m+r)."""
    sum_q = _f64(sum_q)
    B, H, d = sum_q.shape
    W1 = _f64(params["W1"])
    Hg, d_, dg = W1.shape
    assert d_ == d
    F = n // 2 + 1
    W2 = _f64(params["W2"])
    assert W2.shape == (Hg, dg, 2 * F), (W2.shape, (Hg, dg, 2 * F))
    gam, bet = _f64(params["ln_gamma"]), _f64(params["ln_beta"])
    b1, b2 = _f64(params["b1"]), _f64(params["b2"])
    assert gam.shape == (Hg, d) and bet.shape == (Hg, d) and b1.shape == (Hg, dg) and b2.shape == (Hg, 2 * F)
    bias = params.get("modrelu_bias")
    if bias is not None:
        bias = _f64(bias)
        assert bias.shape == (Hg, F)
    taps = params.get("toeplitz")
    r = 0
    if taps is not None:
        taps = _c128(taps)
        assert taps.ndim == 2 and taps.shape[0] == Hg and taps.shape[1] % 2 == 1
        r = taps.shape[1] // 2
    out = np.empty((B, H, F), dtype=np.complex128)
    rc = _L().so_gate(ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(d), ctypes.c_int(dg),
                      ctypes.c_int(n), ctypes.c_int(Hg), _p(sum_q), ctypes.c_double(inv_count),
                      _p(gam), _p(bet), ctypes.c_double(float(params["ln_eps"])),
                      _p(W1), _p(b1), _p(W2), _p(b2), _p(bias), _p(taps), ctypes.c_int(r),
                      ctypes.c_longlong(int(phase_pos)), _p(out))
    if rc:
        raise RuntimeError(f"so_gate rc={rc}")
    return out


def mix_forward(V, g, method=FAST):
    V = _f64(V)
    g = _c128(g)
    B, L, H, d = V.shape
    assert g.shape == (B, H, L // 2 + 1)
    out = np.empty_like(V)
    rc = _L().so_mix_forward(ctypes.c_int(B), ctypes.c_int(L), ctypes.c_int(H), ctypes.c_int(d),
                             _p(V), _p(g), _p(out), ctypes.c_int(method))
    if rc:
        raise RuntimeError(f"so_mix_forward rc={rc}")
    return out


def haar_fwd(x, J):
    """Orthonormal Haar analysis of a 1-D array, J levels, output [a_J | d_J | ... | d_1] (Sec. 3.5 step a)."""
    x = _f64(x)
    w = np.empty_like(x)
    rc = _L().so_haar_fwd(ctypes.c_int(x.shape[0]), ctypes.c_int(J), _p(x), _p(w))
    if rc:
        raise RuntimeError(f"so_haar_fwd rc={rc}")
    return w


def haar_inv(w, J):
    w = _f64(w)
    x = np.empty_like(w)
    rc = _L().so_haar_inv(ctypes.c_int(w.shape[0]), ctypes.c_int(J), _p(w), _p(x))
    if rc:
        raise RuntimeError(f"so_haar_inv rc={rc}")
    return x


def wrm_gates(sum_q, inv_count, params, J):
    """Level gates s [B,H,J+1,d] (Sec. 3.5 step b).  ``params``: ln_gamma, ln_beta [Hg,d], ln_eps,
    W1 [Hg,d,dw], b1 [Hg,dw], W2 [Hg,dw,(J+1)*d], b2 [Hg,(J+1)*d]."""
    sum_q = _f64(sum_q)
    B, H, d = sum_q.shape
    W1 = _f64(params["W1"])
    Hg, d_, dw = W1.shape
    assert d_ == d
    nout = (J + 1) * d
    W2, b1, b2 = _f64(params["W2"]), _f64(params["b1"]), _f64(params["b2"])
    gam, bet = _f64(params["ln_gamma"]), _f64(params["ln_beta"])
    assert W2.shape == (Hg, dw, nout) and b2.shape == (Hg, nout) and b1.shape == (Hg, dw)
    assert gam.shape == (Hg, d) and bet.shape == (Hg, d)
    out = np.empty((B, H, J + 1, d), dtype=np.float64)
    rc = _L().so_wrm_gates(ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(d), ctypes.c_int(dw), ctypes.c_int(J),
                           ctypes.c_int(Hg), _p(sum_q), ctypes.c_double(inv_count), _p(gam), _p(bet),
                           ctypes.c_double(float(params["ln_eps"])), _p(W1), _p(b1), _p(W2), _p(b2), _p(out))
    if rc:
        raise RuntimeError(f"so_wrm_gates rc={rc}")
    return out


def wrm_apply(V, s, J):
    """V + iDWT(s * DWT(V)) along the sequence axis (Sec. 3.5 steps a, c, d); V [B,L,H,d], s [B,H,J+1,d]."""
    V = _f64(V)
    s = _f64(s)
    B, L, H, d = V.shape
    assert s.shape == (B, H, J + 1, d)
    out = np.empty_like(V)
    rc = _L().so_wrm_apply(ctypes.c_int(B), ctypes.c_int(L), ctypes.c_int(H), ctypes.c_int(d), ctypes.c_int(J),
                           _p(V), _p(s), _p(out))
    if rc:
        raise RuntimeError(f"so_wrm_apply rc={rc}")
    return out


def wrm_apply_coeff(V, s, J):
    """The same module with one gate per wavelet coefficient and channel, the shape Sec. 3.5 step (b) prints:
    V [B,L,H,d], s [B,H,L,d] in the analysis' coefficient order [a_J | d_J | ... | d_1]."""
    V = _f64(V)
    s = _f64(s)
    B, L, H, d = V.shape
    assert s.shape == (B, H, L, d)
    out = np.empty_like(V)
    rc = _L().so_wrm_apply_coeff(ctypes.c_int(B), ctypes.c_int(L), ctypes.c_int(H), ctypes.c_int(d), ctypes.c_int(J),
                                 _p(V), _p(s), _p(out))
    if rc:
        raise RuntimeError(f"so_wrm_apply_coeff rc={rc}")
    return out


class PrefixCache:
    """State of Algorithm 1 for B*H heads; ``t`` counts the tokens appended."""

    def __init__(self, B, H, d, N):
        self.B, self.H, self.d, self.N = B, H, d, N
        self.F = N // 2 + 1
        self.t = 0
        self.spec = np.zeros((B, H, self.F, d), dtype=np.complex128)
        self.v_buf = np.zeros((B, H, N, d), dtype=np.float64)
        self.q_buf = np.zeros((B, H, N, d), dtype=np.float64)
        self.sum_q = np.zeros((B, H, d), dtype=np.float64)

    def _dims(self):
        return (ctypes.c_int(self.B), ctypes.c_int(self.H), ctypes.c_int(self.d), ctypes.c_int(self.N))

    def prefill(self, V, Q, method=FAST):
        V, Q = _f64(V), _f64(Q)
        B, T, H, d = V.shape
        assert (B, H, d) == (self.B, self.H, self.d) and Q.shape == V.shape and self.t == 0
        rc = _L().so_prefix_prefill(*self._dims(), ctypes.c_int(T), _p(V), _p(Q), _p(self.spec),
                                    _p(self.v_buf), _p(self.q_buf), _p(self.sum_q), ctypes.c_int(method))
        if rc:
            raise RuntimeError(f"so_prefix_prefill rc={rc}")
        self.t = T

    def update(self, v_t, q_t):
        """Append one token; v_t, q_t are [B,1,H,d] or [B,H,d]."""
        v_t = _f64(v_t).reshape(self.B, self.H, self.d)
        q_t = _f64(q_t).reshape(self.B, self.H, self.d)
        _L().so_prefix_update(*self._dims(), ctypes.c_longlong(self.t), _p(v_t), _p(q_t), _p(self.spec),
                              _p(self.v_buf), _p(self.q_buf), _p(self.sum_q))
        self.t += 1

    def readout_row(self, g, m):
        g = _c128(g)
        assert g.shape == (self.B, self.H, self.F)
        out = np.empty((self.B, self.H, self.d), dtype=np.float64)
        _L().so_prefix_readout_row(*self._dims(), ctypes.c_longlong(int(m)), _p(self.spec), _p(g), _p(out))
        return out

    def readout_newest(self, g):
        """Row of the newest token, slot (t-1) mod N; returned as [B,1,H,d]."""
        return self.readout_row(g, (self.t - 1) % self.N).reshape(self.B, 1, self.H, self.d)

    def readout_window(self, g, method=FAST):
        """Rows N-L'..N-1 of the inverse transform, L' = min(t, N); [B,L',H,d]."""
        g = _c128(g)
        Lw = min(self.t, self.N)
        out = np.empty((self.B, Lw, self.H, self.d), dtype=np.float64)
        rc = _L().so_prefix_readout_window(*self._dims(), ctypes.c_int(Lw), _p(self.spec), _p(g), _p(out),
                                           ctypes.c_int(method))
        if rc:
            raise RuntimeError(f"so_prefix_readout_window rc={rc}")
        return out


class MemoryPrefixCache:
    """Prefix-FFT cache with a persistent memory bank (Sec. 3.4): a window of n = N_mem + N_max rows whose
    first N_mem rows are the memory M [B,H,N_mem,d] and whose other rows are the ring buffer."""

    def __init__(self, B, H, d, N_mem, N_max):
        self.B, self.H, self.d, self.N_mem, self.N_max = B, H, d, N_mem, N_max
        self.n = N_mem + N_max
        self.F = self.n // 2 + 1
        self.t = 0
        self.spec = np.zeros((B, H, self.F, d), dtype=np.complex128)
        self.v_buf = np.zeros((B, H, self.n, d), dtype=np.float64)
        self.q_buf = np.zeros((B, H, self.n, d), dtype=np.float64)
        self.sum_q = np.zeros((B, H, d), dtype=np.float64)

    def _dims(self):
        return (ctypes.c_int(self.B), ctypes.c_int(self.H), ctypes.c_int(self.d), ctypes.c_int(self.N_mem),
                ctypes.c_int(self.N_max))

    def prefill(self, M, V=None, Q=None, method=FAST):
        """Lay down the memory and (optionally) a prompt V, Q [B,T,H,d], transform once."""
        M = _f64(M)
        assert M.shape == (self.B, self.H, self.N_mem, self.d) and self.t == 0
        if V is None:
            V = np.zeros((self.B, 0, self.H, self.d))
            Q = V
        V, Q = _f64(V), _f64(Q)
        T = V.shape[1]
        assert V.shape == (self.B, T, self.H, self.d) and Q.shape == V.shape
        rc = _L().so_memory_prefill(*self._dims(), ctypes.c_int(T), _p(M), _p(V), _p(Q), _p(self.spec),
                                    _p(self.v_buf), _p(self.q_buf), _p(self.sum_q), ctypes.c_int(method))
        if rc:
            raise RuntimeError(f"so_memory_prefill rc={rc}")
        self.t = T

    def update(self, v_t, q_t):
        v_t = _f64(v_t).reshape(self.B, self.H, self.d)
        q_t = _f64(q_t).reshape(self.B, self.H, self.d)
        _L().so_memory_update(*self._dims(), ctypes.c_longlong(self.t), _p(v_t), _p(q_t), _p(self.spec),
                              _p(self.v_buf), _p(self.q_buf), _p(self.sum_q))
        self.t += 1

    def newest_slot(self):
        return self.N_mem + (self.t - 1) % self.N_max

    def readout_row(self, g, m):
        g = _c128(g)
        assert g.shape == (self.B, self.H, self.F)
        out = np.empty((self.B, self.H, self.d), dtype=np.float64)
        _L().so_prefix_readout_row(ctypes.c_int(self.B), ctypes.c_int(self.H), ctypes.c_int(self.d),
                                   ctypes.c_int(self.n), ctypes.c_longlong(int(m)), _p(self.spec), _p(g), _p(out))
        return out

    def readout_newest(self, g):
        return self.readout_row(g, self.newest_slot()).reshape(self.B, 1, self.H, self.d)

    def readout_window(self, g, method=FAST):
        """The live tokens' rows of irfft_n(g * spec), oldest first; [B, min(t, N_max), H, d]."""
        g = _c128(g)
        Lw = min(self.t, self.N_max)
        out = np.empty((self.B, Lw, self.H, self.d), dtype=np.float64)
        rc = _L().so_memory_readout_window(*self._dims(), ctypes.c_longlong(self.t), _p(self.spec), _p(g), _p(out),
                                           ctypes.c_int(method))
        if rc:
            raise RuntimeError(f"so_memory_readout_window rc={rc}")
        return out
