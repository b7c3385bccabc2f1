"""Pins for the oracle's persistent memory extension of the Prefix-FFT cache (Sec. 3.4).

Sec. 3.4's literal concatenation of two half spectra is the spectrum of no signal, so the reading is
unpinned by the paper; under it (memory = the first N_mem rows of an (N_mem + N_max)-row window) the
mathematics fixes everything: the cache equals the transform of the window after every token, the
memory rows never change, the queries of the memory do not exist, readouts equal rows of a from-scratch
mixing of the window, and with no memory the plain cache is recovered bit for bit."""
import numpy as np
import pytest


def _rng(seed):
    return np.random.default_rng(seed)


def _run(oracle, B, H, d, N_mem, N_max, T0, steps, seed, check=None):
    r = _rng(seed)
    M = r.standard_normal((B, H, N_mem, d))
    c = oracle.MemoryPrefixCache(B, H, d, N_mem, N_max)
    toks_v, toks_q = [], []
    if T0:
        V, Q = r.standard_normal((B, T0, H, d)), r.standard_normal((B, T0, H, d))
        c.prefill(M, V, Q, oracle.NAIVE if c.n <= 32 else oracle.FAST)
        toks_v += [V[:, i] for i in range(T0)]
        toks_q += [Q[:, i] for i in range(T0)]
    else:
        c.prefill(M)
    if check:
        check(c, M, toks_v, toks_q)
    for _ in range(steps):
        v, q = r.standard_normal((B, 1, H, d)), r.standard_normal((B, 1, H, d))
        c.update(v, q)
        toks_v.append(v[:, 0])
        toks_q.append(q[:, 0])
        if check:
            check(c, M, toks_v, toks_q)
    return c, M, toks_v, toks_q


@pytest.mark.parametrize("N_mem,N_max,T0,steps", [(2, 6, 3, 20), (4, 12, 0, 40), (16, 48, 48, 100), (3, 13, 5, 30),
                                                  (8, 248, 100, 520)])
def test_cache_is_the_transform_of_memory_plus_ring_after_every_token(oracle, N_mem, N_max, T0, steps):
    B, H, d = 2, 2, 3

    def check(c, M, tv, tq):
        np.testing.assert_allclose(c.spec, np.fft.rfft(c.v_buf, axis=2), atol=1e-9)
        np.testing.assert_array_equal(c.v_buf[:, :, :N_mem], M)              # never evicted, never touched
        assert np.all(c.q_buf[:, :, :N_mem] == 0)                            # memory rows carry no query
        live = tq[-N_max:]
        np.testing.assert_allclose(c.sum_q, sum(live) if live else 0.0, atol=1e-11)
        t = c.t
        for j in range(max(0, t - N_max), t):                                 # token j sits at row N_mem + j mod N_max
            np.testing.assert_array_equal(c.v_buf[:, :, N_mem + j % N_max], tv[j])
        if t < N_max:
            assert np.all(c.v_buf[:, :, N_mem + t:] == 0)

    c, *_ = _run(oracle, B, H, d, N_mem, N_max, T0, steps, seed=N_mem * 100 + N_max, check=check)
    assert c.t >= 2 * N_max + 1                                               # at least two wrap-arounds


def test_without_memory_it_is_the_plain_cache(oracle):
    B, H, d, N = 1, 2, 4, 16
    r = _rng(3)
    V, Q = r.standard_normal((B, 10, H, d)), r.standard_normal((B, 10, H, d))
    a = oracle.PrefixCache(B, H, d, N)
    a.prefill(V, Q)
    b = oracle.MemoryPrefixCache(B, H, d, 0, N)
    b.prefill(np.zeros((B, H, 0, d)), V, Q)
    g = r.standard_normal((B, H, N // 2 + 1)) + 1j * r.standard_normal((B, H, N // 2 + 1))
    for _ in range(40):
        v, q = r.standard_normal((B, 1, H, d)), r.standard_normal((B, 1, H, d))
        a.update(v, q)
        b.update(v, q)
        np.testing.assert_array_equal(a.spec, b.spec)
        np.testing.assert_array_equal(a.sum_q, b.sum_q)
        np.testing.assert_array_equal(a.readout_newest(g), b.readout_newest(g))


@pytest.mark.parametrize("t_extra", [0, 7, 30])
def test_readouts_are_rows_of_a_from_scratch_mixing_of_the_window(oracle, t_extra):
    B, H, d, N_mem, N_max = 2, 2, 3, 4, 12
    c, M, tv, tq = _run(oracle, B, H, d, N_mem, N_max, 5, t_extra, seed=11 + t_extra)
    r = _rng(12)
    g = r.standard_normal((B, H, c.F)) + 1j * r.standard_normal((B, H, c.F))
    window = np.moveaxis(c.v_buf, 2, 1)                                       # [B, n, H, d]
    z = oracle.mix_forward(window, g, oracle.NAIVE)
    np.testing.assert_allclose(c.readout_newest(g)[:, 0], z[:, c.newest_slot()], atol=1e-11)
    out = c.readout_window(g)
    Lw = min(c.t, N_max)
    assert out.shape == (B, Lw, H, d)
    for i in range(Lw):
        tok = c.t - Lw + i
        np.testing.assert_allclose(out[:, i], z[:, N_mem + tok % N_max], atol=1e-11)
        np.testing.assert_array_equal(window[:, N_mem + tok % N_max], tv[tok])   # that row is token `tok`
    # time-domain cross-check: circular convolution of the window with kappa = irfft(gate)
    kap = np.fft.irfft(np.where((np.arange(c.F) == 0) | (2 * np.arange(c.F) == c.n), g.real, g), n=c.n, axis=2)
    s = c.newest_slot()
    want = np.einsum("bhm,bmhc->bhc", kap[:, :, (s - np.arange(c.n)) % c.n], window)
    np.testing.assert_allclose(c.readout_newest(g)[:, 0], want, atol=1e-11)


def test_the_mixing_sees_the_memory(oracle):
    """A pure-shift gate moves row (slot - s) of the window to the newest token's row: choosing s so that
    the source row is a memory row returns that memory row - long after any ring row would have been evicted."""
    B, H, d, N_mem, N_max = 1, 1, 2, 4, 12
    c, M, tv, tq = _run(oracle, B, H, d, N_mem, N_max, 0, 50, seed=21)
    n, k = c.n, np.arange(c.F)
    for m in range(N_mem):
        s = (c.newest_slot() - m) % n
        g = np.broadcast_to(np.exp(-2j * np.pi * ((k * s) % n) / n), (B, H, c.F))
        np.testing.assert_allclose(c.readout_newest(g)[:, 0], M[:, :, m], atol=1e-12)
    g1 = np.ones((B, H, c.F), complex)                                         # identity gate: the newest token itself
    np.testing.assert_allclose(c.readout_newest(g1)[:, 0], tv[-1], atol=1e-12)
    # and the readout depends on M: another memory, same tokens, different answer
    r = _rng(22)
    g = r.standard_normal((B, H, c.F)) + 1j * r.standard_normal((B, H, c.F))
    c2 = oracle.MemoryPrefixCache(B, H, d, N_mem, N_max)
    c2.prefill(M + 1.0)
    for v, q in zip(tv, tq):
        c2.update(v, q)
    assert np.abs(c2.readout_newest(g) - c.readout_newest(g)).max() > 1e-3


def test_prompt_longer_than_the_ring_is_refused(oracle):
    c = oracle.MemoryPrefixCache(1, 1, 2, 2, 6)
    with pytest.raises(RuntimeError):
        c.prefill(np.zeros((1, 1, 2, 2)), np.zeros((1, 7, 1, 2)), np.zeros((1, 7, 1, 2)))
