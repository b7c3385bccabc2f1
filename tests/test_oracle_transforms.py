"""Pins for the oracle's transforms (Sec. 3.1 Eq. 1; App. B Thm. B.1, Cor. B.2).

The oracle is checked against things other than itself: hand-evaluated fixtures,
closed forms, invariants the paper proves, and numpy's FFT as a library routine.
"""
import os

import numpy as np
import pytest

LENGTHS = [2, 3, 4, 5, 7, 8, 16, 49, 64, 196]
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "dft_small.txt")


def _rng(seed):
    return np.random.default_rng(seed)


def test_golden_hand_values(oracle):
    """Eq. (1) on inputs small enough to evaluate by hand."""
    n_cases = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        n_s, x_s, X_s = [p.strip() for p in line.split("|")]
        n = int(n_s)
        x = np.array([float(v) for v in x_s.split()])
        flat = np.array([float(v) for v in X_s.split()])
        want = flat[0::2] + 1j * flat[1::2]
        assert x.shape == (n,) and want.shape == (n // 2 + 1,)
        for method in (oracle.NAIVE, oracle.FAST):
            got = oracle.rfft(x, method)
            np.testing.assert_allclose(got, want, rtol=0, atol=1e-14)
        full = oracle.dft_naive(x.astype(complex), -1)
        np.testing.assert_allclose(full[: n // 2 + 1], want, rtol=0, atol=1e-14)
        n_cases += 1
    assert n_cases >= 8


@pytest.mark.parametrize("n", LENGTHS)
def test_delta_and_constant_closed_forms(oracle, n):
    """Impulse at t0 -> X_k = exp(-j 2 pi k t0/n); constant c -> X_0 = n c, others 0."""
    k = np.arange(n // 2 + 1)
    for t0 in {0, 1, n // 2, n - 1}:
        x = np.zeros(n)
        x[t0] = 1.0
        want = np.exp(-2j * np.pi * ((k * t0) % n) / n)
        for method in (oracle.NAIVE, oracle.FAST):
            np.testing.assert_allclose(oracle.rfft(x, method), want, atol=1e-13)
    c = -2.5
    want = np.zeros(n // 2 + 1, complex)
    want[0] = n * c
    for method in (oracle.NAIVE, oracle.FAST):
        np.testing.assert_allclose(oracle.rfft(np.full(n, c), method), want, atol=1e-12)


@pytest.mark.parametrize("n", LENGTHS + [256, 1024])
def test_complex_dft_matches_library_and_itself(oracle, n):
    r = _rng(n)
    x = r.standard_normal(n) + 1j * r.standard_normal(n)
    for sign, lib in ((-1, np.fft.fft(x)), (+1, np.fft.ifft(x) * n)):
        fast = oracle.fft(x, sign)
        np.testing.assert_allclose(fast, lib, atol=1e-11 * np.sqrt(n))
        if n <= 256:
            naive = oracle.dft_naive(x, sign)
            np.testing.assert_allclose(naive, lib, atol=1e-11 * np.sqrt(n))


def test_single_tone_lands_in_one_bin(oracle):
    """exp(+j 2 pi f t/n) transforms to n at bin f and 0 elsewhere (sign convention of Eq. 1)."""
    n, f = 16, 3
    x = np.exp(2j * np.pi * f * np.arange(n) / n)
    for X in (oracle.dft_naive(x, -1), oracle.fft(x, -1)):
        want = np.zeros(n, complex)
        want[f] = n
        np.testing.assert_allclose(X, want, atol=1e-12)


@pytest.mark.parametrize("n", LENGTHS)
def test_hermitian_symmetry_and_real_dc_nyquist(oracle, n):
    """Thm. B.1: X_{n-k} = conj(X_k); DC and (n even) Nyquist are real."""
    x = _rng(100 + n).standard_normal(n)
    X = oracle.dft_naive(x.astype(complex), -1)
    for k in range(1, n):
        assert abs(X[n - k] - np.conj(X[k])) < 1e-11
    assert abs(X[0].imag) < 1e-12
    if n % 2 == 0:
        assert abs(X[n // 2].imag) < 1e-11
    half = oracle.rfft(x, oracle.FAST)
    np.testing.assert_allclose(half, X[: n // 2 + 1], atol=1e-11)
    assert half.shape == (n // 2 + 1,)  # odd n: ceil(n/2) bins (Remark after Cor. B.2)


@pytest.mark.parametrize("n", LENGTHS)
def test_parseval(oracle, n):
    x = _rng(200 + n).standard_normal(n)
    for method in (oracle.NAIVE, oracle.FAST):
        X = oracle.rfft(x, method)
        w = np.full(n // 2 + 1, 2.0)
        w[0] = 1.0
        if n % 2 == 0:
            w[-1] = 1.0
        assert abs((w * np.abs(X) ** 2).sum() / n - (x ** 2).sum()) < 1e-10 * n


@pytest.mark.parametrize("n", LENGTHS + [512])
def test_rfft_irfft_against_library(oracle, n):
    r = _rng(300 + n)
    x = r.standard_normal(n)
    for method in (oracle.NAIVE, oracle.FAST):
        np.testing.assert_allclose(oracle.rfft(x, method), np.fft.rfft(x), atol=1e-11 * np.sqrt(n))
    # arbitrary half spectrum, including non-real DC / Nyquist: the library's
    # complex-to-real inverse also keeps only their real parts
    Y = r.standard_normal(n // 2 + 1) + 1j * r.standard_normal(n // 2 + 1)
    want = np.fft.irfft(Y, n)
    for method in (oracle.NAIVE, oracle.FAST):
        np.testing.assert_allclose(oracle.irfft(Y, n, method), want, atol=1e-12 * np.sqrt(n))


@pytest.mark.parametrize("n", LENGTHS)
def test_lossless_round_trip(oracle, n):
    """Cor. B.2: the half spectrum reconstructs the sequence exactly."""
    x = _rng(400 + n).standard_normal(n)
    for m1 in (oracle.NAIVE, oracle.FAST):
        for m2 in (oracle.NAIVE, oracle.FAST):
            np.testing.assert_allclose(oracle.irfft(oracle.rfft(x, m1), n, m2), x, atol=1e-12)


def test_irfft_drops_imag_of_dc_and_nyquist(oracle):
    n = 8
    Y = np.zeros(n // 2 + 1, complex)
    Y[0] = 1j * 3.0
    Y[-1] = 1j * 5.0
    for method in (oracle.NAIVE, oracle.FAST):
        np.testing.assert_allclose(oracle.irfft(Y, n, method), np.zeros(n), atol=1e-15)
    Y[0] = 8.0
    np.testing.assert_allclose(oracle.irfft(Y, n), np.ones(n), atol=1e-15)
    Y[0] = 0
    Y[-1] = 8.0
    np.testing.assert_allclose(oracle.irfft(Y, n), (-1.0) ** np.arange(n), atol=1e-15)


def test_fast_transform_large_matches_library(oracle):
    """The length the headline benchmark runs at, and the ViT length."""
    for n in (131072, 32768, 196):
        x = _rng(n).standard_normal(n)
        X = oracle.rfft(x)
        np.testing.assert_allclose(X, np.fft.rfft(x), atol=1e-9)
        np.testing.assert_allclose(oracle.irfft(X, n), x, atol=1e-12)
