"""Pins of the oracle's wavelet refinement (Sec. 3.5) against what the mathematics fixes.

The paper prints no worked example for this module and leaves the wavelet family and the gate
shape open (parity for those choices is unpinned by the paper); under the stated reading
(orthonormal Haar, one gate per band and channel) the checks below fix every line of the oracle:
a hand-computed transform, the explicit basis matrix, orthogonality, perfect reconstruction, and
a closed form of the whole module in terms of block means that shares no step with it."""
import numpy as np
import pytest

from paper_2502_18394_amd import synth



def haar_matrix(n, J):
    """Rows = the basis functions in the oracle's coefficient order, written from their definition:
    the approximation of a block of 2^J samples is its sum / sqrt(2^J); the detail of level l of a
    block of 2^l samples is (sum of first half - sum of second half) / sqrt(2^l)."""
    W = np.zeros((n, n))
    r = 0
    blk = 1 << J
    for i in range(n // blk):
        W[r, i * blk:(i + 1) * blk] = 1.0 / np.sqrt(blk)
        r += 1
    for l in range(J, 0, -1):
        blk = 1 << l
        for i in range(n // blk):
            W[r, i * blk:i * blk + blk // 2] = 1.0 / np.sqrt(blk)
            W[r, i * blk + blk // 2:(i + 1) * blk] = -1.0 / np.sqrt(blk)
            r += 1
    assert r == n
    return W


def test_hand_computed_four_points(oracle):
    x = np.array([1.0, 2.0, 3.0, 4.0])
    r = np.sqrt(0.5)
    np.testing.assert_allclose(oracle.haar_fwd(x, 1), [3 * r, 7 * r, -r, -r], atol=1e-15)
    np.testing.assert_allclose(oracle.haar_fwd(x, 2), [5.0, -2.0, -r, -r], atol=1e-15)
    np.testing.assert_allclose(oracle.haar_fwd(x, 0), x, atol=0)


@pytest.mark.parametrize("n,J", [(2, 1), (8, 3), (8, 2), (16, 4), (12, 2), (196, 2), (40, 3), (7, 0)])
def test_equals_explicit_orthogonal_basis(oracle, n, J):
    rng = np.random.default_rng(n + J)
    x = rng.standard_normal(n)
    W = haar_matrix(n, J)
    np.testing.assert_allclose(W @ W.T, np.eye(n), atol=1e-13)         # "orthogonal DWT"
    np.testing.assert_allclose(oracle.haar_fwd(x, J), W @ x, atol=1e-13)
    np.testing.assert_allclose(oracle.haar_inv(x, J), W.T @ x, atol=1e-13)


@pytest.mark.parametrize("n", [2, 64, 196, 1000, 1024, 3 * 4096])
def test_parseval_and_perfect_reconstruction(oracle, n):
    J = synth.max_wavelet_levels(n)
    rng = np.random.default_rng(n)
    x = rng.standard_normal(n)
    w = oracle.haar_fwd(x, J)
    assert abs(np.sum(w * w) - np.sum(x * x)) <= 1e-12 * np.sum(x * x)
    np.testing.assert_allclose(oracle.haar_inv(w, J), x, atol=1e-13)
    # the approximation band of a full-depth analysis of 2^J points is sum / sqrt n
    if n == 1 << J:
        assert abs(w[0] - x.sum() / np.sqrt(n)) < 1e-12


def test_invalid_depth_is_refused(oracle):
    with pytest.raises(RuntimeError):
        oracle.haar_fwd(np.zeros(12), 3)


def block_mean(V, size):
    B, L, H, d = V.shape
    m = V.reshape(B, L // size, size, H, d).mean(axis=2, keepdims=True)
    return np.broadcast_to(m, (B, L // size, size, H, d)).reshape(B, L, H, d)


def closed_form(V, s, J):
    """V + sum over bands of gate * (projection of V on the band).  The projection on the span of the
    level-l approximations is the mean over aligned blocks of 2^l samples, A_l (A_0 = V); the details of
    level l span the difference A_(l-1) - A_l."""
    out = V.copy()
    sb = s[:, None]                                   # [B,1,H,J+1,d]
    for l in range(1, J + 1):
        out += sb[:, :, :, l] * (block_mean(V, 1 << (l - 1)) - block_mean(V, 1 << l))
    out += sb[:, :, :, 0] * block_mean(V, 1 << J)
    return out


@pytest.mark.parametrize("B,L,H,d,J", [(2, 64, 3, 4, 6), (1, 196, 2, 8, 2), (1, 1024, 1, 64, 10), (2, 96, 2, 6, 3),
                                       (1, 4096, 2, 64, 5), (1, 50, 1, 2, 1), (1, 9, 2, 2, 0)])
def test_module_equals_block_mean_closed_form(oracle, B, L, H, d, J):
    rng = np.random.default_rng(L + J)
    V = rng.standard_normal((B, L, H, d))
    s = rng.standard_normal((B, H, J + 1, d))
    np.testing.assert_allclose(oracle.wrm_apply(V, s, J), closed_form(V, s, J), atol=1e-12)


def test_module_special_gates(oracle):
    rng = np.random.default_rng(5)
    B, L, H, d, J = 2, 128, 2, 4, 7
    V = rng.standard_normal((B, L, H, d))
    zero = np.zeros((B, H, J + 1, d))
    np.testing.assert_allclose(oracle.wrm_apply(V, zero, J), V, atol=0)                   # gates 0: skipped
    np.testing.assert_allclose(oracle.wrm_apply(V, zero + 1.0, J), 2.0 * V, atol=1e-13)   # gates 1: iDWT(DWT V) = V
    s = zero.copy()
    s[:, :, 0] = 1.0                                   # only the coarsest band of a full-depth analysis:
    np.testing.assert_allclose(oracle.wrm_apply(V, s, J), V + V.mean(axis=1, keepdims=True), atol=1e-13)
    s = zero.copy()
    s[:, :, 1] = 1.0                                   # only the finest details: half differences of pairs
    pair = V.reshape(B, L // 2, 2, H, d)
    det = (pair - pair.mean(axis=2, keepdims=True)).reshape(B, L, H, d)
    np.testing.assert_allclose(oracle.wrm_apply(V, s, J), V + det, atol=1e-13)
    # a gate acts on its own channel and head only
    s = zero.copy()
    s[1, 0, 3, 2] = 0.7
    out = oracle.wrm_apply(V, s, J)
    changed = np.abs(out - V).max(axis=1) > 0
    want = np.zeros((B, H, d), bool)
    want[1, 0, 2] = True
    assert np.array_equal(changed, want)


def band_of(i, n, J):
    """Band (0 = approximation, l = details of level l) of coefficient i in the order [a_J | d_J | ... | d_1]."""
    if i < n >> J:
        return 0
    l = J
    while i >= n >> (l - 1):
        l -= 1
    return l


@pytest.mark.parametrize("B,L,H,d,J", [(2, 64, 3, 4, 6), (1, 196, 2, 8, 2), (1, 96, 2, 6, 3), (1, 50, 1, 2, 1), (1, 9, 2, 2, 0),
                                       (1, 1024, 1, 16, 10)])
def test_per_coefficient_gates_equal_the_explicit_basis_form(oracle, B, L, H, d, J):
    """One gate per coefficient and channel (the printed shape, s in R^(n x d)): out = v + W^T diag(s) W v with the
    basis matrix W written from the definition of the Haar functions - no step shared with the oracle's
    analyse / multiply / synthesise."""
    rng = np.random.default_rng(3 * L + J)
    V = rng.standard_normal((B, L, H, d))
    s = rng.standard_normal((B, H, L, d))
    W = haar_matrix(L, J)
    want = np.empty_like(V)
    for b in range(B):
        for h in range(H):
            for c in range(d):
                want[b, :, h, c] = V[b, :, h, c] + W.T @ (s[b, h, :, c] * (W @ V[b, :, h, c]))
    np.testing.assert_allclose(oracle.wrm_apply_coeff(V, s, J), want, atol=1e-12)


def test_per_coefficient_gates_reduce_to_the_band_form(oracle):
    """Gates that are constant over each band are the band form: same output as wrm_apply, to rounding."""
    rng = np.random.default_rng(8)
    B, L, H, d, J = 2, 192, 2, 4, 5
    V = rng.standard_normal((B, L, H, d))
    sb = rng.standard_normal((B, H, J + 1, d))
    band = np.array([band_of(i, L, J) for i in range(L)])
    s = sb[:, :, band, :]                               # [B,H,L,d]
    np.testing.assert_allclose(oracle.wrm_apply_coeff(V, s, J), oracle.wrm_apply(V, sb, J), atol=1e-13)


def test_per_coefficient_gates_hand_computed_and_local(oracle):
    """n = 4, J = 2, x = (1, 2, 3, 4): coefficients (5, -2, -r, -r), r = sqrt(1/2).  A unit gate on one coefficient
    adds that coefficient times its basis function: the approximation adds the mean 2.5 everywhere, the level-2
    detail adds (-1, -1, +1, +1), the first level-1 detail adds (-1/2, +1/2, 0, 0).  A single gate touches only the
    rows its basis function covers, and only its own head and channel."""
    x = np.array([1.0, 2.0, 3.0, 4.0]).reshape(1, 4, 1, 1)
    adds = {0: [2.5, 2.5, 2.5, 2.5], 1: [-1.0, -1.0, 1.0, 1.0], 2: [-0.5, 0.5, 0.0, 0.0], 3: [0.0, 0.0, -0.5, 0.5]}
    for i, add in adds.items():
        s = np.zeros((1, 1, 4, 1))
        s[0, 0, i, 0] = 1.0
        np.testing.assert_allclose(oracle.wrm_apply_coeff(x, s, 2)[0, :, 0, 0], x[0, :, 0, 0] + np.array(add), atol=1e-14)
    rng = np.random.default_rng(9)
    B, L, H, d, J = 2, 64, 2, 3, 4
    V = rng.standard_normal((B, L, H, d))
    s = np.zeros((B, H, L, d))
    i = (L >> 3) + 5                                    # detail of level 3, block 5: rows 40..47
    assert band_of(i, L, J) == 3
    s[1, 0, i, 2] = -0.75
    out = oracle.wrm_apply_coeff(V, s, J)
    changed = np.abs(out - V) > 0
    want = np.zeros_like(changed)
    want[1, 40:48, 0, 2] = True
    assert np.array_equal(changed, want)
    blk = V[1, 40:48, 0, 2]
    coef = (blk[:4].sum() - blk[4:].sum()) / np.sqrt(8.0)
    np.testing.assert_allclose(out[1, 40:48, 0, 2] - blk, -0.75 * coef * np.array([1, 1, 1, 1, -1, -1, -1, -1]) / np.sqrt(8.0),
                               atol=1e-14)
    np.testing.assert_allclose(oracle.wrm_apply_coeff(V, np.zeros((B, H, L, d)), J), V, atol=0)
    np.testing.assert_allclose(oracle.wrm_apply_coeff(V, np.ones((B, H, L, d)), J), 2.0 * V, atol=1e-13)


def test_module_is_linear_in_v(oracle):
    rng = np.random.default_rng(6)
    B, L, H, d, J = 1, 96, 2, 4, 5
    V1, V2 = rng.standard_normal((2, B, L, H, d))
    s = rng.standard_normal((B, H, J + 1, d))
    a = oracle.wrm_apply(2.0 * V1 - 3.0 * V2, s, J)
    b = 2.0 * oracle.wrm_apply(V1, s, J) - 3.0 * oracle.wrm_apply(V2, s, J)
    np.testing.assert_allclose(a, b, atol=1e-12)


@pytest.mark.parametrize("shared", [False, True])
def test_level_gates_against_library_pieces(oracle, shared):
    from scipy.special import erf
    B, H, d, dw, J = 2, 3, 8, 5, 4
    Hg = 1 if shared else H
    p = synth.wrm_params(11, Hg, d, J, d_w=dw)
    rng = np.random.default_rng(12)
    sum_q = rng.standard_normal((B, H, d)) * 30
    inv = 1.0 / 37
    got = oracle.wrm_gates(sum_q, inv, p, J)
    x = sum_q * inv
    hsel = [0] * H if shared else list(range(H))
    for b in range(B):
        for h in range(H):
            hp = hsel[h]
            xc = x[b, h] - x[b, h].mean()
            qbar = p["ln_gamma"][hp].astype(np.float64) * xc / np.sqrt((xc * xc).mean() + p["ln_eps"]) + p["ln_beta"][hp]
            a = qbar @ p["W1"][hp].astype(np.float64) + p["b1"][hp]
            hid = 0.5 * a * (1 + erf(a / np.sqrt(2)))
            want = (hid @ p["W2"][hp].astype(np.float64) + p["b2"][hp]).reshape(J + 1, d)
            np.testing.assert_allclose(got[b, h], want, rtol=1e-12, atol=1e-14)


def test_level_gates_hand_computable(oracle):
    """One-hot weights route a known hidden unit to a known (band, channel)."""
    B, H, d, dw, J = 1, 1, 4, 3, 2
    nout = (J + 1) * d
    p = dict(ln_gamma=np.ones((1, d)), ln_beta=np.zeros((1, d)), ln_eps=0.0,
             W1=np.zeros((1, d, dw)), b1=np.zeros((1, dw)), W2=np.zeros((1, dw, nout)), b2=np.zeros((1, nout)))
    p["b1"][0, 1] = 10.0                      # GELU(10) = 10 to 1e-20: hidden unit 1 carries 10
    p["W2"][0, 1, 2 * d + 3] = 0.5            # -> band 2, channel 3
    p["b2"][0, 0 * d + 1] = -1.25             # bias only: band 0, channel 1
    s = oracle.wrm_gates(np.array([[[1.0, 2.0, 3.0, 4.0]]]), 1.0, p, J)
    want = np.zeros((J + 1, d))
    want[2, 3] = 5.0
    want[0, 1] = -1.25
    np.testing.assert_allclose(s[0, 0], want, atol=1e-12)
