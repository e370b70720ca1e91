"""Pins for the oracle's stage 3, Spectral Score Smoothing (Sec. 3.3, Eqs. 13-20).

The oracle's DFTs are direct sums; they are pinned here by a loop-level O(L^2)
DFT written from the textbook definition, by numpy's FFT (a library
cross-check, not used by the oracle), and by the properties an ideal low-pass
projection must have."""
import cmath
import math

import numpy as np
import pytest

from oracle import audiokv_oracle as O


def _dft_loops(s):
    L = len(s)
    return [sum(s[n] * cmath.exp(-2j * math.pi * k * n / L) for n in range(L)) for k in range(L)]


def _sss_loops(s, ks, alpha):
    """Full complex DFT, zero every frequency whose |frequency index| > ks, inverse, mix."""
    L = len(s)
    F = _dft_loops(s)
    for k in range(L):
        fidx = min(k, L - k)                 # bin index of the two-sided frequency
        if fidx > ks:
            F[k] = 0.0
    out = []
    for n in range(L):
        v = sum(F[k] * cmath.exp(2j * math.pi * k * n / L) for k in range(L)) / L
        assert abs(v.imag) < 1e-9
        out.append((1 - alpha) * s[n] + alpha * v.real)
    return np.array(out)


@pytest.mark.parametrize("L", [8, 9, 15, 16, 33])
def test_rdft_matches_loop_dft(L):
    s = np.random.default_rng(L).standard_normal(L)
    F = O.rdft(s)
    assert F.shape[0] == L // 2 + 1                         # Eq. 13: L/2 + 1 bins
    ref = _dft_loops(list(s))
    np.testing.assert_allclose(F, ref[:L // 2 + 1], rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("L", [8, 9, 15, 16, 33])
@pytest.mark.parametrize("c,alpha", [(0.25, 1.0), (0.5, 0.6), (1.0, 1.0), (0.0, 1.0)])
def test_smooth_matches_loop_definition(L, c, alpha):
    s = np.random.default_rng(L + 100).standard_normal(L)
    ks = O.cutoff_bin(L, c)
    assert ks == int(math.floor(c * (L // 2)))
    got = O.smooth(s, c, alpha)
    ref = _sss_loops(list(s), ks, alpha)
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("L", [64, 100, 257, 1000, 2048])
def test_library_cross_check(L):
    s = np.random.default_rng(L).standard_normal(L) + 0.3
    for c in (1.0 / 8, 1.0 / 4, 0.7):
        ks = O.cutoff_bin(L, c)
        F = np.fft.rfft(s)
        F[ks + 1:] = 0.0
        ref = np.fft.irfft(F, L)
        np.testing.assert_allclose(O.smooth(s, c, 1.0), ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("L", [16, 31, 256, 1001])
def test_cutoff_at_nyquist_is_identity(L):
    s = np.random.default_rng(L + 1).standard_normal(L)
    np.testing.assert_allclose(O.smooth(s, 1.0, 1.0), s, rtol=0, atol=1e-12 * np.abs(s).max())


@pytest.mark.parametrize("L", [16, 31, 300])
def test_constant_signal_unchanged(L):
    for c in (0.0, 0.125, 0.5):
        np.testing.assert_allclose(O.smooth(np.full(L, 2.5), c, 1.0), 2.5, rtol=1e-13)


def test_single_cosine_passes_iff_below_cutoff():
    L = 128
    n = np.arange(L)
    ks = O.cutoff_bin(L, 0.25)        # 16
    assert ks == 16
    for kbin in (1, 5, 16):
        s = np.cos(2 * np.pi * kbin * n / L + 0.4)
        np.testing.assert_allclose(O.smooth(s, 0.25, 1.0), s, atol=1e-12)
    for kbin in (17, 40, 64):
        s = np.cos(2 * np.pi * kbin * n / L + 0.4)
        np.testing.assert_allclose(O.smooth(s, 0.25, 1.0), 0.0, atol=1e-12)


def test_mean_preserved_idempotent_linear_energy():
    rng = np.random.default_rng(21)
    L = 513
    x, y = rng.standard_normal(L), rng.standard_normal(L)
    sx = O.smooth(x, 0.125, 1.0)
    assert abs(sx.mean() - x.mean()) < 1e-13                           # DC bin always kept
    np.testing.assert_allclose(O.smooth(sx, 0.125, 1.0), sx, atol=1e-12)  # projection
    lin = O.smooth(2.0 * x - 3.0 * y, 0.125, 1.0)
    np.testing.assert_allclose(lin, 2.0 * sx - 3.0 * O.smooth(y, 0.125, 1.0), atol=1e-12)
    assert (sx ** 2).sum() <= (x ** 2).sum() + 1e-12                    # Parseval


def test_alpha_zero_is_bitwise_identity_and_alpha_is_linear():
    s = np.random.default_rng(22).standard_normal(200)
    assert np.array_equal(O.smooth(s, 0.125, 0.0), s)
    a0, a1, ah = O.smooth(s, 0.125, 0.0), O.smooth(s, 0.125, 1.0), O.smooth(s, 0.125, 0.5)
    np.testing.assert_allclose(ah, 0.5 * (a0 + a1), atol=1e-13)


def test_irdft_inverts_rdft_even_and_odd():
    for L in (10, 11, 64, 127):
        s = np.random.default_rng(L).standard_normal(L)
        np.testing.assert_allclose(O.irdft(O.rdft(s), L), s, atol=1e-12)


def test_large_L_twiddles_stay_accurate():
    L = 32768
    n = np.arange(L)
    s = np.cos(2 * np.pi * 2047 * n / L) + np.cos(2 * np.pi * 2049 * n / L)
    out = O.smooth(s, 0.125, 1.0)     # k* = 2048: first passes, second is removed
    np.testing.assert_allclose(out, np.cos(2 * np.pi * 2047 * n / L), atol=1e-9)


def test_energy_cutoff_known_spectrum():
    # DC of amplitude a plus cosines: one-sided energies are known in closed form
    L = 64
    n = np.arange(L)
    s = 1.0 + 2.0 * np.cos(2 * np.pi * 3 * n / L) + 1.0 * np.cos(2 * np.pi * 10 * n / L)
    F = O.rdft(s)
    # |F_0|^2 = L^2, |F_3|^2 = (2*L/2)^2 = L^2, |F_10|^2 = (L/2)^2 -> cumulative 1, 2, 2.25 (x L^2)
    assert O.energy_cutoff_bin(F, 0.40) == 0
    assert O.energy_cutoff_bin(F, 0.50) == 3
    assert O.energy_cutoff_bin(F, 0.88) == 3
    assert O.energy_cutoff_bin(F, 0.95) == 10
    out = O.smooth(s, 0.0, 1.0, energy_rho=0.6)
    np.testing.assert_allclose(out, 1.0 + 2.0 * np.cos(2 * np.pi * 3 * n / L), atol=1e-12)
