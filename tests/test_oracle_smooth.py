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


def test_energy_cutoff_is_the_loop_definition_and_dc_variant():
    # Eqs. 14-16 written out as loops on random spectra, with and without the DC bin
    rng = np.random.default_rng(7)
    for trial in range(20):
        nb = int(rng.integers(2, 40))
        F = rng.normal(size=nb) + 1j * rng.normal(size=nb)
        rho = float(rng.uniform(0.05, 1.0))
        for skip in (False, True):
            first = 1 if skip else 0
            total = sum(abs(F[i]) ** 2 for i in range(first, nb))
            acc, want = 0.0, None
            for k in range(first, nb):
                acc += abs(F[k]) ** 2
                if acc >= rho * total:
                    want = k
                    break
            assert O.energy_cutoff_bin(F, rho, skip) == want
    # known spectrum without DC: |F_3|^2 = L^2, |F_10|^2 = L^2/4 -> cumulative 1, 1.25 (x L^2)
    L = 64
    n = np.arange(L)
    s = 1.0 + 2.0 * np.cos(2 * np.pi * 3 * n / L) + 1.0 * np.cos(2 * np.pi * 10 * n / L)
    F = O.rdft(s)
    assert O.energy_cutoff_bin(F, 0.5, True) == 3
    assert O.energy_cutoff_bin(F, 0.9, True) == 10
    # monotone in rho
    ks = [O.energy_cutoff_bin(F, r) for r in (0.1, 0.3, 0.5, 0.7, 0.9, 0.99, 1.0)]
    assert ks == sorted(ks)


def test_taper_mask_shape():
    # T = 0 is the hard mask of Eq. 17
    w0 = O.mask_weights(5, 0, 20)
    assert np.array_equal(w0, (np.arange(20) <= 5).astype(float))
    for ks, T, nb in [(5, 4, 20), (0, 7, 9), (10, 3, 12), (3, 1, 8)]:
        w = O.mask_weights(ks, T, nb)
        assert np.all(w[:ks + 1] == 1.0) and np.all(w[ks + T + 1:] == 0.0)
        band = w[ks + 1:min(ks + T + 1, nb)]
        assert np.all(band > 0.0) and np.all(band < 1.0) and np.all(np.diff(np.concatenate([[1.0], band, [0.0]])) < 0)
        # half-cosine: values mirrored about the middle of the band add up to one
        if ks + T < nb:
            full = w[ks + 1:ks + T + 1]
            np.testing.assert_allclose(full + full[::-1], 1.0, atol=1e-15)
            # closed form at the middle of an odd band: exactly one half
            if T % 2 == 1:
                assert abs(full[T // 2] - 0.5) < 1e-15


def test_taper_scales_single_cosines_and_keeps_invariants():
    L, ks_frac, T = 256, 0.125, 6            # k* = 16, band 17..22
    n = np.arange(L)
    ks = O.cutoff_bin(L, ks_frac)
    w = O.mask_weights(ks, T, L // 2 + 1)
    for k in (3, 16, 17, 19, 22, 23, 60):
        s = np.cos(2 * np.pi * k * n / L + 0.3)
        out = O.smooth(s, ks_frac, 1.0, taper_bins=T)
        np.testing.assert_allclose(out, w[k] * s, atol=1e-12)
    rng = np.random.default_rng(11)
    a, b = rng.normal(size=L), rng.normal(size=L)
    fa, fb = O.smooth(a, ks_frac, 1.0, taper_bins=T), O.smooth(b, ks_frac, 1.0, taper_bins=T)
    np.testing.assert_allclose(O.smooth(2 * a - 3 * b, ks_frac, 1.0, taper_bins=T), 2 * fa - 3 * fb, atol=1e-12)
    assert abs(fa.mean() - a.mean()) < 1e-13
    # a tapered mask removes less than the hard mask at k* and no more than the hard mask at k* + T
    e = lambda x: float(np.sum(x * x))
    assert e(O.smooth(a, ks_frac, 1.0)) <= e(fa) + 1e-12 <= e(O.smooth(a, 0, 1.0, k_star=ks + T)) + 2e-12
    # against the library transform with the same weights
    ref = np.fft.irfft(np.fft.rfft(a) * w, L)
    np.testing.assert_allclose(fa, ref, atol=1e-12)
    # band running past the Nyquist bin is simply cut there
    out = O.smooth(a, 1.0, 1.0, taper_bins=5)
    np.testing.assert_allclose(out, a, atol=1e-12)
    # forced cutoff = the same cutoff reached by its fraction
    np.testing.assert_array_equal(O.smooth(a, 0, 0.5, k_star=ks), O.smooth(a, ks_frac, 0.5))
