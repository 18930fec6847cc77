"""Pins of the calibration oracle (oracle/ebc_oracle.py) to what the paper and the mathematics
fix: Parseval's identity, where single frequencies fall, the band rule of the appendix, and
the selection problem of Eq. 5 against hand-solvable instances."""
import numpy as np
import pytest

from oracle import ebc_oracle as eo


def test_low_rule_counts_and_centre():
    # within floor(n/4) of the fftshift centre: 2*floor(n/4)+1 positions, symmetric in frequency
    for n in (4, 5, 8, 21, 30, 52):
        m = eo.low_mask(n)
        assert m.sum() == 2 * (n // 4) + 1
        freqs = np.fft.fftshift(np.fft.fftfreq(n, 1.0 / n)).round().astype(int)
        assert set(freqs[m]) == set(range(-(n // 4), n // 4 + 1))


def test_parseval_total_energy():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 6, 8, 10))
    # unnormalised DFT: sum |X|^2 = (T*Y*X) * sum |x|^2; the four bands partition the grid
    assert np.isclose(eo.band_energies(x).sum(), 6 * 8 * 10 * (x ** 2).sum(), rtol=1e-12)


@pytest.mark.parametrize("ft,fy,fx,band", [(0, 0, 0, 0), (1, 2, 3, 0), (0, 0, 4, 1), (1, 3, 0, 1),
                                            (3, 0, 0, 2), (4, 2, 3, 2), (3, 3, 0, 3), (4, 0, 6, 3)])
def test_single_frequency_lands_in_its_band(ft, fy, fx, band):
    T, Y, X = 8, 8, 12  # low: |f| <= 2, 2, 3
    t, y, x = np.meshgrid(np.arange(T), np.arange(Y), np.arange(X), indexing="ij")
    wave = np.cos(2 * np.pi * (ft * t / T + fy * y / Y + fx * x / X))
    e = eo.band_energies(wave)
    assert np.isclose(e[band], e.sum(), rtol=1e-12) and e.sum() > 0


def test_shift_invariance_and_channel_additivity():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 5, 6, 7))
    assert np.allclose(eo.band_energies(np.roll(x, (2, 1, 3), axis=(-3, -2, -1))), eo.band_energies(x))
    assert np.allclose(eo.band_energies(x), eo.band_energies(x[0]) + eo.band_energies(x[1]))


def test_band_error_weights_and_normalisation():
    T, Y, X = 8, 8, 8
    t, y, x = np.meshgrid(np.arange(T), np.arange(Y), np.arange(X), indexing="ij")
    dense = np.cos(2 * np.pi * x / X) * 3.0
    ll = np.cos(2 * np.pi * (t / T + y / Y))          # LL
    hh = np.cos(2 * np.pi * (4 * t / T + 4 * x / X))  # HH
    n = T * Y * X
    den = n * (dense ** 2).sum() + 1e-10
    assert np.isclose(eo.band_error(ll, dense), 1.0 * n * (ll ** 2).sum() / den, rtol=1e-12)
    assert np.isclose(eo.band_error(hh, dense), 0.01 * n * (hh ** 2).sum() / den, rtol=1e-12)
    # additive over bands for orthogonal components; quadratic in the error's scale
    assert np.isclose(eo.band_error(ll + hh, dense), eo.band_error(ll, dense) + eo.band_error(hh, dense))
    assert np.isclose(eo.band_error(2 * ll, dense), 4 * eo.band_error(ll, dense))
    # zero reference: only epsilon in the denominator
    assert np.isclose(eo.band_error(ll, np.zeros_like(ll)), n * (ll ** 2).sum() / 1e-10)


def test_selection_hand_instances():
    # two heads, candidates (error, sparsity): the budget forces one head to its sparser choice,
    # and the cheaper one is taken
    E = np.array([[0.0, 1.0], [0.0, 3.0]])
    S = np.array([[0.2, 0.8], [0.2, 0.8]])
    c, e = eo.select_bruteforce(E, S, 0.5)
    assert list(c) == [1, 0] and e == 1.0
    c, e = eo.select_bruteforce(E, S, 0.8)
    assert list(c) == [1, 1] and e == 4.0
    c, e = eo.select_bruteforce(E, S, 0.1)
    assert list(c) == [0, 0] and e == 0.0
    c, e = eo.select_bruteforce(E, S, 0.81)
    assert c is None and e == np.inf
    # the budget is on the MEAN sparsity over heads
    E = np.array([[0.0, 5.0, 9.0]] * 3)
    S = np.array([[0.0, 0.5, 1.0]] * 3)
    c, e = eo.select_bruteforce(E, S, 0.5)
    assert e == 14.0 and sorted(c) == [0, 1, 2]  # 0+5+9 beats 5+5+5
