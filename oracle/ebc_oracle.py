"""CPU oracle for Error-guided Budgeted Calibration -- TEST INFRASTRUCTURE ONLY.

Plain numpy, fp64.  Two definitions, written out as the paper states them:

  band_error   the frequency-weighted velocity error of Eq. 6: 3D discrete Fourier
               transform of the sparse-induced error over (time, height, width), the
               frequency grid split into four bands by the rule of the appendix on the
               frequency-aware velocity error (after fftshift, a frequency is "low" along
               an axis of length n when it lies within floor(n/4) of the zero-frequency
               centre; LL = low temporal and low on both spatial axes, LH = low temporal
               and high on at least one spatial axis, HL = high temporal and low on both
               spatial axes, HH = the rest), band energies weighted by
               (1.0, 0.5, 0.01, 0.01) and normalised by the spectral energy of the dense
               reference plus 1e-10.
  select_bruteforce   the one-candidate-per-head selection of Eq. 5 by enumeration:
               minimise the summed error subject to mean sparsity >= S_min.

Readings: the transform runs over the last three axes and energies are summed over every
leading axis (channels, batch); numpy's unnormalised forward transform is used for both
numerator and denominator, so the normalisation cancels.
"""
from __future__ import annotations

import itertools

import numpy as np

BAND_WEIGHTS = (1.0, 0.5, 0.01, 0.01)  # LL, LH, HL, HH
EPSILON = 1e-10


def low_mask(n: int) -> np.ndarray:
    """Boolean [n] over fftshift-ed frequency positions: within floor(n/4) of the centre."""
    centre = n // 2  # position of the zero frequency after fftshift
    return np.abs(np.arange(n) - centre) <= n // 4


def band_energies(x: np.ndarray) -> np.ndarray:
    """Spectral energy of x (last three axes = time, height, width) in LL, LH, HL, HH."""
    x = np.asarray(x, dtype=np.float64)
    spec = np.fft.fftshift(np.fft.fftn(x, axes=(-3, -2, -1)), axes=(-3, -2, -1))
    energy = (spec.real ** 2 + spec.imag ** 2).reshape((-1,) + x.shape[-3:]).sum(0)
    lt = low_mask(x.shape[-3])[:, None, None]
    ls = low_mask(x.shape[-2])[None, :, None] & low_mask(x.shape[-1])[None, None, :]
    return np.array([energy[lt & ls].sum(), energy[lt & ~ls].sum(),
                     energy[~lt & ls].sum(), energy[~lt & ~ls].sum()])


def band_error(err: np.ndarray, dense: np.ndarray, weights=BAND_WEIGHTS, epsilon=EPSILON) -> float:
    """Eq. 6: sum_q w_q * (energy of err in band q) / (total spectral energy of dense + eps)."""
    num = band_energies(err)
    dense = np.asarray(dense, dtype=np.float64)
    spec = np.fft.fftn(dense, axes=(-3, -2, -1))
    den = float((spec.real ** 2 + spec.imag ** 2).sum()) + epsilon
    return float(np.dot(np.asarray(weights, dtype=np.float64), num) / den)


def select_bruteforce(E: np.ndarray, S: np.ndarray, s_min: float):
    """Eq. 5 by enumeration.  E, S: [n_heads, n_candidates].  Returns (choice [n_heads] or None
    if infeasible, total error).  Ties: the lexicographically smallest choice."""
    E = np.asarray(E, dtype=np.float64)
    S = np.asarray(S, dtype=np.float64)
    n, k = E.shape
    best, best_e = None, np.inf
    for choice in itertools.product(range(k), repeat=n):
        s = sum(S[i, c] for i, c in enumerate(choice)) / n
        if s + 1e-15 < s_min:
            continue
        e = sum(E[i, c] for i, c in enumerate(choice))
        if e < best_e:
            best, best_e = choice, e
    return (None, np.inf) if best is None else (np.array(best), float(best_e))


def select_dp_integer(E: np.ndarray, S_int: np.ndarray, need_total: int) -> float:
    """Eq. 5 for INTEGER sparsity scores by dynamic programming over the total (exact, for
    mid-size checks): minimum summed error with sum of S_int >= need_total; inf if infeasible."""
    E = np.asarray(E, dtype=np.float64)
    S_int = np.asarray(S_int, dtype=np.int64)
    n, k = E.shape
    cap = int(need_total)
    best = np.full(cap + 1, np.inf)  # best[t] = least error with total sparsity min(total, cap) == t
    best[0] = 0.0
    for i in range(n):
        new = np.full(cap + 1, np.inf)
        for c in range(k):
            for t in range(cap + 1):
                if best[t] == np.inf:
                    continue
                t2 = min(cap, t + int(S_int[i, c]))
                v = best[t] + E[i, c]
                if v < new[t2]:
                    new[t2] = v
        best = new
    return float(best[cap])
