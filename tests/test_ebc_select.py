"""The exact budgeted selection (heart_ebc_select, host code of libheart) against the oracle's
enumeration of Eq. 5 on small random instances, and against properties on larger ones.  Runs
without a GPU."""
import numpy as np
import pytest

import paper_2605_14513_amd as heart
from oracle import ebc_oracle as eo


def random_tables(rng, n, k, monotone):
    S = np.sort(rng.uniform(0.0, 1.0, size=(n, k)), axis=1)
    if monotone:  # more sparsity costs more error, convex-ish with noise (the realistic shape)
        E = np.cumsum(rng.uniform(0.0, 1.0, size=(n, k)) * np.linspace(0.2, 2.0, k), axis=1) * rng.uniform(0.1, 3.0, size=(n, 1))
    else:
        E = rng.uniform(0.0, 1.0, size=(n, k))
    return E, S


@pytest.mark.parametrize("seed", range(32))
def test_matches_enumeration_on_small_instances(seed):
    rng = np.random.default_rng(seed)
    n, k = int(rng.integers(1, 6)), int(rng.integers(1, 5))
    E, S = random_tables(rng, n, k, monotone=bool(seed % 2))
    for s_min in (0.0, float(rng.uniform(0.1, 0.9)), float(S.max(1).mean()), float(S.max(1).mean()) + 1e-3):
        want_c, want_e = eo.select_bruteforce(E, S, s_min)
        if want_c is None:
            with pytest.raises(heart.HeartError):
                heart.heart_ebc_select(E, S, s_min)
            continue
        c, e = heart.heart_ebc_select(E, S, s_min)
        assert S[np.arange(n), c].mean() >= s_min - 1e-12
        assert np.isclose(e, E[np.arange(n), c].sum(), rtol=0, atol=1e-12)
        assert np.isclose(e, want_e, rtol=1e-12, atol=1e-12), (seed, s_min, c, want_c)


@pytest.mark.parametrize("seed", range(6))
def test_matches_dynamic_programme_on_integer_sparsities(seed):
    rng = np.random.default_rng(100 + seed)
    n, k = 40, 5
    S_int = np.sort(rng.integers(0, 12, size=(n, k)), axis=1)
    E = rng.uniform(0.0, 1.0, size=(n, k)) * (1 + S_int)  # sparser tends to cost more, with ties in S
    for need in (0, int(S_int.max(1).sum() * 0.4), int(S_int.max(1).sum() * 0.8), int(S_int.max(1).sum())):
        want = eo.select_dp_integer(E, S_int, need)
        c, e = heart.heart_ebc_select(E, S_int.astype(np.float64), need / n)
        assert S_int[np.arange(n), c].sum() >= need
        assert np.isclose(e, want, rtol=1e-12, atol=1e-12), (seed, need)


def test_dynamic_programme_agrees_with_enumeration():
    rng = np.random.default_rng(7)
    S_int = rng.integers(0, 5, size=(5, 3))
    E = rng.uniform(size=(5, 3))
    for need in range(0, 21, 3):
        _, want = eo.select_bruteforce(E, S_int.astype(float), need / 5)
        assert np.isclose(eo.select_dp_integer(E, S_int, need), want) or (want == np.inf and eo.select_dp_integer(E, S_int, need) == np.inf)


def test_large_instance_is_feasible_and_not_beaten_by_local_moves():
    rng = np.random.default_rng(123)
    n, k = 1600, 8  # 40 layers x 40 heads, 8 candidate thresholds
    E, S = random_tables(rng, n, k, monotone=True)
    s_min = 0.6
    c, e = heart.heart_ebc_select(E, S, s_min)
    idx = np.arange(n)
    tot_s = S[idx, c].sum()
    assert tot_s >= s_min * n - 1e-9 and np.isclose(e, E[idx, c].sum())
    # no single-head change and no pair exchange (sampled) improves the objective while staying feasible
    for i in range(n):
        for cc in range(k):
            if E[i, cc] < E[i, c[i]] - 1e-12:
                assert tot_s - S[i, c[i]] + S[i, cc] < s_min * n - 1e-9
    for _ in range(20000):
        i, j = rng.integers(0, n, size=2)
        ci, cj = rng.integers(0, k, size=2)
        if i == j:
            continue
        de = E[i, ci] + E[j, cj] - E[i, c[i]] - E[j, c[j]]
        ds = S[i, ci] + S[j, cj] - S[i, c[i]] - S[j, c[j]]
        assert not (de < -1e-12 and tot_s + ds >= s_min * n - 1e-9)
    # a shared candidate index (the same threshold for every head) that meets the budget is never better
    for cc in range(k):
        if S[:, cc].mean() >= s_min:
            assert e <= E[:, cc].sum() + 1e-9


def test_bad_tables_are_rejected():
    with pytest.raises(heart.HeartError):
        heart.heart_ebc_select(np.array([[0.0, np.nan]]), np.array([[0.1, 0.2]]), 0.1)
    with pytest.raises(ValueError):
        heart.heart_ebc_select(np.zeros((2, 3)), np.zeros((3, 2)), 0.1)
