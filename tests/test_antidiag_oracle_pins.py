"""Pins of the antidiagonal-style estimator's oracle (CPU only).

The paper names the estimator's setting (antidiagonal scoring stride 16, blocks of 128 tokens,
appendix on baseline configurations) but does not define it, so nothing here is a value of the
paper's.  The pins are: brute force over the dense logit matrix written with explicit token
indices, the exact block attention mass at stride 1, invariants, and planted mistakes that
these pins must catch.
"""
import numpy as np
import pytest
from scipy.special import softmax

from oracle import antidiag_oracle as ao


def _qk(N, D, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((N, D)), rng.standard_normal((N, D))


def _brute_logits(q, k, S):
    """Antidiagonal of every S x S tile of the zero-padded dense Q K^T, token by token."""
    N, D = q.shape
    M = (N + S - 1) // S
    A = np.zeros((M * S, M * S))
    A[:N, :N] = q @ k.T
    L = np.zeros((M, M))
    for a in range(M):
        for b in range(M):
            s = 0.0
            for i in range(S):
                for j in range(S):
                    if i + j == S - 1:
                        s += A[a * S + i, b * S + j]
            L[a, b] = s / (S * np.sqrt(D))
    return L


@pytest.mark.parametrize("N,D,S", [(32, 8, 4), (37, 4, 4), (48, 16, 8), (21, 4, 2), (16, 4, 16)])
def test_reduced_logits_equal_tile_antidiagonals(N, D, S):
    q, k = _qk(N, D, N + S)
    np.testing.assert_allclose(ao.reduced_logits(q, k, S), _brute_logits(q, k, S), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("N,block,S", [(64, 16, 4), (70, 16, 4), (61, 8, 8), (40, 8, 2)])
def test_scores_equal_brute_force(N, block, S):
    q, k = _qk(N, 8, 3 * N + S)
    L = _brute_logits(q, k, S)
    P = softmax(L, axis=1)
    kb = block // S
    M = L.shape[0]
    Nb = (N + block - 1) // block
    ref = np.zeros((Nb, Nb))
    for I in range(Nb):
        rows = [a for a in range(M) if a // kb == I]
        for J in range(Nb):
            cols = [b for b in range(M) if b // kb == J]
            ref[I, J] = sum(P[a, b] for a in rows for b in cols) / len(rows)
    np.testing.assert_allclose(ao.antidiag_scores(q, k, block, S), ref, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("N,block", [(64, 16), (50, 16), (33, 8)])
def test_stride_one_is_exact_block_attention_mass(N, block):
    """With stride 1 every logit is on an antidiagonal: the score of (I, J) is the attention
    mass the queries of block I put on the keys of block J, averaged over the queries."""
    q, k = _qk(N, 8, 7 * N)
    P = softmax(q @ k.T / np.sqrt(8.0), axis=1)
    Nb = (N + block - 1) // block
    ref = np.zeros((Nb, Nb))
    for I in range(Nb):
        i0, i1 = I * block, min(N, (I + 1) * block)
        for J in range(Nb):
            j0, j1 = J * block, min(N, (J + 1) * block)
            ref[I, J] = P[i0:i1, j0:j1].sum() / (i1 - i0)
    np.testing.assert_allclose(ao.antidiag_scores(q, k, block, 1), ref, rtol=1e-12, atol=1e-14)


def test_rows_sum_to_one_and_are_nonnegative():
    q, k = _qk(203, 16, 5)
    s = ao.antidiag_scores(q, k, 32, 4)
    assert s.shape == (7, 7)
    assert (s >= 0).all()
    np.testing.assert_allclose(s.sum(axis=1), 1.0, rtol=1e-12)


def test_direction_of_the_diagonal_matters():
    """A logit matrix that is large exactly on the antidiagonals of its tiles: the
    antidiagonal sum sees it, the main-diagonal sum (the planted mistake: r against r) does not."""
    S, D, M = 4, 8, 6
    N = S * M
    # token S a + i of q carries feature e_{(S-1-i)}, token S b + j of k carries e_j, scaled by a
    # per-tile pattern: q.k is nonzero only where i + j == S - 1
    q = np.zeros((N, D)); k = np.zeros((N, D))
    for a in range(M):
        for i in range(S):
            q[a * S + i, S - 1 - i] = 1.0 + 0.1 * a
            k[a * S + i, i] = 2.0
    L = ao.reduced_logits(q, k, S)
    assert np.all(L > 0.5)
    # the mistaken pairing r <-> r gives q[S a + r] . k[S b + r] = 0 for S even except r == S-1-r (never)
    qp = q.reshape(M, S, D); kp = k.reshape(M, S, D)
    wrong = np.einsum("ard,brd->ab", qp, kp) / (S * np.sqrt(D))
    assert np.allclose(wrong, 0.0)


def test_not_symmetric_in_q_and_k():
    """Swapping the operands must change the result (a transposed contraction is caught)."""
    q, k = _qk(48, 8, 11)
    a = ao.antidiag_scores(q, k, 16, 4)
    b = ao.antidiag_scores(k, q, 16, 4)
    assert np.abs(a - b).max() > 1e-3
    # and the swap equals the transpose of the reduced logits, not the logits themselves
    np.testing.assert_allclose(ao.reduced_logits(k, q, 4), ao.reduced_logits(q, k, 4).T, rtol=1e-12, atol=1e-12)


def test_planted_block_wins():
    """Keys of one block aligned with the queries of another: that pair gets the top score."""
    N, D, block, S = 128, 16, 32, 8
    rng = np.random.default_rng(2)
    q = 0.05 * rng.standard_normal((N, D)); k = 0.05 * rng.standard_normal((N, D))
    v = rng.standard_normal(D); v /= np.linalg.norm(v)
    q[32:64] += 6.0 * v      # query block 1
    k[96:128] += 6.0 * v     # key block 3
    s = ao.antidiag_scores(q, k, block, S)
    assert s[1].argmax() == 3 and s[1, 3] > 0.9
    # other query blocks are indifferent
    assert s[0].max() < 0.5


def test_stride_must_divide_block():
    q, k = _qk(32, 4, 0)
    with pytest.raises(ValueError):
        ao.antidiag_scores(q, k, 16, 3)
