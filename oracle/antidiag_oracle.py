"""CPU oracle of the antidiagonal-style block-importance estimator -- TEST INFRASTRUCTURE ONLY.

The paper delegates block-importance ranking to the sparse-attention backbone it is attached
to and only names the backbone's setting (baseline configurations in the appendix: antidiagonal
scoring with stride 16 on blocks of 128 tokens, threshold 0.9).  It does not define the
estimator, so there is no value of the paper's to pin it to: PARITY UNPINNED with respect to
the paper.  What is implemented is this definition, which the tests pin to brute force over the
dense logit matrix and to the exact block attention mass in the special case stride = 1:

  S = stride, kb = block / S.  Tokens past N count as zero vectors.  For reduced query a and
  reduced key b (a, b in [0, ceil(N/S))), the strided antidiagonal sum of the S x S tile (a, b) of
  Q K^T:
      L[a, b] = 1 / (S sqrt(D)) * sum_{r=0}^{S-1}  q[S a + (S-1-r)] . k[S b + r]
  P[a, :] = softmax_b L[a, :]                     (over all reduced keys)
  score[I, J] = mean over the reduced queries a of block I of  sum_{b in block J} P[a, b]

Every row of `score` sums to one, so it can be ranked by the same top-p rule as the pooled
scores.  Plain numpy in fp64; one head at a time.
"""
from __future__ import annotations

import numpy as np

__all__ = ["reduced_logits", "antidiag_scores"]


def _pad_rows(x: np.ndarray, rows: int) -> np.ndarray:
    out = np.zeros((rows, x.shape[1]), dtype=np.float64)
    out[: x.shape[0]] = x
    return out


def reduced_logits(q: np.ndarray, k: np.ndarray, stride: int) -> np.ndarray:
    """L[a, b] of the definition above for one head; q, k: [N, D]."""
    N, D = q.shape
    S = int(stride)
    M = (N + S - 1) // S
    qp = _pad_rows(np.asarray(q, dtype=np.float64), M * S).reshape(M, S, D)
    kp = _pad_rows(np.asarray(k, dtype=np.float64), M * S).reshape(M, S, D)
    # query sub-rows in reverse order against key sub-rows in order: r <-> S-1-r
    qr = qp[:, ::-1, :].reshape(M, S * D)
    kr = kp.reshape(M, S * D)
    return (qr @ kr.T) / (S * np.sqrt(float(D)))


def antidiag_scores(q: np.ndarray, k: np.ndarray, block: int, stride: int) -> np.ndarray:
    """score[I, J] of the definition above for one head; q, k: [N, D]; returns [Nb, Nb]."""
    N = q.shape[0]
    S = int(stride)
    if block % S != 0:
        raise ValueError("stride must divide the block size")
    kb = block // S
    L = reduced_logits(q, k, S)
    M = L.shape[0]
    L = L - L.max(axis=1, keepdims=True)
    P = np.exp(L)
    P /= P.sum(axis=1, keepdims=True)
    Nb = (N + block - 1) // block
    out = np.zeros((Nb, Nb), dtype=np.float64)
    for I in range(Nb):
        a0, a1 = I * kb, min((I + 1) * kb, M)
        for J in range(Nb):
            b0, b1 = J * kb, min((J + 1) * kb, M)
            out[I, J] = P[a0:a1, b0:b1].sum() / (a1 - a0)
    return out
