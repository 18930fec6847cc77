"""ctypes loader and numpy wrappers for the C oracle (test infrastructure only).

Each wrapper names the passage of the paper its C function follows; the C file
holds the arithmetic.  Inputs that are bf16 are passed as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "heart_oracle.c")
_SO = os.path.join(_HERE, "libheart_oracle.so")
_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  No fast-math, no FMA contraction."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = [
            "gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
            "-fno-fast-math", "-o", _SO, _SRC, "-lm",
        ]
        subprocess.run(cmd, check=True)
    return _SO


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_SO)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a: np.ndarray, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _strides3(x: np.ndarray) -> np.ndarray:
    """Element strides (b, h, n) of a [B,H,N,D] array whose D axis is contiguous."""
    assert x.ndim == 4 and x.strides[3] == x.itemsize
    return np.array([s // x.itemsize for s in x.strides[:3]], dtype=np.int64)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def pool(x_u16: np.ndarray, block: int) -> Tuple[np.ndarray, np.ndarray]:
    """Block means and token means of bf16 x [B,H,N,D] (Alg. 1 step 1; Eq. 4)."""
    lib = _load()
    assert x_u16.dtype == np.uint16
    B, H, N, D = x_u16.shape
    st = _strides3(x_u16)
    Nb = (N + block - 1) // block
    blk = np.empty((B, H, Nb, D), dtype=np.float32)
    mean = np.empty((B, H, D), dtype=np.float32)
    lib.oracle_pool(
        ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(N), ctypes.c_int(D), ctypes.c_int(block),
        _p(x_u16), ctypes.c_longlong(int(st[0])), ctypes.c_longlong(int(st[1])),
        ctypes.c_longlong(int(st[2])), _p(blk), _p(mean),
    )
    return blk, mean


def drift(qmean, kmean, qanchor, kanchor, has_anchor, delta, gate_lo=0.4, gate_hi=0.8,
          commit=True):
    """Mean-pooled drift, reuse rule, layer gate, anchor commit (Eq. 4; Alg. 1; Sec. 4.2).

    qanchor, kanchor, has_anchor are updated IN PLACE (must be contiguous arrays of
    float32 / float32 / uint8).  Returns (drift [B,H] f32, refresh [B,H] u8).
    """
    lib = _load()
    qmean = _c(qmean, np.float32)
    kmean = _c(kmean, np.float32)
    B, H, D = qmean.shape
    assert D & (D - 1) == 0, "D must be a power of two"
    for a, dt in ((qanchor, np.float32), (kanchor, np.float32), (has_anchor, np.uint8)):
        assert a.dtype == dt and a.flags["C_CONTIGUOUS"]
    delta = _c(delta, np.float32)
    assert delta.shape == (H,)
    d = np.empty((B, H), dtype=np.float32)
    r = np.empty((B, H), dtype=np.uint8)
    lib.oracle_drift(
        ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(D), _p(qmean), _p(kmean), _p(qanchor),
        _p(kanchor), _p(has_anchor), _p(delta), ctypes.c_float(gate_lo), ctypes.c_float(gate_hi),
        ctypes.c_int(1 if commit else 0), _p(d), _p(r),
    )
    return d, r


def scores(qblk, kblk) -> np.ndarray:
    """Block importance P = softmax_j(qblk_i . kblk_j / sqrt(D)), [B,H,Nb,Nb] f32."""
    lib = _load()
    qblk = _c(qblk, np.float32)
    kblk = _c(kblk, np.float32)
    B, H, Nb, D = qblk.shape
    out = np.empty((B, H, Nb, Nb), dtype=np.float32)
    lib.oracle_scores(ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(Nb), ctypes.c_int(D),
                      _p(qblk), _p(kblk), _p(out))
    return out


def topp(scores_, tau, refresh=None, n_always_kv=0, n_dense_q=0, min_keep=1,
         mask=None, kept_idx=None, kept_count=None):
    """Top-p block selection (Sec. 3.2; minimal set of Eq. 1).

    Returns (mask u8 [B,H,Nb,Nb], kept_idx i32 [B,H,Nb,Nb], kept_count i32 [B,H,Nb]).
    If mask/kept_idx/kept_count are given they are updated in place for refreshed
    heads only (cached masks of reused heads persist, Alg. 1).
    """
    lib = _load()
    scores_ = _c(scores_, np.float32)
    B, H, Nb, Nb2 = scores_.shape
    assert Nb == Nb2
    tau = _c(tau, np.float32)
    assert tau.shape == (H,)
    if refresh is not None:
        refresh = _c(refresh, np.uint8)
        assert refresh.shape == (B, H)
    if mask is None:
        mask = np.zeros((B, H, Nb, Nb), dtype=np.uint8)
        kept_idx = np.full((B, H, Nb, Nb), -1, dtype=np.int32)
        kept_count = np.zeros((B, H, Nb), dtype=np.int32)
    lib.oracle_topp(
        ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(Nb), _p(scores_), _p(tau), _p(refresh),
        ctypes.c_int(n_always_kv), ctypes.c_int(n_dense_q), ctypes.c_int(min_keep),
        _p(mask), _p(kept_idx), _p(kept_count),
    )
    return mask, kept_idx, kept_count


def attn(q_u16, k_u16, v_u16, block, kept_idx, kept_count, scale=0.0,
         qblocks: Optional[Sequence[int]] = None, want_lse=False):
    """Softmax attention over the tokens of kept key blocks; out f32 [B,H,N,D].

    With `qblocks` only those query blocks are computed; other rows are NaN.
    """
    lib = _load()
    B, H, N, D = q_u16.shape
    for a in (q_u16, k_u16, v_u16):
        assert a.dtype == np.uint16 and a.shape == (B, H, N, D)
    Nb = (N + block - 1) // block
    kept_idx = _c(kept_idx, np.int32)
    kept_count = _c(kept_count, np.int32)
    assert kept_idx.shape == (B, H, Nb, Nb) and kept_count.shape == (B, H, Nb)
    out = np.full((B, H, N, D), np.nan, dtype=np.float32)
    lse = np.full((B, H, N), np.nan, dtype=np.float32) if want_lse else None
    qs, ks, vs = _strides3(q_u16), _strides3(k_u16), _strides3(v_u16)
    qb = None if qblocks is None else np.ascontiguousarray(qblocks, dtype=np.int32)
    lib.oracle_attn(
        ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(N), ctypes.c_int(D), ctypes.c_int(block),
        _p(q_u16), _p(k_u16), _p(v_u16), _p(qs), _p(ks), _p(vs), _p(kept_idx), _p(kept_count),
        ctypes.c_float(scale), _p(qb), ctypes.c_int(0 if qb is None else len(qb)), _p(out),
        _p(lse),
    )
    return (out, lse) if want_lse else out


def dense_attn(q_u16, k_u16, v_u16, scale=0.0) -> np.ndarray:
    """Unblocked dense attention softmax(QK^T * scale) V, out f32 [B,H,N,D]."""
    lib = _load()
    B, H, N, D = q_u16.shape
    out = np.empty((B, H, N, D), dtype=np.float32)
    qs, ks, vs = _strides3(q_u16), _strides3(k_u16), _strides3(v_u16)
    lib.oracle_dense_attn(
        ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(N), ctypes.c_int(D), _p(q_u16),
        _p(k_u16), _p(v_u16), _p(qs), _p(ks), _p(vs), ctypes.c_float(scale), _p(out),
    )
    return out
