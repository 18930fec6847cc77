"""ctypes binding of libheart.so.  Argument marshalling only.

Functions take torch tensors that live on the GPU, pass their device pointers,
shapes and strides to the C ABI declared in include/heart.h, and enqueue on
torch's current HIP stream.  There is no fallback: if the library is missing or
a tensor is not on the GPU, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libheart.so")
_lib: Optional[ctypes.CDLL] = None


class HeartError(RuntimeError):
    """A libheart entry point returned a negative code."""

    def __init__(self, fn: str, code: int, msg: str):
        super().__init__(f"{fn} failed with code {code}: {msg}")
        self.code = code


class HeartShape(ctypes.Structure):
    """Mirror of `heart_shape` in include/heart.h."""

    _fields_ = [
        ("B", ctypes.c_int), ("H", ctypes.c_int), ("N", ctypes.c_int), ("D", ctypes.c_int),
        ("block", ctypes.c_int),
        ("q_stride", ctypes.c_longlong * 3), ("k_stride", ctypes.c_longlong * 3),
        ("v_stride", ctypes.c_longlong * 3), ("o_stride", ctypes.c_longlong * 3),
    ]


def lib_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libheart.so (built by paper_2605_14513_amd.build); raise if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is not built; run `python -m paper_2605_14513_amd.build` "
            "(there is no CPU or PyTorch fallback for the HEART kernels)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    sp = ctypes.POINTER(HeartShape)
    lib.heart_pool_qk.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp]
    lib.heart_drift.argtypes = [ci, ci, ci, vp, vp, vp, vp, vp, vp, cf, cf, ci, vp, vp, vp]
    lib.heart_mask_topp.argtypes = [ci, ci, ci, ci, vp, vp, vp, vp, vp, ci, ci, ci, vp, vp, vp,
                                    vp, vp]
    lib.heart_mask_topp_ws.argtypes = [ci, ci, ci, ci, vp, vp, vp, vp, vp, ci, ci, ci, vp, vp, vp,
                                       vp, vp, ctypes.c_size_t, vp]
    lib.heart_mask_topp_ws.restype = ci
    lib.heart_mask_topp_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.heart_mask_topp_workspace_bytes.restype = ctypes.c_size_t
    lib.heart_block_sparse_attn.argtypes = [sp, vp, vp, vp, vp, vp, cf, vp, vp, vp,
                                            ctypes.c_size_t, vp]
    lib.heart_pool_drift.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, cf, cf, ci, vp, vp, vp,
                                     ctypes.c_size_t, vp]
    lib.heart_pool_drift.restype = ci
    lib.heart_pool_drift_workspace_bytes.argtypes = [ci, ci]
    lib.heart_pool_drift_workspace_bytes.restype = ctypes.c_size_t
    lib.heart_block_sparse_attn_flags.argtypes = [sp, vp, vp, vp, vp, vp, cf, ctypes.c_uint, vp, vp,
                                                  vp, ctypes.c_size_t, vp]
    lib.heart_block_sparse_attn_static.argtypes = [sp, vp, vp, vp, vp, vp, cf, ctypes.c_uint, vp, vp, vp]
    lib.heart_block_sparse_attn_static.restype = ci
    lib.heart_attn_workspace_bytes.argtypes = [sp]
    lib.heart_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.heart_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.heart_workspace_bytes.restype = ctypes.c_size_t
    for f in (lib.heart_pool_qk, lib.heart_drift, lib.heart_mask_topp,
              lib.heart_block_sparse_attn, lib.heart_block_sparse_attn_flags, lib.heart_version):
        f.restype = ci
    lib.heart_ubench_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    lib.heart_ubench_read.restype = ci
    lib.heart_ubench_mfma_bf16.argtypes = [vp, vp, ci, ci, vp, vp]
    lib.heart_ubench_mfma_bf16.restype = ci
    lib.heart_ubench_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.heart_ubench_copy.restype = ci
    lib.heart_ebc_band_error.argtypes = [ctypes.c_longlong, ci, ci, ci, vp, vp, vp, ctypes.c_double, vp,
                                         ctypes.c_size_t, vp, vp]
    lib.heart_ebc_band_error.restype = ci
    lib.heart_ebc_workspace_bytes.argtypes = [ctypes.c_longlong, ci, ci, ci]
    lib.heart_ebc_workspace_bytes.restype = ctypes.c_size_t
    lib.heart_ebc_select.argtypes = [ci, ci, vp, vp, ctypes.c_double, vp, vp]
    lib.heart_ebc_select.restype = ci
    lib.heart_scores_antidiag.argtypes = [sp, vp, vp, ci, vp, vp, vp, ctypes.c_size_t, vp]
    lib.heart_scores_antidiag.restype = ci
    lib.heart_scores_antidiag_workspace_bytes.argtypes = [sp, ci]
    lib.heart_scores_antidiag_workspace_bytes.restype = ctypes.c_size_t
    lib.heart_last_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


def heart_last_error() -> str:
    return load_library().heart_last_error().decode()


def heart_version() -> int:
    return int(load_library().heart_version())


def _check(fn: str, rc: int) -> None:
    if rc != 0:
        raise HeartError(fn, rc, heart_last_error())


def _dev(t: Optional[torch.Tensor], dtype, name: str, contiguous: bool = True):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or t.device.type != "cuda":
        raise TypeError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if contiguous and not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _strides_bhn(t: torch.Tensor, name: str) -> Tuple[int, int, int]:
    if t.dim() != 4 or t.stride(3) != 1:
        raise ValueError(f"{name} must be [B,H,N,D] with a contiguous D axis")
    return t.stride(0), t.stride(1), t.stride(2)


def make_shape(q: torch.Tensor, k: torch.Tensor, block: int, v: Optional[torch.Tensor] = None,
               o: Optional[torch.Tensor] = None) -> HeartShape:
    B, H, N, D = q.shape
    s = HeartShape()
    s.B, s.H, s.N, s.D, s.block = B, H, N, D, block
    s.q_stride[:] = _strides_bhn(q, "q")
    s.k_stride[:] = _strides_bhn(k, "k")
    s.v_stride[:] = _strides_bhn(v if v is not None else k, "v")
    s.o_stride[:] = _strides_bhn(o if o is not None else q, "out")
    return s


def heart_pool_qk(q: torch.Tensor, k: torch.Tensor, block: int, qblk=None, kblk=None, qmean=None,
                  kmean=None):
    """Block means [B,H,Nb,D] and token means [B,H,D] of bf16 q, k ([B,H,N,D] views)."""
    lib = load_library()
    if q.shape != k.shape:
        raise ValueError("q and k must have the same shape")
    B, H, N, D = q.shape
    Nb = (N + block - 1) // block
    f32 = dict(dtype=torch.float32, device=q.device)
    qblk = torch.empty((B, H, Nb, D), **f32) if qblk is None else qblk
    kblk = torch.empty((B, H, Nb, D), **f32) if kblk is None else kblk
    qmean = torch.empty((B, H, D), **f32) if qmean is None else qmean
    kmean = torch.empty((B, H, D), **f32) if kmean is None else kmean
    shape = make_shape(q, k, block)
    rc = lib.heart_pool_qk(ctypes.byref(shape), _dev(q, torch.bfloat16, "q", False),
                           _dev(k, torch.bfloat16, "k", False), _dev(qblk, torch.float32, "qblk"),
                           _dev(kblk, torch.float32, "kblk"), _dev(qmean, torch.float32, "qmean"),
                           _dev(kmean, torch.float32, "kmean"), _stream())
    _check("heart_pool_qk", rc)
    return qblk, kblk, qmean, kmean


def heart_drift(qmean, kmean, qanchor, kanchor, has_anchor, delta, gate_lo: float = 0.4,
                gate_hi: float = 0.8, commit: bool = True, drift=None, refresh=None):
    """Drift, reuse rule, layer gate; updates qanchor/kanchor/has_anchor in place."""
    lib = load_library()
    B, H, D = qmean.shape
    drift = torch.empty((B, H), dtype=torch.float32, device=qmean.device) if drift is None else drift
    refresh = torch.empty((B, H), dtype=torch.uint8, device=qmean.device) if refresh is None else refresh
    if delta.numel() != H:
        raise ValueError("delta must have H entries")
    for t, n in ((kmean, "kmean"), (qanchor, "qanchor"), (kanchor, "kanchor")):
        if tuple(t.shape) != (B, H, D):
            raise ValueError(f"{n} must be [B,H,D]")
    if tuple(has_anchor.shape) != (B, H) or tuple(drift.shape) != (B, H) or tuple(refresh.shape) != (B, H):
        raise ValueError("has_anchor, drift, refresh must be [B,H]")
    rc = lib.heart_drift(B, H, D, _dev(qmean, torch.float32, "qmean"),
                         _dev(kmean, torch.float32, "kmean"),
                         _dev(qanchor, torch.float32, "qanchor"),
                         _dev(kanchor, torch.float32, "kanchor"),
                         _dev(has_anchor, torch.uint8, "has_anchor"),
                         _dev(delta, torch.float32, "delta"), float(gate_lo), float(gate_hi),
                         1 if commit else 0, _dev(drift, torch.float32, "drift"),
                         _dev(refresh, torch.uint8, "refresh"), _stream())
    _check("heart_drift", rc)
    return drift, refresh


def heart_pool_drift_workspace_bytes(B: int, H: int) -> int:
    return int(load_library().heart_pool_drift_workspace_bytes(int(B), int(H)))


def heart_pool_drift(q, k, block: int, qanchor, kanchor, has_anchor, delta, workspace,
                     gate_lo: float = 0.4, gate_hi: float = 0.8, commit: bool = True, qblk=None,
                     kblk=None, qmean=None, kmean=None, drift=None, refresh=None):
    """heart_pool_qk and heart_drift with one launch fewer (token means and drift share a launch).  workspace: a GPU tensor of at least
    heart_pool_drift_workspace_bytes(B, H) bytes that was zero before its first use (the call
    leaves it zero).  Returns (qblk, kblk, qmean, kmean, drift, refresh)."""
    lib = load_library()
    if q.shape != k.shape:
        raise ValueError("q and k must have the same shape")
    B, H, N, D = q.shape
    Nb = (N + block - 1) // block
    f32 = dict(dtype=torch.float32, device=q.device)
    qblk = torch.empty((B, H, Nb, D), **f32) if qblk is None else qblk
    kblk = torch.empty((B, H, Nb, D), **f32) if kblk is None else kblk
    qmean = torch.empty((B, H, D), **f32) if qmean is None else qmean
    kmean = torch.empty((B, H, D), **f32) if kmean is None else kmean
    drift = torch.empty((B, H), **f32) if drift is None else drift
    refresh = torch.empty((B, H), dtype=torch.uint8, device=q.device) if refresh is None else refresh
    if delta.numel() != H:
        raise ValueError("delta must have H entries")
    for t, n in ((qanchor, "qanchor"), (kanchor, "kanchor"), (qmean, "qmean"), (kmean, "kmean")):
        if tuple(t.shape) != (B, H, D):
            raise ValueError(f"{n} must be [B,H,D]")
    if tuple(has_anchor.shape) != (B, H) or tuple(drift.shape) != (B, H) or tuple(refresh.shape) != (B, H):
        raise ValueError("has_anchor, drift, refresh must be [B,H]")
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    shape = make_shape(q, k, block)
    rc = lib.heart_pool_drift(
        ctypes.byref(shape), _dev(q, torch.bfloat16, "q", False), _dev(k, torch.bfloat16, "k", False),
        _dev(qblk, torch.float32, "qblk"), _dev(kblk, torch.float32, "kblk"),
        _dev(qmean, torch.float32, "qmean"), _dev(kmean, torch.float32, "kmean"),
        _dev(qanchor, torch.float32, "qanchor"), _dev(kanchor, torch.float32, "kanchor"),
        _dev(has_anchor, torch.uint8, "has_anchor"), _dev(delta, torch.float32, "delta"),
        float(gate_lo), float(gate_hi), 1 if commit else 0, _dev(drift, torch.float32, "drift"),
        _dev(refresh, torch.uint8, "refresh"), ctypes.c_void_p(workspace.data_ptr()),
        workspace.numel() * workspace.element_size(), _stream())
    _check("heart_pool_drift", rc)
    return qblk, kblk, qmean, kmean, drift, refresh


def heart_mask_topp(qblk, kblk, tau, refresh=None, scores_in=None, n_always_kv_blocks: int = 0,
                    n_dense_q_blocks: int = 0, min_keep: int = 1, mask=None, kept_idx=None,
                    kept_count=None, scores_out=None, workspace=None):
    """Top-p block mask; writes mask/kept_idx/kept_count in place for refreshed heads.
    workspace: a contiguous GPU tensor of at least heart_mask_topp_workspace_bytes(B, H, Nb, D)
    bytes (heart_mask_topp_ws: score stage on the int8 matrix cores), or None."""
    lib = load_library()
    if scores_in is not None:
        B, H, Nb, _ = scores_in.shape
        D = 0 if qblk is None else qblk.shape[-1]
        dev = scores_in.device
    else:
        B, H, Nb, D = qblk.shape
        dev = qblk.device
    if mask is None:
        mask = torch.zeros((B, H, Nb, Nb), dtype=torch.uint8, device=dev)
    if kept_idx is None:
        kept_idx = torch.full((B, H, Nb, Nb), -1, dtype=torch.int32, device=dev)
    if kept_count is None:
        kept_count = torch.zeros((B, H, Nb), dtype=torch.int32, device=dev)
    if tau.numel() != H:
        raise ValueError("tau must have H entries")
    for t, shp, n in ((mask, (B, H, Nb, Nb), "mask"), (kept_idx, (B, H, Nb, Nb), "kept_idx"),
                      (kept_count, (B, H, Nb), "kept_count")):
        if tuple(t.shape) != shp:
            raise ValueError(f"{n} must have shape {shp}")
    if scores_out is not None and tuple(scores_out.shape) != (B, H, Nb, Nb):
        raise ValueError("scores_out must be [B,H,Nb,Nb]")
    if refresh is not None and tuple(refresh.shape) != (B, H):
        raise ValueError("refresh must be [B,H]")
    if scores_in is None and tuple(kblk.shape) != (B, H, Nb, D):
        raise ValueError("kblk must match qblk")
    args = (B, H, Nb, D, _dev(qblk, torch.float32, "qblk"), _dev(kblk, torch.float32, "kblk"),
            _dev(scores_in, torch.float32, "scores_in"), _dev(tau, torch.float32, "tau"),
            _dev(refresh, torch.uint8, "refresh"), int(n_always_kv_blocks), int(n_dense_q_blocks),
            int(min_keep), _dev(mask, torch.uint8, "mask"), _dev(kept_idx, torch.int32, "kept_idx"),
            _dev(kept_count, torch.int32, "kept_count"), _dev(scores_out, torch.float32, "scores_out"))
    if workspace is None:
        rc = lib.heart_mask_topp(*args, _stream())
        _check("heart_mask_topp", rc)
    else:
        if not workspace.is_contiguous():
            raise ValueError("workspace must be contiguous")
        rc = lib.heart_mask_topp_ws(*args, ctypes.c_void_p(workspace.data_ptr()),
                                    workspace.numel() * workspace.element_size(), _stream())
        _check("heart_mask_topp_ws", rc)
    return mask, kept_idx, kept_count


def heart_mask_topp_ws(qblk, kblk, tau, workspace, **kw):
    """heart_mask_topp with a workspace (same keyword arguments)."""
    if workspace is None:
        raise ValueError("heart_mask_topp_ws needs a workspace")
    return heart_mask_topp(qblk, kblk, tau, workspace=workspace, **kw)


def heart_mask_topp_workspace_bytes(B: int, H: int, Nb: int, D: int) -> int:
    """Bytes of workspace for heart_mask_topp(workspace=...)."""
    return int(load_library().heart_mask_topp_workspace_bytes(int(B), int(H), int(Nb), int(D)))


HEART_ATTN_FOLD_SCALE = 1  # flag of heart_block_sparse_attn_flags (include/heart.h)


def heart_workspace_bytes(B: int, H: int, Nb: int, D: int) -> int:
    """Bytes of workspace one call of the hot path can use (the attention launch plan)."""
    return int(load_library().heart_workspace_bytes(int(B), int(H), int(Nb), int(D)))


def heart_attn_workspace_bytes(q, block: int) -> int:
    """Bytes of workspace heart_block_sparse_attn can use for tensors shaped like q."""
    return int(load_library().heart_attn_workspace_bytes(ctypes.byref(make_shape(q, q, block))))


def heart_block_sparse_attn(q, k, v, block: int, kept_idx, kept_count, scale: float = 0.0,
                            out=None, lse=None, workspace="auto", flags: int = 0):
    """Block-sparse attention over the kept key blocks; returns bf16 out like q.

    workspace: a uint8/int32 GPU tensor of at least heart_attn_workspace_bytes, None (natural
    launch order), or "auto" (a fresh tensor from torch's allocator).
    flags: 0 (heart_block_sparse_attn) or HEART_ATTN_FOLD_SCALE (heart_block_sparse_attn_flags)."""
    lib = load_library()
    if q.shape != k.shape or q.shape != v.shape:
        raise ValueError("q, k, v must have the same shape")
    B, H, N, D = q.shape
    Nb = (N + block - 1) // block
    if out is None:
        out = torch.empty_like(q)
    if tuple(kept_idx.shape) != (B, H, Nb, Nb) or tuple(kept_count.shape) != (B, H, Nb):
        raise ValueError("kept_idx must be [B,H,Nb,Nb] and kept_count [B,H,Nb]")
    if lse is not None and tuple(lse.shape) != (B, H, N):
        raise ValueError("lse must be [B,H,N]")
    shape = make_shape(q, k, block, v, out)
    if isinstance(workspace, str):
        if workspace != "auto":
            raise ValueError("workspace must be a tensor, None or 'auto'")
        workspace = torch.empty(int(lib.heart_attn_workspace_bytes(ctypes.byref(shape))),
                                dtype=torch.uint8, device=q.device)
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        if not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("workspace must be a contiguous GPU tensor")
        ws_ptr, ws_bytes = ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()
    args = [ctypes.byref(shape), _dev(q, torch.bfloat16, "q", False),
            _dev(k, torch.bfloat16, "k", False), _dev(v, torch.bfloat16, "v", False),
            _dev(kept_idx, torch.int32, "kept_idx"), _dev(kept_count, torch.int32, "kept_count"),
            float(scale)]
    tail = [_dev(out, torch.bfloat16, "out", False), _dev(lse, torch.float32, "lse"), ws_ptr,
            ws_bytes, _stream()]
    if flags:
        _check("heart_block_sparse_attn_flags",
               lib.heart_block_sparse_attn_flags(*args, int(flags), *tail))
    else:
        _check("heart_block_sparse_attn", lib.heart_block_sparse_attn(*args, *tail))
    return out


def heart_block_sparse_attn_flags(q, k, v, block: int, kept_idx, kept_count, flags: int,
                                  scale: float = 0.0, out=None, lse=None, workspace="auto"):
    """heart_block_sparse_attn with option flags (HEART_ATTN_FOLD_SCALE)."""
    return heart_block_sparse_attn(q, k, v, block, kept_idx, kept_count, scale=scale, out=out,
                                   lse=lse, workspace=workspace, flags=flags)


def heart_block_sparse_attn_static(q, k, v, block: int, kept_idx, kept_count, out, flags: int = 0,
                                   scale: float = 0.0, lse=None):
    """heart_block_sparse_attn with the launch plan in the library's static device array: the
    call allocates nothing (so `out` must be given)."""
    lib = load_library()
    if q.shape != k.shape or q.shape != v.shape or out.shape != q.shape:
        raise ValueError("q, k, v, out must have the same shape")
    B, H, N, D = q.shape
    Nb = (N + block - 1) // block
    if tuple(kept_idx.shape) != (B, H, Nb, Nb) or tuple(kept_count.shape) != (B, H, Nb):
        raise ValueError("kept_idx must be [B,H,Nb,Nb] and kept_count [B,H,Nb]")
    if lse is not None and tuple(lse.shape) != (B, H, N):
        raise ValueError("lse must be [B,H,N]")
    shape = make_shape(q, k, block, v, out)
    rc = lib.heart_block_sparse_attn_static(
        ctypes.byref(shape), _dev(q, torch.bfloat16, "q", False), _dev(k, torch.bfloat16, "k", False),
        _dev(v, torch.bfloat16, "v", False), _dev(kept_idx, torch.int32, "kept_idx"),
        _dev(kept_count, torch.int32, "kept_count"), float(scale), int(flags),
        _dev(out, torch.bfloat16, "out", False), _dev(lse, torch.float32, "lse"), _stream())
    _check("heart_block_sparse_attn_static", rc)
    return out


def heart_ubench_mfma_bf16(a, b, n_workgroups: int, iters: int, sink=None):
    """Enqueue the MFMA-only diagnostic loop; returns the FLOPs it performs."""
    lib = load_library()
    if a.numel() != 8192 or b.numel() != 8192:
        raise ValueError("operands must hold 8192 bf16 elements")
    if sink is None:
        sink = torch.zeros(1, dtype=torch.float32, device=a.device)
    rc = lib.heart_ubench_mfma_bf16(_dev(a, torch.bfloat16, "a"), _dev(b, torch.bfloat16, "b"),
                                    int(n_workgroups), int(iters), _dev(sink, torch.float32, "sink"),
                                    _stream())
    _check("heart_ubench_mfma_bf16", rc)
    return float(n_workgroups) * 4 * iters * 16 * 32768


def heart_ubench_copy(src, dst):
    """Enqueue a plain device copy src -> dst; returns the HBM bytes it moves (read + write)."""
    lib = load_library()
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst must have the same size")
    rc = lib.heart_ubench_copy(_dev(src, src.dtype, "src"), _dev(dst, dst.dtype, "dst"), nbytes, _stream())
    _check("heart_ubench_copy", rc)
    return 2.0 * nbytes


def heart_ubench_read(src, sink=None):
    """Enqueue a read-only stream over src (the pooling kernel's access pattern); returns the
    HBM bytes it moves."""
    lib = load_library()
    nbytes = src.numel() * src.element_size()
    if sink is None:
        sink = torch.zeros(1, dtype=torch.int32, device=src.device)
    rc = lib.heart_ubench_read(_dev(src, src.dtype, "src"), nbytes, _dev(sink, torch.int32, "sink"), _stream())
    _check("heart_ubench_read", rc)
    return float(nbytes)


def heart_scores_antidiag_workspace_bytes(q, block: int, stride: int) -> int:
    """Bytes of workspace heart_scores_antidiag needs for tensors shaped like q."""
    return int(load_library().heart_scores_antidiag_workspace_bytes(
        ctypes.byref(make_shape(q, q, block)), int(stride)))


def heart_scores_antidiag(q, k, block: int, stride: int, scores=None, workspace=None, refresh=None):
    """Antidiagonal-style block scores fp32 [B,H,Nb,Nb] of bf16 q, k ([B,H,N,D] views), for
    heart_mask_topp(scores_in=...).  workspace: a contiguous GPU tensor of at least
    heart_scores_antidiag_workspace_bytes, or None (a fresh tensor from torch's allocator);
    refresh: uint8 [B,H] or None: heads with 0 are skipped (their scores stay as they are)."""
    lib = load_library()
    if q.shape != k.shape:
        raise ValueError("q and k must have the same shape")
    B, H, N, D = q.shape
    Nb = (N + block - 1) // block
    if refresh is not None and tuple(refresh.shape) != (B, H):
        raise ValueError("refresh must be [B,H]")
    shape = make_shape(q, k, block)
    need = int(lib.heart_scores_antidiag_workspace_bytes(ctypes.byref(shape), int(stride)))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    if scores is None:
        scores = torch.empty((B, H, Nb, Nb), dtype=torch.float32, device=q.device)
    elif tuple(scores.shape) != (B, H, Nb, Nb):
        raise ValueError("scores must be [B,H,Nb,Nb]")
    rc = lib.heart_scores_antidiag(ctypes.byref(shape), _dev(q, torch.bfloat16, "q", False),
                                   _dev(k, torch.bfloat16, "k", False), int(stride),
                                   _dev(refresh, torch.uint8, "refresh"),
                                   _dev(scores, torch.float32, "scores"),
                                   ctypes.c_void_p(workspace.data_ptr()),
                                   workspace.numel() * workspace.element_size(), _stream())
    _check("heart_scores_antidiag", rc)
    return scores


def heart_ebc_workspace_bytes(C: int, T: int, Y: int, X: int) -> int:
    return int(load_library().heart_ebc_workspace_bytes(C, T, Y, X))


def heart_ebc_band_error(err, dense, weights=(1.0, 0.5, 0.01, 0.01), epsilon: float = 1e-10,
                         workspace=None, out=None):
    """Frequency-weighted velocity error of fp32 GPU tensors [..., T, Y, X] (leading axes are
    summed over).  Returns a GPU float64 tensor [6]: error, E_LL, E_LH, E_HL, E_HH, dense energy."""
    lib = load_library()
    if err.shape != dense.shape or err.dim() < 3:
        raise ValueError("err and dense must have the same shape [..., T, Y, X]")
    T, Y, X = (int(v) for v in err.shape[-3:])
    C = int(err.numel() // (T * Y * X))
    need = int(lib.heart_ebc_workspace_bytes(C, T, Y, X))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=err.device)
    if out is None:
        out = torch.empty(6, dtype=torch.float64, device=err.device)
    w = (ctypes.c_double * 4)(*[float(x) for x in weights])
    rc = lib.heart_ebc_band_error(C, T, Y, X, _dev(err, torch.float32, "err"),
                                  _dev(dense, torch.float32, "dense"), w, float(epsilon),
                                  _dev(workspace, workspace.dtype, "workspace"),
                                  workspace.numel() * workspace.element_size(),
                                  _dev(out, torch.float64, "out"), _stream())
    _check("heart_ebc_band_error", rc)
    return out


def heart_ebc_select(error, sparsity, min_mean_sparsity: float):
    """Exact one-candidate-per-head selection (host).  error, sparsity: array-likes
    [n_heads, n_candidates].  Returns (choice int32 numpy [n_heads], total error)."""
    import numpy as np

    lib = load_library()
    E = np.ascontiguousarray(error, dtype=np.float64)
    S = np.ascontiguousarray(sparsity, dtype=np.float64)
    if E.ndim != 2 or E.shape != S.shape:
        raise ValueError("error and sparsity must be [n_heads, n_candidates]")
    choice = np.zeros(E.shape[0], dtype=np.int32)
    total = ctypes.c_double(0.0)
    rc = lib.heart_ebc_select(E.shape[0], E.shape[1], E.ctypes.data_as(ctypes.c_void_p),
                              S.ctypes.data_as(ctypes.c_void_p), float(min_mean_sparsity),
                              choice.ctypes.data_as(ctypes.c_void_p), ctypes.byref(total))
    _check("heart_ebc_select", rc)
    return choice, float(total.value)
