"""CPU-side checks of the boundary: the library builds, loads and exports every
symbol that include/heart.h and include/heart_diag.h declare, and host-side validation
rejects bad calls before anything touches a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2605_14513_amd import build as hb
    from paper_2605_14513_amd import binding

    if hb.is_stale():
        hb.build(force=True)
    return binding.load_library()


def declared_symbols(headers=("heart.h", "heart_diag.h")):
    syms = set()
    for h in headers:
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        syms |= set(re.findall(r"\b(heart_[a-z_0-9]+)\s*\(", text))
    return sorted(syms)


def test_header_declares_the_four_hot_path_calls():
    syms = declared_symbols(("heart.h",))
    for s in ("heart_pool_qk", "heart_drift", "heart_mask_topp", "heart_block_sparse_attn",
              "heart_workspace_bytes", "heart_last_error", "heart_version"):
        assert s in syms
    # diagnostics live in their own header
    assert not [s for s in syms if "ubench" in s]
    assert "heart_ubench_read" in declared_symbols(("heart_diag.h",))


def test_library_exports_every_declared_symbol(lib):
    for s in declared_symbols():
        assert hasattr(lib, s), f"libheart.so does not export {s}"
    assert lib.heart_version() >= 100


def test_binding_names_match_header():
    import paper_2605_14513_amd as pkg

    for s in declared_symbols():
        assert hasattr(pkg, s), f"python binding lacks {s}"


def test_shape_struct_layout_matches_header():
    from paper_2605_14513_amd.binding import HeartShape

    # 5 ints (20 bytes, padded to 24) + 4 * 3 long long
    assert ctypes.sizeof(HeartShape) == 24 + 4 * 3 * 8
    assert HeartShape.q_stride.offset == 24 and HeartShape.o_stride.offset == 24 + 72


def test_host_validation_rejects_bad_calls_without_a_gpu(lib):
    from paper_2605_14513_amd.binding import HeartShape

    assert lib.heart_pool_qk(None, None, None, None, None, None, None, None) == -1
    assert b"shape is NULL" in lib.heart_last_error()
    s = HeartShape()
    s.B, s.H, s.N, s.D, s.block = 1, 2, 100, 96, 128
    assert lib.heart_pool_qk(ctypes.byref(s), None, None, None, None, None, None, None) == -2
    assert b"D must be 64 or 128" in lib.heart_last_error()
    s.D = 128
    assert lib.heart_pool_qk(ctypes.byref(s), None, None, None, None, None, None, None) == -1
    s.block = 100
    assert lib.heart_block_sparse_attn(ctypes.byref(s), None, None, None, None, None, 0.0, None,
                                       None, None, 0, None) == -2
    s.block = 128
    assert lib.heart_attn_workspace_bytes(ctypes.byref(s)) == (1 * 2 * (1 + 2) + 24) * 4
    assert lib.heart_attn_workspace_bytes(None) == 0
    assert lib.heart_workspace_bytes(1, 2, 1, 128) == (1 * 2 * (1 + 2) + 24) * 4
    assert lib.heart_workspace_bytes(1, 40, 256, 128) == (40 * 258 + 24) * 4
    assert lib.heart_workspace_bytes(0, 2, 1, 128) == 0
    fake = ctypes.c_void_p(0x10000)
    for arr in (s.q_stride, s.k_stride, s.v_stride, s.o_stride):
        arr[0], arr[1], arr[2] = 2 * 100 * 128, 100 * 128, 128
    # unknown option bits are refused before anything is launched
    assert lib.heart_block_sparse_attn_flags(ctypes.byref(s), fake, fake, fake, fake, fake, 0.0, 2,
                                             fake, None, None, 0, None) == -1
    assert b"flag" in lib.heart_last_error()
    assert lib.heart_drift(1, 2, 96, None, None, None, None, None, None, 0.4, 0.8, 1, None, None,
                           None) == -2
    assert lib.heart_drift(1, 2, 64, None, None, None, None, None, None, 0.4, 0.8, 1, None, None,
                           None) == -1
    assert lib.heart_mask_topp(1, 1, 2000, 128, None, None, None, None, None, 0, 0, 1, None, None,
                               None, None, None) == -2
    assert b"HEART_MAX_NB" in lib.heart_last_error()
    assert lib.heart_mask_topp(1, 1, 8, 128, None, None, None, None, None, 0, 0, 1, None, None,
                               None, None, None) == -1


def test_mask_topp_workspace_validation_without_a_gpu(lib):
    f = ctypes.c_void_p(0x10000)
    need = 1 * 40 * 256 * (2 * 4 * 128 + 2 * 4)  # slices of Q and K blocks and their exponents
    assert lib.heart_mask_topp_workspace_bytes(1, 40, 256, 128) == need
    assert lib.heart_mask_topp_workspace_bytes(1, 0, 256, 128) == 0
    args = lambda ws, nbytes: (1, 40, 256, 128, f, f, None, f, None, 0, 0, 1, f, f, f, None, ws, nbytes, None)
    assert lib.heart_mask_topp_ws(*args(f, need - 1)) == -1                     # too small
    assert b"workspace" in lib.heart_last_error()
    assert lib.heart_mask_topp_ws(*args(ctypes.c_void_p(0x10008), need)) == -2  # misaligned
    assert lib.heart_mask_topp_ws(1, 1, 2000, 128, f, f, None, f, None, 0, 0, 1, f, f, f, None, f,
                                  1 << 30, None) == -2                           # the checks of heart_mask_topp
    assert b"HEART_MAX_NB" in lib.heart_last_error()


def test_pool_drift_validation_without_a_gpu(lib):
    from paper_2605_14513_amd.binding import HeartShape

    s = HeartShape()
    s.B, s.H, s.N, s.D, s.block = 2, 40, 1000, 128, 128
    for arr in (s.q_stride, s.k_stride, s.v_stride, s.o_stride):
        arr[0], arr[1], arr[2] = 40 * 1000 * 128, 1000 * 128, 128
    f = ctypes.c_void_p(0x10000)
    args = lambda ws, nbytes, hi=0.8: (ctypes.byref(s), f, f, f, f, f, f, f, f, f, f, 0.4, hi, 1, f, f, ws, nbytes, None)
    assert lib.heart_pool_drift_workspace_bytes(2, 40) == 2 * 4  # one ticket per batch item
    assert lib.heart_pool_drift_workspace_bytes(0, 40) == 0
    assert lib.heart_pool_drift(*args(None, 8)) == -1                     # no workspace
    assert lib.heart_pool_drift(*args(f, 4)) == -1                        # too small
    assert b"workspace" in lib.heart_last_error()
    assert lib.heart_pool_drift(*args(ctypes.c_void_p(0x10002), 8)) == -2  # misaligned
    assert lib.heart_pool_drift(*args(f, 8, hi=0.1)) == -1                # gate_lo > gate_hi
    s.H = 5000
    assert lib.heart_pool_drift(*args(f, 1 << 20)) == -2                  # more heads than the drift stage holds


def test_estimator_validation_without_a_gpu(lib):
    """heart_scores_antidiag checks shape, stride relation, pointers, alignment and workspace
    size on the host; the pointers below are never dereferenced."""
    from paper_2605_14513_amd.binding import HeartShape

    s = HeartShape()
    s.B, s.H, s.N, s.D, s.block = 1, 2, 1000, 128, 128
    for arr in (s.q_stride, s.k_stride, s.v_stride, s.o_stride):
        arr[0], arr[1], arr[2] = 2 * 1000 * 128, 1000 * 128, 128
    fake = ctypes.c_void_p(0x10000)
    call = lib.heart_scores_antidiag
    assert call(None, fake, fake, 16, None, fake, fake, 1 << 30, None) == -1
    assert call(ctypes.byref(s), fake, fake, 8, None, fake, fake, 1 << 30, None) == -2
    assert b"8 * stride" in lib.heart_last_error()
    assert call(ctypes.byref(s), None, fake, 16, None, fake, fake, 1 << 30, None) == -1
    assert call(ctypes.byref(s), ctypes.c_void_p(0x10008), fake, 16, None, fake, fake, 1 << 30, None) == -2
    need = lib.heart_scores_antidiag_workspace_bytes(ctypes.byref(s), 16)
    # 63 reduced rows -> one 256-row tile -> 2 records of 128 keys: 16 * 2 sums + 2 maxima per row
    assert need == 1 * 2 * 63 * (32 + 2) * 4
    assert call(ctypes.byref(s), fake, fake, 16, None, fake, fake, need - 1, None) == -1
    assert b"workspace" in lib.heart_last_error()
    s.k_stride[2] = 132   # not a multiple of 8 elements
    assert call(ctypes.byref(s), fake, fake, 16, None, fake, fake, need, None) == -2
    s.k_stride[2] = 128
    s.N = 128 * 1025      # more key blocks than the mask kernel ranks
    assert call(ctypes.byref(s), fake, fake, 16, None, fake, fake, 1 << 40, None) == -2
    assert b"HEART_MAX_NB" in lib.heart_last_error()
    assert lib.heart_scores_antidiag_workspace_bytes(None, 16) == 0


def test_binding_refuses_cpu_tensors(lib):
    import torch

    import paper_2605_14513_amd as pkg

    q = torch.zeros((1, 1, 128, 128), dtype=torch.bfloat16)
    with pytest.raises(TypeError):
        pkg.heart_pool_qk(q, q, 128, qblk=torch.zeros(1, 1, 1, 128), kblk=torch.zeros(1, 1, 1, 128),
                          qmean=torch.zeros(1, 1, 128), kmean=torch.zeros(1, 1, 128))


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2605_14513_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "heart_oracle" not in text, f
