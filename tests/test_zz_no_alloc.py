"""heart_block_sparse_attn_static -- the entry point for callers that cannot allocate (HIP graph
capture, serving loops): its launch plan lives in a static device array of the library instead of
a caller workspace.  Called through the C ABI twice in a row, the second time with a smaller
input (the array still holds the first call's plan), its output must equal that of
heart_block_sparse_attn_flags with a workspace -- the same kernels on the same plan, so bit for
bit -- and the oracle's within the attention tolerance."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from heart_synth import make_generator
from heart_testlib import ATTN_ATOL, gpu, np_gpu, u16

pytestmark = pytest.mark.gpu


def _lists(g, st):
    cfg = g.cfg
    nt = cfg.n_text_blocks
    qb, _ = oracle.pool(u16(st.q), cfg.block)
    kb, _ = oracle.pool(u16(st.k), cfg.block)
    _, idx, cnt = oracle.topp(oracle.scores(qb, kb), g.tau, n_always_kv=nt, n_dense_q=nt)
    return idx, cnt


@pytest.mark.parametrize("flags", [0, 1])
def test_static_plan_entry_point_matches_workspace_entry_point(flags):
    import paper_2605_14513_amd as heart

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    heart.load_library()
    # first call: the larger input (B=2, H=3, N=690 ragged); second call: a smaller one
    for call, name in enumerate(["small_ragged", "small_d64"]):
        g = make_generator(name)
        cfg = g.cfg
        st = g.step(0)
        idx, cnt = _lists(g, st)
        q, k, v = gpu(st.q), gpu(st.k), gpu(st.v)
        gi, gc = np_gpu(idx), np_gpu(cnt)
        print(f"static plan call {call}: {name} B={cfg.B} H={cfg.H} N={cfg.N} D={cfg.D} flags={flags}", flush=True)
        ws = torch.empty(heart.heart_workspace_bytes(cfg.B, cfg.H, cfg.Nb, cfg.D), dtype=torch.uint8, device="cuda")
        lse_ref = torch.empty((cfg.B, cfg.H, cfg.N), dtype=torch.float32, device="cuda")
        ref = heart.heart_block_sparse_attn(q, k, v, cfg.block, gi, gc, workspace=ws, flags=flags, lse=lse_ref)
        out = torch.full_like(q, float("nan"))
        lse = torch.full_like(lse_ref, float("nan"))
        heart.heart_block_sparse_attn_static(q, k, v, cfg.block, gi, gc, out, flags=flags, lse=lse)
        torch.cuda.synchronize()
        assert torch.equal(out, ref), f"call {call}: output differs from the workspace entry point"
        assert torch.equal(lse, lse_ref)
        want = oracle.attn(u16(st.q), u16(st.k), u16(st.v), cfg.block, idx, cnt)
        err = np.abs(out.float().cpu().numpy().astype(np.float64) - want).max()
        assert err <= ATTN_ATOL, f"call {call}: max abs err {err:.4f} against the oracle"


def test_static_plan_entry_point_rejects_shapes_beyond_its_array():
    import paper_2605_14513_amd as heart
    from paper_2605_14513_amd.binding import HeartShape

    lib = heart.load_library()
    s = HeartShape()
    s.B, s.H, s.N, s.D, s.block = 1, 300, 128 * 1024, 128, 128  # plan of 300 * 1026 + 24 ints > 2^18
    for arr in (s.q_stride, s.k_stride, s.v_stride, s.o_stride):
        arr[0], arr[1], arr[2] = 0, 128, 300 * 128
    fake = ctypes.c_void_p(0x10000)  # never dereferenced: the size check comes first
    rc = lib.heart_block_sparse_attn_static(ctypes.byref(s), fake, fake, fake, fake, fake, 0.0, 0, fake, None, None)
    assert rc == -2 and b"static array" in lib.heart_last_error()
