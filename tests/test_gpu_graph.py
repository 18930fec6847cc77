"""The whole step pool -> drift -> mask -> attention captured in one HIP graph and replayed.

The library promises that a call only enqueues kernels on the given stream: no allocation, no
synchronisation, no memset nodes, no host-side state that changes between calls.  Capturing a
step (including the attention launch plan, whose list cursors a kernel resets on every
launch) and replaying it several times, with eager work and synchronisations in between, must
give the eager results bit for bit on every replay."""
import numpy as np
import pytest
import torch

from heart_synth import make_generator
from heart_testlib import gpu, np_gpu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("estimator", ["pooled", "antidiag"])
def test_captured_step_replays_bit_exact(estimator):
    import paper_2605_14513_amd as heart

    g = make_generator("small_text")
    cfg = g.cfg
    B, H, D, Nb, N, blk, nt = cfg.B, cfg.H, cfg.D, cfg.Nb, cfg.N, cfg.block, cfg.n_text_blocks
    dev = "cuda"
    steps = [g.step(s) for s in range(cfg.steps)]
    tau, delta = np_gpu(g.tau), np_gpu(g.delta)
    f32 = dict(dtype=torch.float32, device=dev)

    def new_state():
        return dict(
            q=torch.empty((B, H, N, D), dtype=torch.bfloat16, device=dev),
            k=torch.empty((B, H, N, D), dtype=torch.bfloat16, device=dev),
            v=torch.empty((B, H, N, D), dtype=torch.bfloat16, device=dev),
            qblk=torch.empty((B, H, Nb, D), **f32), kblk=torch.empty((B, H, Nb, D), **f32),
            qmean=torch.empty((B, H, D), **f32), kmean=torch.empty((B, H, D), **f32),
            qa=torch.zeros((B, H, D), **f32), ka=torch.zeros((B, H, D), **f32),
            has=torch.zeros((B, H), dtype=torch.uint8, device=dev),
            drift=torch.zeros((B, H), **f32), refresh=torch.zeros((B, H), dtype=torch.uint8, device=dev),
            mask=torch.zeros((B, H, Nb, Nb), dtype=torch.uint8, device=dev),
            kidx=torch.zeros((B, H, Nb, Nb), dtype=torch.int32, device=dev),
            kcnt=torch.zeros((B, H, Nb), dtype=torch.int32, device=dev),
            out=torch.zeros((B, H, N, D), dtype=torch.bfloat16, device=dev),
            ws=torch.empty(heart.heart_attn_workspace_bytes(
                torch.empty((B, H, N, D), dtype=torch.bfloat16, device=dev), blk), dtype=torch.uint8, device=dev),
            scores=torch.zeros((B, H, Nb, Nb), **f32),
            ews=torch.empty(heart.heart_scores_antidiag_workspace_bytes(
                torch.empty((B, H, N, D), dtype=torch.bfloat16, device=dev), blk, blk // 8),
                dtype=torch.uint8, device=dev))

    def step(s):
        heart.heart_pool_qk(s["q"], s["k"], blk, s["qblk"], s["kblk"], s["qmean"], s["kmean"])
        heart.heart_drift(s["qmean"], s["kmean"], s["qa"], s["ka"], s["has"], delta, 0.4, 0.8, True,
                          s["drift"], s["refresh"])
        if estimator == "pooled":
            heart.heart_mask_topp(s["qblk"], s["kblk"], tau, refresh=s["refresh"], n_always_kv_blocks=nt,
                                  n_dense_q_blocks=nt, mask=s["mask"], kept_idx=s["kidx"], kept_count=s["kcnt"])
        else:
            heart.heart_scores_antidiag(s["q"], s["k"], blk, blk // 8, scores=s["scores"], workspace=s["ews"],
                                        refresh=s["refresh"])
            heart.heart_mask_topp(None, None, tau, scores_in=s["scores"], refresh=s["refresh"],
                                  n_always_kv_blocks=nt, n_dense_q_blocks=nt, mask=s["mask"],
                                  kept_idx=s["kidx"], kept_count=s["kcnt"])
        heart.heart_block_sparse_attn(s["q"], s["k"], s["v"], blk, s["kidx"], s["kcnt"], out=s["out"],
                                      workspace=s["ws"])

    def load(s, st):
        s["q"].copy_(gpu(st.q)); s["k"].copy_(gpu(st.k)); s["v"].copy_(gpu(st.v))

    # eager reference over the schedule
    eager = new_state()
    want = []
    for st in steps:
        load(eager, st)
        step(eager)
        torch.cuda.synchronize()
        want.append({k: eager[k].clone() for k in ("out", "refresh", "drift", "mask", "kcnt", "has")})

    # captured: warm up once on the side stream (per-function attributes are set on first use),
    # reset the state, capture one step, then replay it for every step of the schedule
    cap = new_state()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        load(cap, steps[0])
        step(cap)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for key in ("qa", "ka", "has", "mask", "kidx", "kcnt", "out", "scores"):
        cap[key].zero_()
    graph = torch.cuda.CUDAGraph()
    load(cap, steps[0])
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        step(cap)
    # the capture itself does not execute: state is still the reset one
    assert not cap["has"].any().item()
    for rep, st in enumerate(steps):
        load(cap, st)                      # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for key, ref in want[rep].items():
            assert torch.equal(cap[key], ref), f"replay {rep}: {key} differs from the eager run"
    # and once more from a fresh cache: the same graph, replayed after a reset
    for key in ("qa", "ka", "has"):
        cap[key].zero_()
    load(cap, steps[0])
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(cap["out"], want[0]["out"]) and torch.equal(cap["refresh"], want[0]["refresh"])
