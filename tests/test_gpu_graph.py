"""The whole step pool -> drift -> mask -> attention captured in one HIP graph and replayed.

The library promises that a call only enqueues kernels on the given stream: no allocation, no
synchronisation, no memset nodes, no host-side state that changes between calls.  Capturing a
step (including the attention launch plan, whose list cursors a kernel resets on every
launch) and replaying it several times, with eager work and synchronisations in between, must
give the eager results bit for bit on every replay -- and every replay is also checked against
the oracle's chained run of the same schedule (decisions exact, masks equal up to threshold
rows, attention within tolerance), so the captured path is held to the same parity bar as the
eager one."""
import numpy as np
import pytest
import torch

import oracle
from oracle import antidiag_oracle
from heart_synth import make_generator
from heart_testlib import (ATTN_ATOL, SCORE_RTOL, OracleChain, assert_masks_equal_up_to_threshold, gpu,
                           np_gpu, pooled_mean_score_shift, u16)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("estimator", ["pooled", "pooled_sliced", "antidiag"])
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
            tickets=torch.zeros(heart.heart_pool_drift_workspace_bytes(B, H), dtype=torch.uint8, device=dev),
            scores=torch.zeros((B, H, Nb, Nb), **f32),
            ews=torch.empty(heart.heart_scores_antidiag_workspace_bytes(
                torch.empty((B, H, N, D), dtype=torch.bfloat16, device=dev), blk, blk // 8),
                dtype=torch.uint8, device=dev),
            # heart_mask_topp_ws: the score stage on 8-bit slices, one more launch in the graph
            tws=(torch.empty(heart.heart_mask_topp_workspace_bytes(B, H, Nb, D), dtype=torch.uint8, device=dev)
                 if estimator == "pooled_sliced" else None))

    def step(s):
        # pooling pass, then token means, drift and gate in one launch (its ticket counters return to zero
        # by themselves, which a replayed graph relies on)
        heart.heart_pool_drift(s["q"], s["k"], blk, s["qa"], s["ka"], s["has"], delta, s["tickets"], 0.4, 0.8,
                               True, s["qblk"], s["kblk"], s["qmean"], s["kmean"], s["drift"], s["refresh"])
        if estimator.startswith("pooled"):
            heart.heart_mask_topp(s["qblk"], s["kblk"], tau, refresh=s["refresh"], n_always_kv_blocks=nt,
                                  n_dense_q_blocks=nt, mask=s["mask"], kept_idx=s["kidx"], kept_count=s["kcnt"],
                                  workspace=s["tws"])
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
    chain = OracleChain(cfg, g.tau, g.delta)
    for rep, st in enumerate(steps):
        load(cap, st)                      # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for key, ref in want[rep].items():
            assert torch.equal(cap[key], ref), f"replay {rep}: {key} differs from the eager run"
        # the same replay against the oracle's chain
        od, orf = chain.step(st)
        assert np.array_equal(cap["refresh"].cpu().numpy(), orf), f"replay {rep}: decisions differ from the oracle"
        assert np.array_equal(cap["has"].cpu().numpy(), chain.has)
        fin = np.isfinite(od)
        assert np.allclose(cap["drift"].cpu().numpy()[fin], od[fin], rtol=1e-4, atol=1e-6)
        if estimator.startswith("pooled"):
            osc, tol = chain.scores, SCORE_RTOL
            shift = pooled_mean_score_shift(osc, cap["qblk"], cap["kblk"])
        else:
            # the oracle's lists for this estimator: its own scores, the same top-p rule and cache
            osc = np.stack([np.stack([antidiag_oracle.antidiag_scores(
                st.q[b, h].double().numpy(), st.k[b, h].double().numpy(), blk, blk // 8)
                for h in range(H)]) for b in range(B)]).astype(np.float32)
            if rep == 0:
                amask, aidx, acnt = (np.zeros_like(chain.mask), np.zeros_like(chain.idx), np.zeros_like(chain.cnt))
            oracle.topp(osc, g.tau, refresh=orf, n_always_kv=nt, n_dense_q=nt, mask=amask, kept_idx=aidx,
                        kept_count=acnt)
            chain.mask, chain.idx, chain.cnt = amask, aidx, acnt
            tol, shift = 2e-3, None  # score tolerance of the antidiagonal-style estimator
        gm = cap["mask"].cpu().numpy()
        fresh = orf.astype(bool)[:, :, None, None]
        assert_masks_equal_up_to_threshold(np.where(fresh, gm, chain.mask), chain.mask, osc, chain.cnt, g.tau,
                                           f"{estimator} replay {rep}", tol=tol, row_tol=shift)
        same = ~(gm != chain.mask).any(-1)
        assert np.array_equal(cap["kcnt"].cpu().numpy()[same], chain.cnt[same])
        oout = oracle.attn(u16(st.q), u16(st.k), u16(st.v), blk, chain.idx, chain.cnt)
        rows_same = np.repeat(same, blk, axis=2)[:, :, :N]
        err = np.abs(cap["out"].float().cpu().numpy().astype(np.float64) - oout)[rows_same].max()
        assert err <= ATTN_ATOL, f"replay {rep}: attention max abs err {err:.4f} against the oracle"
    # and once more from a fresh cache: the same graph, replayed after a reset
    for key in ("qa", "ka", "has"):
        cap[key].zero_()
    load(cap, steps[0])
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(cap["out"], want[0]["out"]) and torch.equal(cap["refresh"], want[0]["refresh"])
