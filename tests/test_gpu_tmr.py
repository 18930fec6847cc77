"""Multi-step, multi-layer Temporal Mask Reuse (paper_2605_14513_amd.tmr) against a plain
simulation of the same schedule built from the oracle's single-step functions: the reuse
decisions of Alg. 1 over several steps with per-(layer) caches, the dense warm-up steps
(Experimental Setup), and the two shared schedules the paper's ablation compares with
(fixed-interval refresh, switch-to-reuse after a preset step)."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from oracle import antidiag_oracle
from heart_synth import CONFIGS, HeartInputGenerator
from heart_testlib import (ATTN_ATOL, SCORE_RTOL, assert_masks_equal_up_to_threshold, gpu, np_gpu,
                           pooled_mean_score_shift, u16)

ANTIDIAG_SCORE_RTOL = 2e-3  # score tolerance of the antidiagonal-style estimator (fp32 sums of bf16 products)

pytestmark = pytest.mark.gpu

STEPS, DENSE_STEPS, LAYERS = 7, 2, 2


@pytest.fixture(scope="module")
def inputs():
    cfg = dataclasses.replace(CONFIGS["small_ragged"], name="small_ragged_tmr", steps=STEPS)
    g = HeartInputGenerator(cfg)
    return g, [g.step(s) for s in range(STEPS)]


def oracle_refreshes(policy, sparse_call):
    name, _, arg = policy.partition(":")
    if name == "always":
        return True
    if name == "interval":
        return sparse_call % int(arg) == 0
    if name == "warmup":
        return sparse_call < int(arg)
    raise AssertionError(policy)


@pytest.mark.parametrize("policy,estimator", [("heart", "pooled"), ("always", "pooled"), ("interval:2", "pooled"),
                                              ("warmup:2", "pooled"), ("heart", "antidiag"),
                                              ("interval:2", "antidiag")])
def test_tmr_driver_matches_oracle_simulation(inputs, policy, estimator):
    from paper_2605_14513_amd.tmr import TmrConfig, TmrDriver

    g, steps = inputs
    cfg = g.cfg
    B, H, D, Nb, N, blk = cfg.B, cfg.H, cfg.D, cfg.Nb, cfg.N, cfg.block
    drv = TmrDriver(TmrConfig(B=B, H=H, N=N, D=D, block=blk, tau=np_gpu(g.tau), delta=np_gpu(g.delta),
                              policy=policy, estimator=estimator, dense_steps=DENSE_STEPS),
                    n_layers=LAYERS, n_branches=1, record=True)
    # oracle-side caches, one per layer
    ost = [dict(qa=np.zeros((B, H, D), np.float32), ka=np.zeros((B, H, D), np.float32),
                has=np.zeros((B, H), np.uint8), mask=np.zeros((B, H, Nb, Nb), np.uint8),
                idx=np.zeros((B, H, Nb, Nb), np.int32), cnt=np.zeros((B, H, Nb), np.int32), calls=0)
           for _ in range(LAYERS)]
    dense_idx = np.broadcast_to(np.arange(Nb, dtype=np.int32), (B, H, Nb, Nb)).copy()
    dense_cnt = np.full((B, H, Nb), Nb, np.int32)
    n_reuse = n_refresh = 0
    for s in range(STEPS):
        for layer in range(LAYERS):
            st = steps[(s + layer) % STEPS]  # every layer sees its own sequence of inputs
            print(f"{policy}: step {s} layer {layer}", flush=True)
            out = drv.attention(layer, 0, s, gpu(st.q), gpu(st.k), gpu(st.v))
            torch.cuda.synchronize()
            got = out.float().cpu().numpy().astype(np.float64)
            o = ost[layer]
            qu, ku, vu = u16(st.q), u16(st.k), u16(st.v)
            if s < DENSE_STEPS:
                want = oracle.attn(qu, ku, vu, blk, dense_idx, dense_cnt)
                assert np.abs(got - want).max() <= ATTN_ATOL
                assert not o["has"].any() and not drv.states[(layer, 0)].has_anchor.any().item()
                continue
            qb, qm = oracle.pool(qu, blk)
            kb, km = oracle.pool(ku, blk)
            if estimator == "pooled":
                osc = oracle.scores(qb, kb)
            else:
                osc = np.stack([np.stack([antidiag_oracle.antidiag_scores(
                    st.q[b, h].double().numpy(), st.k[b, h].double().numpy(), blk, blk // 8)
                    for h in range(H)]) for b in range(B)]).astype(np.float32)
            if policy == "heart":
                _, orf = oracle.drift(qm, km, o["qa"], o["ka"], o["has"], g.delta, 0.4, 0.8)
                grf = drv.states[(layer, 0)].refresh.cpu().numpy()
                assert np.array_equal(grf, orf), f"step {s} layer {layer}: reuse decisions differ"
                assert np.array_equal(drv.states[(layer, 0)].has_anchor.cpu().numpy(), o["has"])
            else:
                orf = np.full((B, H), 1 if oracle_refreshes(policy, o["calls"]) else 0, np.uint8)
                assert drv.records[-1].kind == ("refresh" if orf.any() else "reuse")
            o["calls"] += 1
            n_refresh += int(orf.sum())
            n_reuse += int((1 - orf).sum())
            oracle.topp(osc, g.tau, refresh=orf, mask=o["mask"], kept_idx=o["idx"], kept_count=o["cnt"])
            # heads refreshed in this call: rows may differ from the oracle's only where the
            # cumulative mass passes within the estimator's score tolerance of the threshold
            # (reused heads keep masks that were checked in the call that made them)
            gm = drv.states[(layer, 0)].mask.cpu().numpy()
            fresh = orf.astype(bool)[:, :, None, None]
            shift = None
            if estimator == "pooled" and orf.any():
                shift = pooled_mean_score_shift(osc, drv.qblk, drv.kblk)
            assert_masks_equal_up_to_threshold(np.where(fresh, gm, o["mask"]), o["mask"], osc, o["cnt"], g.tau,
                                               f"{policy} step {s} layer {layer}", row_tol=shift,
                                               tol=SCORE_RTOL if estimator == "pooled" else ANTIDIAG_SCORE_RTOL)
            same = ~(gm != o["mask"]).any(-1)
            want = oracle.attn(qu, ku, vu, blk, o["idx"], o["cnt"])
            rows_same = np.repeat(same, blk, axis=2)[:, :, :N]
            assert np.abs(got - want)[rows_same].max() <= ATTN_ATOL
    # the schedule exercises both branches of every policy except "always"
    assert n_refresh > 0 and (policy == "always" or n_reuse > 0)
    summ = drv.summary()
    assert summ["sparse_calls"] == (STEPS - DENSE_STEPS) * LAYERS and summ["dense_calls"] == DENSE_STEPS * LAYERS
    assert abs(summ["refreshed_head_fraction"] - n_refresh / (n_refresh + n_reuse)) < 1e-9


def test_tmr_policy_names_are_validated():
    from paper_2605_14513_amd.tmr import TmrDriver

    for bad in ("interval", "interval:0", "warmup:x", "sometimes"):
        with pytest.raises(ValueError):
            TmrDriver._parse_policy(bad)
    assert TmrDriver._parse_policy("interval:4") == ("interval", 4)
