#!/usr/bin/env python3
"""Benchmark of the HEART sparse-attention hot path on one MI355X.

A "step" is one pass of the whole path -- heart_pool_qk -> heart_drift ->
heart_mask_topp -> heart_block_sparse_attn -- over the bf16 Q/K/V of one simulated
denoising step of the Wan2.1-14B-shaped 480P workload (B=1, H=40, D=128,
N=32760 = 21x30x52, block 128), with the inputs already resident in HBM.  The
10-step synthetic schedule is cycled; TMR state (anchors, cached masks) carries
from step to step and is cleared when the schedule wraps.

Prints ONE JSON line.  `value` is kept-block attention FLOPs per step divided by
the time of the WHOLE step (all four kernels), in TFLOP/s; per-kernel times, the
mask-refresh time (pool + drift + mask), the roofline of the dominant kernel and
the CPU oracle's rate on a bounded sample are reported beside it.
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "block_sparse_attn_wan14b_480p_hbm_traffic.txt")
PEAK_BF16_MFMA_TFLOPS = 2500.0  # MI355X dense bf16
PEAK_FP64_VALU_TFLOPS = 78.6    # MI355X fp64 vector
PEAK_HBM_GBS = 8000.0           # MI355X HBM3E


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="wan14b_480p")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fp64-scores", action="store_true",
                    help="score stage of the mask kernel on the fp64 matrix cores also for long rows "
                         "(default: 8-bit slices on the int8 matrix cores above 256 key blocks per row)")
    ap.add_argument("--no-power-probe", action="store_true",
                    help="skip the 1.5 s of untimed attention launches under which board power and clock are read")
    ap.add_argument("--gate", default="0.4,0.8", help="layer gate lo,hi (0,1 disables)")
    ap.add_argument("--unfused", action="store_true",
                    help="call heart_pool_qk and heart_drift separately (three launches) instead of "
                         "heart_pool_drift (two launches)")
    ap.add_argument("--fold-scale", action="store_true",
                    help="time the headline step with HEART_ATTN_FOLD_SCALE (softmax scale folded into "
                         "Q: one more bf16 rounding of the query, no per-logit multiply) instead of the "
                         "library's default precision; the other path is always reported beside it")
    ap.add_argument("--policy-sweep", action="store_true",
                    help="instead of the headline step: run a multi-layer, multi-step TMR schedule "
                         "(dense warm-up, then sparse steps) under each reuse policy and print one "
                         "JSON line with refresh counts and kernel times per policy")
    ap.add_argument("--ebc-demo", action="store_true",
                    help="instead of the headline step: calibrate per-head thresholds on the workload "
                         "(errors measured with the library's sparse attention on synthetic tensors) "
                         "and print one JSON line comparing them with the shared threshold 0.9")
    ap.add_argument("--estimator-demo", action="store_true",
                    help="instead of the headline step: time the antidiagonal-style importance estimator "
                         "(heart_scores_antidiag -> heart_mask_topp(scores_in)) on the workload, compare its "
                         "masks with the pooled estimator's and print one JSON line")
    ap.add_argument("--sweep-steps", type=int, default=15)
    ap.add_argument("--sweep-layers", type=int, default=2)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 1 GiB device copies (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


def kept_flops(kept_idx, kept_count, N, block, D):
    """4*D*sum over kept (i,j) of n_i*n_j, exactly, from the kept lists (torch, on GPU)."""
    import torch

    Nb = kept_count.shape[-1]
    n = torch.full((Nb,), block, dtype=torch.float64, device=kept_count.device)
    n[Nb - 1] = N - (Nb - 1) * block
    ar = torch.arange(Nb, device=kept_count.device)
    valid = ar[None, None, None, :] < kept_count[..., None]
    nj = n[kept_idx.clamp(0, Nb - 1).long()] * valid
    per_row = nj.sum(-1) * n[None, None, :]
    return float(4.0 * D * per_row.sum().item())


def attn_profile(workload):
    """Figures of the attention kernel from the committed rocprofv3 --pmc summary: HBM bytes
    per launch (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy of known size) and the
    matrix-pipe, LDS and L2 counters.  Empty when the summary covers another workload."""
    try:
        t = {}
        with open(TRAFFIC_FILE) as f:
            for line in f:
                if ":" in line and not line.startswith("#"):
                    key, val = line.split(":", 1)
                    t[key.strip()] = val.strip()
        if t.get("workload") != workload:
            return {}
        out = {"traffic": float(t["fetch_bytes_per_launch"]) + float(t["write_bytes_per_launch"])}
        for key, name in (("mfma_util_percent", "mfma_pipe_busy_frac"), ("lds_util_percent", "lds_busy_frac"),
                          ("l2_hit_rate_percent", "l2_hit_rate")):
            if key in t:
                out[name] = round(float(t[key]) / 100.0, 3)
        return out
    except (OSError, ValueError, KeyError):
        return {}


def measured_ceilings(heart, torch, q0, k0):
    """What the chip sustains, measured live: MFMA-only loop on zero operands (nominal clock)
    and on operands taken from the workload's own Q and K (the chip is power limited and clocks
    down on real data), a read-only stream over 1 GiB with the pooling kernel's access pattern
    (what a streaming read sustains), and a plain 1 GiB copy (read + write; the reference for
    scaling the traffic counters, not a ceiling for a read-only kernel)."""
    dev = q0.device
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    zeros = torch.zeros(8192, dtype=torch.bfloat16, device=dev)
    a = k0.reshape(-1)[:8192].contiguous()
    b = q0.reshape(-1)[:8192].contiguous()
    out = {}
    for tag, (x, y) in (("zero_operands", (zeros, zeros)), ("workload_operands", (a, b))):
        best = 0.0
        for rep in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fl = heart.heart_ubench_mfma_bf16(x, y, 512, 20000, sink)
            e1.record()
            torch.cuda.synchronize()
            if rep:  # first repetition warms up
                best = max(best, fl / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        out[tag] = best
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    best = 0.0
    for rep in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        nb = heart.heart_ubench_copy(src, dst)
        e1.record()
        torch.cuda.synchronize()
        if rep:
            best = max(best, nb / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    out["hbm_copy_gbs"] = best
    best = 0.0
    isink = torch.zeros(1, dtype=torch.int32, device=dev)
    for rep in range(4):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        nb = heart.heart_ubench_read(src, isink)
        e1.record()
        torch.cuda.synchronize()
        if rep:
            best = max(best, nb / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    out["hbm_read_gbs"] = best
    del src, dst
    return out


def power_probe(torch, launch, seconds=1.5):
    """Board power and shader clock while `launch` (one attention call) is repeated for about
    `seconds`: read from the amdgpu driver's sysfs files of the one GPU of the box (hwmon power
    sensor and cap in microwatts, current level of pp_dpm_sclk), sampled from the host every
    0.1 s while the queued launches run; the first 0.7 s (the sensor's settling time) are dropped.
    Extra information, outside every timed region; None where the files cannot be read."""
    import numpy as np

    def first_readable(patterns):
        for pat in patterns:
            for path in sorted(glob.glob(pat)):
                try:
                    with open(path) as f:
                        f.read()
                    return path
                except OSError:
                    pass
        return None
    hw = "/sys/class/drm/card*/device/hwmon/hwmon*/"
    p_power = first_readable([hw + "power1_average", hw + "power1_input"])
    p_cap = first_readable([hw + "power1_cap"])
    p_sclk = first_readable(["/sys/class/drm/card*/device/pp_dpm_sclk"])
    if p_power is None:
        return None
    def read(path):
        with open(path) as f:
            return f.read()
    try:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        launch()
        e1.record()
        torch.cuda.synchronize()
        n = max(1, int(seconds / (e0.elapsed_time(e1) * 1e-3)))
        idle_w = int(read(p_power)) / 1e6
        t0 = time.perf_counter()
        for _ in range(n):
            launch()
        watts, mhz = [], []
        while not torch.cuda.current_stream().query() and time.perf_counter() - t0 < 4 * seconds:
            if time.perf_counter() - t0 >= 0.7:
                watts.append(int(read(p_power)) / 1e6)
                if p_sclk:
                    cur = [ln for ln in read(p_sclk).splitlines() if ln.rstrip().endswith("*")]
                    if cur:
                        mhz.append(float(cur[0].split(":")[1].lower().replace("mhz", "").replace("*", "")))
            time.sleep(0.1)
        torch.cuda.synchronize()
        if not watts:
            return None
        return {"launches": n, "seconds": time.perf_counter() - t0,
                "board_power_w": float(np.mean(watts)), "board_power_w_max": float(np.max(watts)),
                "board_power_cap_w": int(read(p_cap)) / 1e6 if p_cap else None,
                "board_power_before_w": idle_w,
                "shader_clock_mhz": float(np.mean(mhz)) if mhz else None,
                "samples": len(watts), "source": "amdgpu sysfs (hwmon power sensor, pp_dpm_sclk)"}
    except (OSError, ValueError, IndexError) as e:
        print(f"[bench] power probe skipped: {e}", file=sys.stderr, flush=True)
        return None


def policy_sweep(args, heart, torch, g, steps_in, tau, delta):
    """Structure of the paper's reuse-policy ablation on synthetic inputs: refresh counts and
    time per policy over L layers x 2 guidance branches x S denoising steps (the first 5 dense).
    Quality metrics are out of reach here (they need the models); this reports cost only."""
    from paper_2605_14513_amd.tmr import TmrConfig, TmrDriver

    cfg = g.cfg
    S = len(steps_in)
    res = []
    # the four policies of the ablation, then the drift-threshold sweep: the paper sweeps
    # delta over {0, 10, 30, 100} with 30 its operating point; here the same ratios to the
    # synthetic operating point (delta = 0 refreshes every head whose features moved at all)
    variants = [("always", "always", 1.0, "pooled"), ("heart", "heart", 1.0, "pooled"),
                ("interval:4", "interval:4", 1.0, "pooled"), ("warmup:5", "warmup:5", 1.0, "pooled"),
                ("heart, delta x 0", "heart", 0.0, "pooled"), ("heart, delta x 1/3", "heart", 1.0 / 3.0, "pooled"),
                ("heart, delta x 10/3", "heart", 10.0 / 3.0, "pooled"),
                # the same with the antidiagonal-style estimator, whose cost a reused mask also saves
                ("always, antidiag estimator", "always", 1.0, "antidiag"),
                ("heart, antidiag estimator", "heart", 1.0, "antidiag"),
                ("interval:4, antidiag estimator", "interval:4", 1.0, "antidiag")]
    for label, policy, dscale, estimator in variants:
        drv = TmrDriver(TmrConfig(B=cfg.B, H=cfg.H, N=cfg.N, D=cfg.D, block=cfg.block, tau=tau,
                                  delta=delta * dscale, policy=policy, estimator=estimator, dense_steps=5,
                                  n_always_kv_blocks=cfg.n_text_blocks,
                                  n_dense_q_blocks=cfg.n_text_blocks),
                        n_layers=args.sweep_layers, n_branches=2, record=True, time_kernels=True)
        out = torch.empty_like(steps_in[0][0])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(args.sweep_steps):
            for layer in range(args.sweep_layers):
                for br in range(2):
                    q, k, v = steps_in[(s + layer + 3 * br) % S]
                    drv.attention(layer, br, s, q, k, v, out=out)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        summ = drv.summary()
        summ["policy"] = label
        summ["wall_ms_per_call"] = wall * 1e3 / summ["calls"]
        res.append(summ)
        print(f"[bench] policy {label}: {summ}", file=sys.stderr, flush=True)
        del drv
    return {"metric": "TMR policy sweep (cost only), " + cfg.name, "layers": args.sweep_layers,
            "branches": 2, "steps": args.sweep_steps, "dense_steps": 5, "policies": res,
            "data": "synthetic"}


def ebc_demo(args, heart, torch, g, steps_in):
    """Error-guided Budgeted Calibration on synthetic tensors: the attention output of a head
    stands in for the denoising velocity (the models are not available), the candidates are
    shared thresholds, the budget is the sparsity of the shared threshold 0.9."""
    import numpy as np

    cfg = g.cfg
    B, H, N, D, Nb, blk, nt = cfg.B, cfg.H, cfg.N, cfg.D, cfg.Nb, cfg.block, cfg.n_text_blocks
    T, Yg, Xg = cfg.grid
    q, k, v = steps_in[0]
    qblk, kblk, _, _ = heart.heart_pool_qk(q, k, blk)
    cands = [0.6, 0.7, 0.8, 0.85, 0.9, 0.95, 0.98, 1.0]
    ones = torch.ones(H, device=q.device)
    _, didx, dcnt = heart.heart_mask_topp(qblk, kblk, ones, n_always_kv_blocks=nt, n_dense_q_blocks=nt)
    dense = heart.heart_block_sparse_attn(q, k, v, blk, didx, dcnt)
    n_grid = T * Yg * Xg

    def as_field(x, h):  # [B, N, D] of head h -> [B*D, T, Y, X] over the video tokens
        return x[:, h, N - n_grid:].float().permute(0, 2, 1).reshape(B * D, T, Yg, Xg).contiguous()

    E = np.zeros((H, len(cands))); S = np.zeros((H, len(cands)))
    ws = torch.empty(heart.heart_ebc_workspace_bytes(B * D, T, Yg, Xg), dtype=torch.uint8, device=q.device)
    dens = [as_field(dense, h) for h in range(H)]
    ev = []
    for ci, tc in enumerate(cands):
        tau = torch.full((H,), tc, device=q.device)
        _, idx, cnt = heart.heart_mask_topp(qblk, kblk, tau, n_always_kv_blocks=nt, n_dense_q_blocks=nt)
        out = heart.heart_block_sparse_attn(q, k, v, blk, idx, cnt)
        cnt_h = cnt.float().sum(dim=(0, 2)).cpu().numpy()
        for h in range(H):
            err = as_field(out, h) - dens[h]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            r = heart.heart_ebc_band_error(err, dens[h], workspace=ws)
            e1.record()
            ev.append((e0, e1))
            E[h, ci] = r[0].item()
            S[h, ci] = 1.0 - cnt_h[h] / (B * Nb * Nb)
    torch.cuda.synchronize()
    shared = cands.index(0.9)
    budget = float(S[:, shared].mean())
    t0 = time.perf_counter()
    choice, total = heart.heart_ebc_select(E, S, budget)
    t_sel = time.perf_counter() - t0
    # the same solver at the size of a full model: 40 layers x 40 heads, tables tiled with noise
    rng = np.random.default_rng(0)
    reps = max(1, 1600 // H)
    Eb = np.tile(E, (reps, 1)) * rng.uniform(0.5, 2.0, size=(reps * H, 1))
    Sb = np.tile(S, (reps, 1))
    t0 = time.perf_counter()
    _, total_big = heart.heart_ebc_select(Eb, Sb, budget)
    t_big = time.perf_counter() - t0
    return {
        "metric": "EBC on synthetic tensors, " + cfg.name, "data": "synthetic",
        "candidates": cands, "budget_mean_sparsity": budget,
        "shared_threshold_error": float(E[:, shared].sum()), "calibrated_error": total,
        "calibrated_thresholds": [cands[c] for c in choice],
        "calibrated_mean_sparsity": float(S[np.arange(H), choice].mean()),
        "band_error_us_per_call": float(np.median([a.elapsed_time(b) for a, b in ev]) * 1e3),
        "band_error_tensor": [B * D, T, Yg, Xg],
        "select_ms": t_sel * 1e3, "select_ms_at_1600_heads": t_big * 1e3,
        "shared_vs_calibrated_error_at_1600_heads": [float(Eb[:, shared].sum()), total_big],
    }


def estimator_demo(args, heart, torch, g, steps_in, tau):
    """The alternative importance estimator behind heart_mask_topp's scores_in: time of its two
    kernels, its matrix-core rate, and how its masks compare with the pooled estimator's."""
    cfg = g.cfg
    B, H, N, D, Nb, blk, nt = cfg.B, cfg.H, cfg.N, cfg.D, cfg.Nb, cfg.block, cfg.n_text_blocks
    stride = blk // 8
    q, k, v = steps_in[0]
    ws = torch.empty(heart.heart_scores_antidiag_workspace_bytes(q, blk, stride), dtype=torch.uint8, device=q.device)
    sc = torch.empty((B, H, Nb, Nb), dtype=torch.float32, device=q.device)
    K, W = max(1, args.steps), max(1, args.warmup)
    for _ in range(W):
        heart.heart_scores_antidiag(q, k, blk, stride, scores=sc, workspace=ws)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    torch.cuda.synchronize()
    ev[0].record()
    for i in range(K):
        heart.heart_scores_antidiag(*steps_in[i % len(steps_in)][:2], blk, stride, scores=sc, workspace=ws)
        ev[i + 1].record()
    torch.cuda.synchronize()
    ms = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(K))
    M = (N + stride - 1) // stride
    flops = 2.0 * M * M * stride * D * B * H
    heart.heart_scores_antidiag(q, k, blk, stride, scores=sc, workspace=ws)
    m1, i1, c1 = heart.heart_mask_topp(None, None, tau, scores_in=sc, n_always_kv_blocks=nt, n_dense_q_blocks=nt)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    heart.heart_mask_topp(None, None, tau, scores_in=sc, n_always_kv_blocks=nt, n_dense_q_blocks=nt,
                          mask=m1, kept_idx=i1, kept_count=c1)
    e1.record()
    qblk, kblk, _, _ = heart.heart_pool_qk(q, k, blk)
    m0, i0, c0 = heart.heart_mask_topp(qblk, kblk, tau, n_always_kv_blocks=nt, n_dense_q_blocks=nt)
    torch.cuda.synchronize()
    inter = (m0 & m1).sum(dim=(2, 3)).float()
    union = (m0 | m1).sum(dim=(2, 3)).float()
    mean_ms = sum(ms) / len(ms)
    return {
        "metric": "antidiagonal-style importance estimator, " + cfg.name, "data": "synthetic",
        "stride": stride, "block": blk, "reduced_rows": M, "steps": K, "warmup": W,
        "scores_ms": mean_ms, "scores_ms_min": ms[0],
        "scores_tflops_bf16": flops / (mean_ms * 1e-3) / 1e12,
        "roofline": {"kernel": "antidiag_tile_kernel + antidiag_combine_kernel", "bound": "mfma",
                     "achieved": flops / (mean_ms * 1e-3) / 1e12, "peak": PEAK_BF16_MFMA_TFLOPS,
                     "unit": "TFLOP/s", "frac": flops / (mean_ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS},
        "workspace_mb": ws.numel() / 1e6,
        "select_from_scores_us": e0.elapsed_time(e1) * 1e3,
        "kept_block_density": {"pooled": float(m0.float().mean().item()), "antidiag": float(m1.float().mean().item())},
        "mask_iou_with_pooled_estimator_per_head": [round(float(x), 3) for x in (inter / union).flatten().cpu().tolist()],
    }


def cpu_baseline(name, tau_all, delta_all):
    """Oracle timed on host cores on a bounded sample of the same workload."""
    import numpy as np

    import oracle
    from heart_synth import HeartInputGenerator, as_u16, get_config

    cfg = get_config(name)
    heads = sorted(set(np.linspace(0, cfg.H - 1, num=min(8, cfg.H)).astype(int).tolist()))
    g = HeartInputGenerator(cfg, heads=heads)
    st = g.step(0)
    q, k, v = as_u16(st.q), as_u16(st.k), as_u16(st.v)
    nh = len(heads)
    t0 = time.perf_counter()
    qb, qm = oracle.pool(q, cfg.block)
    kb, km = oracle.pool(k, cfg.block)
    qa = np.zeros_like(qm); ka = np.zeros_like(km); has = np.zeros((cfg.B, nh), np.uint8)
    oracle.drift(qm, km, qa, ka, has, delta_all[heads], 0.4, 0.8)
    sc = oracle.scores(qb, kb)
    nt = cfg.n_text_blocks
    m, idx, cnt = oracle.topp(sc, tau_all[heads], n_always_kv=nt, n_dense_q=nt)
    t_mask = time.perf_counter() - t0
    # attention on a sample of query blocks per head, sized for roughly 10-20 s of CPU work
    rng = np.random.default_rng(0)
    nq = min(128, cfg.Nb)
    qblocks = sorted(set([0, cfg.Nb - 1] + rng.choice(cfg.Nb, size=nq, replace=False).tolist()))
    t0 = time.perf_counter()
    oracle.attn(q, k, v, cfg.block, idx, cnt, qblocks=qblocks)
    t_attn = time.perf_counter() - t0
    n = np.full(cfg.Nb, cfg.block, np.float64)
    n[-1] = cfg.N - (cfg.Nb - 1) * cfg.block
    fl = 0.0
    for b in range(cfg.B):
        for h in range(nh):
            for i in qblocks:
                fl += 4.0 * cfg.D * n[i] * n[idx[b, h, i, :cnt[b, h, i]]].sum()
    return {
        # whole step like `value`: the sample's share of the pooling/drift/mask time is included
        "value": fl / (t_attn + t_mask * len(qblocks) / cfg.Nb) / 1e12,
        "unit": "TFLOP/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": (f"step 0 of {name}, heads {heads}: pool+drift+scores+top-p in full for these "
                   f"heads, sparse attention on query blocks {qblocks} of each; value = kept-block "
                   f"attention FLOPs of the sample / (oracle attention time + the sampled share of "
                   f"its pool/drift/mask time)"),
        "attn_seconds_on_sample": t_attn,
        "mask_refresh_us_per_step_extrapolated": t_mask * 1e6 * cfg.H / nh,
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one MI355X per box; no collectives, no "
              f"sharding). --gpus {args.gpus} is not supported; run with --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2605_14513_amd as heart
    from heart_synth import make_generator

    if not os.path.exists(heart.lib_path()):
        from paper_2605_14513_amd import build as hb

        hb.build(force=True)
    heart.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    gate_lo, gate_hi = (float(x) for x in args.gate.split(","))

    t_setup = time.perf_counter()
    g = make_generator(args.workload)
    cfg = g.cfg
    B, H, N, D, Nb, blk = cfg.B, cfg.H, cfg.N, cfg.D, cfg.Nb, cfg.block
    nt = cfg.n_text_blocks
    S = cfg.steps
    steps_in = []
    for s in range(S):
        st = g.step(s)
        steps_in.append((st.q.to(dev), st.k.to(dev), st.v.to(dev)))
        print(f"[bench] generated step {s + 1}/{S}", file=sys.stderr, flush=True)
    tau = torch.from_numpy(g.tau).to(dev)
    delta = torch.from_numpy(g.delta).to(dev)
    del st
    print(f"[bench] inputs resident after {time.perf_counter() - t_setup:.1f} s", file=sys.stderr,
          flush=True)

    if args.policy_sweep:
        print(json.dumps(policy_sweep(args, heart, torch, g, steps_in, tau, delta)))
        return
    if args.ebc_demo:
        print(json.dumps(ebc_demo(args, heart, torch, g, steps_in)))
        return
    if args.estimator_demo:
        print(json.dumps(estimator_demo(args, heart, torch, g, steps_in, tau)))
        return

    f32 = dict(dtype=torch.float32, device=dev)
    qblk = torch.empty((B, H, Nb, D), **f32); kblk = torch.empty((B, H, Nb, D), **f32)
    qmean = torch.empty((B, H, D), **f32); kmean = torch.empty((B, H, D), **f32)
    qa = torch.zeros((B, H, D), **f32); ka = torch.zeros((B, H, D), **f32)
    has = torch.zeros((B, H), dtype=torch.uint8, device=dev)
    drift = torch.empty((B, H), **f32)
    refresh = torch.empty((B, H), dtype=torch.uint8, device=dev)
    mask = torch.zeros((B, H, Nb, Nb), dtype=torch.uint8, device=dev)
    kidx = torch.zeros((B, H, Nb, Nb), dtype=torch.int32, device=dev)
    kcnt = torch.zeros((B, H, Nb), dtype=torch.int32, device=dev)
    out = torch.empty_like(steps_in[0][0])
    attn_ws = torch.empty(heart.heart_workspace_bytes(B, H, Nb, D), dtype=torch.uint8, device=dev)
    tickets = torch.zeros(heart.heart_pool_drift_workspace_bytes(B, H), dtype=torch.uint8, device=dev)
    # heart_mask_topp_ws (score stage on 8-bit slices: one launch more, pays for long rows)
    from paper_2605_14513_amd.tmr import SLICED_SCORES_MIN_NB
    topp_ws = None
    if Nb > SLICED_SCORES_MIN_NB and not args.fp64_scores:
        topp_ws = torch.empty(heart.heart_mask_topp_workspace_bytes(B, H, Nb, D), dtype=torch.uint8, device=dev)
    flags_main = heart.HEART_ATTN_FOLD_SCALE if args.fold_scale else 0
    flags_other = 0 if args.fold_scale else heart.HEART_ATTN_FOLD_SCALE
    path_name = {0: "fp32_scale (default)", heart.HEART_ATTN_FOLD_SCALE: "fold_scale"}
    gate = [gate_lo, gate_hi]

    def one_step(it, ev=None, inner=False, flags=flags_main):
        """ev: five events; [0], [3], [4] bracket the mask-refresh side and the attention call,
        [1] and [2] (between pool, drift and mask) are only recorded when `inner` is set: every
        event record costs a few microseconds of gap between two kernels."""
        s = it % S
        q, k, v = steps_in[s]
        if s == 0:
            has.zero_()  # schedule wraps: no cached anchors
        if ev: ev[0].record()
        if args.unfused:
            heart.heart_pool_qk(q, k, blk, qblk, kblk, qmean, kmean)
            if ev and inner: ev[1].record()
            heart.heart_drift(qmean, kmean, qa, ka, has, delta, gate[0], gate[1], True, drift, refresh)
        else:  # pooling pass, then token means + drift + reuse rule + gate in one launch
            heart.heart_pool_drift(q, k, blk, qa, ka, has, delta, tickets, gate[0], gate[1], True,
                                   qblk, kblk, qmean, kmean, drift, refresh)
            if ev and inner: ev[1].record()
        if ev and inner: ev[2].record()
        heart.heart_mask_topp(qblk, kblk, tau, refresh=refresh, n_always_kv_blocks=nt,
                              n_dense_q_blocks=nt, mask=mask, kept_idx=kidx, kept_count=kcnt,
                              workspace=topp_ws)
        if ev: ev[3].record()
        heart.heart_block_sparse_attn(q, k, v, blk, kidx, kcnt, out=out, workspace=attn_ws, flags=flags)
        if ev: ev[4].record()

    K, W = args.steps, args.warmup

    def timed_schedule():
        """W warm-up steps, then exactly K timed steps with HIP events on the launch stream around
        the mask-refresh side (pool + drift + mask as one interval) and around the attention call;
        then the same K steps once more, untimed, with events between pool, drift and mask too
        (the split of the mask-refresh side; each of the three figures includes its event gap)."""
        has.zero_()
        for it in range(W):
            one_step(it)
        torch.cuda.synchronize()
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(K)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for it in range(K):
            one_step(it, events[it])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        r = {"ms_per_step": (t1 - t0) * 1e3 / K,
             "refresh_ms": float(np.mean([events[i][0].elapsed_time(events[i][3]) for i in range(K)])),
             "attn_ms": float(np.mean([events[i][3].elapsed_time(events[i][4]) for i in range(K)]))}
        events2 = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(K)]
        for it in range(K):
            one_step(it, events2[it], inner=True)
        torch.cuda.synchronize()
        r["per"] = np.array([[events2[i][j].elapsed_time(events2[i][j + 1]) for j in range(3)]
                             for i in range(K)])  # ms: pool, drift, mask per step
        return r

    def replay_stats():
        """Untimed replay of the same K steps: kept-block FLOPs, density, refresh ratio, mask IoU."""
        has.zero_(); kcnt.zero_()
        flops, dens, refr, ious = [], [], [], []
        dens_head = torch.zeros(H, device=dev)
        prev_mask = None
        for it in range(K):
            one_step(it)
            torch.cuda.synchronize()
            flops.append(kept_flops(kidx, kcnt, N, blk, D))
            dens.append(float(kcnt.sum().item()) / (B * H * Nb * Nb))
            dens_head += kcnt.float().sum(dim=(0, 2)) / (B * Nb * Nb)
            refr.append(float(refresh.float().mean().item()))
            if prev_mask is not None and it % S != 0:
                inter = (mask & prev_mask).sum().item()
                union = (mask | prev_mask).sum().item()
                ious.append(inter / max(1, union))
            prev_mask = mask.clone()
        return flops, dens, refr, ious, dens_head

    # ---- headline: the gate as given on the command line (default 0.4 / 0.8) ----
    tm = timed_schedule()
    ms_per_step, refresh_ms, attn_ms, per = tm["ms_per_step"], tm["refresh_ms"], tm["attn_ms"], tm["per"]
    pool_ms, drift_ms, mask_ms = per.mean(0)
    flops, dens, refr, ious, dens_head = replay_stats()

    # ---- the other precision path of the attention kernel on the lists of the last step ----
    for _ in range(2):
        heart.heart_block_sparse_attn(*steps_in[(K - 1) % S], blk, kidx, kcnt, out=out, workspace=attn_ws,
                                      flags=flags_other)
    ev_o = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    ev_o[0].record()
    for i in range(K):
        heart.heart_block_sparse_attn(*steps_in[(K - 1) % S], blk, kidx, kcnt, out=out, workspace=attn_ws,
                                      flags=flags_other)
        ev_o[i + 1].record()
    torch.cuda.synchronize()
    other_ms = float(np.mean([ev_o[i].elapsed_time(ev_o[i + 1]) for i in range(K)]))
    other_tflops = flops[-1] / (other_ms * 1e-3) / 1e12

    # ---- board power and clock under the attention kernel (default path, same lists) ----
    power = None
    if not args.no_power_probe:
        power = power_probe(torch, lambda: heart.heart_block_sparse_attn(
            *steps_in[(K - 1) % S], blk, kidx, kcnt, out=out, workspace=attn_ws, flags=flags_main))

    # ---- the same schedule with the layer gate off (0 / 1), for the headline workload ----
    gate_off = None
    if (gate_lo, gate_hi) != (0.0, 1.0):
        gate[:] = [0.0, 1.0]
        tg = timed_schedule()
        fl_g, dens_g, refr_g, _, _ = replay_stats()
        gate[:] = [gate_lo, gate_hi]
        gate_off = {"ms_per_step": tg["ms_per_step"], "mask_refresh_us_per_step": tg["refresh_ms"] * 1e3,
                    "kernels_us": {"pool_qk": float(tg["per"][:, 0].mean() * 1e3),
                                   "drift": float(tg["per"][:, 1].mean() * 1e3),
                                   "mask_topp": float(tg["per"][:, 2].mean() * 1e3),
                                   "block_sparse_attn": tg["attn_ms"] * 1e3},
                    "value": float(np.mean(fl_g)) / (tg["ms_per_step"] * 1e-3) / 1e12,
                    "refreshed_head_fraction_per_step": [round(x, 3) for x in refr_g],
                    "kept_block_density": float(np.mean(dens_g))}

    # ---- launch overhead: schedule step 1 repeated K times, eagerly and as one HIP graph ----
    # (extra information; `value` comes from the eager region above.  After the first
    # repetition nothing drifts any more, so these steps are pool + drift + attention.)
    launch = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            one_step(1)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        t0e = time.perf_counter()
        for _ in range(K):
            one_step(1)
        torch.cuda.synchronize()
        eager_rep_ms = (time.perf_counter() - t0e) * 1e3 / K
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            one_step(1)
        torch.cuda.synchronize()
        t0g = time.perf_counter()
        for _ in range(K):
            gr.replay()
        torch.cuda.synchronize()
        launch = {"repeated_step_eager_ms": eager_rep_ms,
                  "repeated_step_hip_graph_ms": (time.perf_counter() - t0g) * 1e3 / K}
        del gr
    except Exception as e:  # optional figure
        print(f"[bench] HIP graph timing skipped: {e}", file=sys.stderr, flush=True)

    flops_per_step = float(np.mean(flops))
    dense_flops = 4.0 * N * N * D * H * B

    value = flops_per_step / (ms_per_step * 1e-3) / 1e12
    attn_tflops = flops_per_step / (attn_ms * 1e-3) / 1e12
    pool_bytes = 2 * B * H * N * D * 2 + 2 * B * H * (Nb + 1) * D * 4
    refreshed = float(np.mean(refr))
    mask_bytes = refreshed * B * H * (2 * Nb * D * 4 + Nb * Nb * (1 + 4))

    ceil = measured_ceilings(heart, torch, steps_in[0][0], steps_in[0][1])
    prof = attn_profile(args.workload)
    mask_f64_flops = refreshed * B * H * 2.0 * Nb * Nb * D  # fp64 dot products of the score stage
    # the mask kernel only works on steps where some head refreshes: its time on those steps,
    # and per refreshed head (per-step figures come from the untimed, event-split repetition)
    refr_steps = np.array(refr)
    mask_us_steps = per[:, 2] * 1e3
    busy = refr_steps > 0
    mask_detail = {
        "us_per_refreshing_step": float(mask_us_steps[busy].mean()) if busy.any() else None,
        "us_per_step_without_refresh": float(mask_us_steps[~busy].mean()) if (~busy).any() else None,
        "us_per_refreshed_head": (float(mask_us_steps[busy].sum() / (refr_steps[busy].sum() * B * H))
                                  if busy.any() else None),
        "refreshing_steps": int(busy.sum()),
    }
    refresh_bytes = pool_bytes + 4 * B * H * D * 4 + mask_bytes  # pool + drift + mask, algorithmic

    result = {
        "metric": "sparse-attn effective TFLOP/s + mask-refresh us/step, Wan-14B 480P shape, 1 GPU",
        "value": value,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{cfg.name}: B={B} H={H} D={D} N={N} grid={'x'.join(map(str, cfg.grid))} "
                        f"block={blk}, {S}-step synthetic TMR schedule, gate {gate_lo}/{gate_hi}",
            "attention_precision_path": path_name[flags_main],
            "value_definition": "kept-block attention FLOPs (4*D*sum n_i*n_j over kept blocks) per "
                                "step / wall time of the whole step (pool+drift+mask+attention)",
        },
        "mask_refresh_us_per_step": refresh_ms * 1e3,
        "launch_overhead": launch,
        # (heart_pool_drift: "pool_qk" covers its two launches and "drift" is only an event gap)
        "token_means_and_drift_share_a_launch": not args.unfused,
        "mask_score_stage": "int8 slices (heart_mask_topp_ws)" if topp_ws is not None else "fp64",
        "kernels_us": {"pool_qk": pool_ms * 1e3, "drift": drift_ms * 1e3,
                       "mask_topp": mask_ms * 1e3, "block_sparse_attn": attn_ms * 1e3},
        "attn_kept_tflops": attn_tflops,
        "attn_kept_tflops_other_path": {"path": path_name[flags_other], "tflops": other_tflops,
                                        "us": other_ms * 1e3,
                                        "note": "same lists (last timed step), K back-to-back launches"},
        "mask_topp_detail": mask_detail,
        "mask_refresh_side": {"bound": "hbm", "algorithmic_bytes": refresh_bytes,
                              "achieved": refresh_bytes / (refresh_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                              "unit": "GB/s", "frac": refresh_bytes / (refresh_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
        "gate_off": gate_off,
        "attn_dense_equiv_tflops": dense_flops / (attn_ms * 1e-3) / 1e12,
        "kept_block_density": float(np.mean(dens)),
        "kept_block_density_per_head": [round(float(x), 4) for x in (dens_head / K).cpu().tolist()],
        "refreshed_head_fraction": refreshed,
        "refreshed_head_fraction_per_step": [round(x, 3) for x in refr],
        "mask_iou_between_consecutive_steps": [round(x, 4) for x in ious],
        "roofline": {
            "kernel": "heart_block_sparse_attn",
            "bound": "mfma",
            "achieved": attn_tflops,
            "peak": PEAK_BF16_MFMA_TFLOPS,
            "unit": "TFLOP/s",
            "frac": attn_tflops / PEAK_BF16_MFMA_TFLOPS,
            "traffic": prof.get("traffic"),
            "profiled_counters": {k_: v_ for k_, v_ in prof.items() if k_ != "traffic"} or None,
            # the same kernel against what the matrix cores sustain on this chip, measured in
            # this run by an MFMA-only loop (the clock drops on real data: power limit)
            "measured_mfma_only_tflops": {"zero_operands": ceil["zero_operands"],
                                          "workload_operands": ceil["workload_operands"]},
            "frac_of_measured_workload_operands": attn_tflops / ceil["workload_operands"],
            # board power against its cap and the shader clock while this kernel runs back to
            # back (the published peak is quoted at 2.4 GHz)
            "power_probe": power,
        },
        "roofline_hbm_kernels": {
            "heart_pool_qk": {"bound": "hbm", "achieved": pool_bytes / (pool_ms * 1e-3) / 1e9,
                              "peak": PEAK_HBM_GBS, "unit": "GB/s",
                              "frac": pool_bytes / (pool_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
            "heart_mask_topp": {"bound": "hbm", "achieved": mask_bytes / (mask_ms * 1e-3) / 1e9,
                                "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                "frac": mask_bytes / (mask_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                "note": "bound by its fp64 score stage and per-row search, not by HBM",
                                "alu_fp64": {"bound": "alu", "achieved": mask_f64_flops / (mask_ms * 1e-3) / 1e12,
                                             "peak": PEAK_FP64_VALU_TFLOPS, "unit": "TFLOP/s",
                                             "frac": mask_f64_flops / (mask_ms * 1e-3) / 1e12 / PEAK_FP64_VALU_TFLOPS}},
            # what a read-only stream with the pooling kernel's access pattern sustains (its
            # measured ceiling), and a plain copy (read + write: the counter-scaling reference)
            "measured_stream_read_gbs": ceil["hbm_read_gbs"],
            "measured_copy_gbs": ceil["hbm_copy_gbs"],
        },
    }
    if args.calibrate_copy:
        src = torch.empty(256 * 1024 * 1024, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline:
        print("[bench] timing the CPU oracle on a bounded sample", file=sys.stderr, flush=True)
        result["cpu_baseline"] = cpu_baseline(args.workload, g.tau, g.delta)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
