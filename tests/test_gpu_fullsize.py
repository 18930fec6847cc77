"""Parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (all heads of the workload in one call).

The oracle is cheap for pooling, drift, scores and top-p even at these sizes, so those
are compared for EVERY head and row; attention is compared on a seeded sample of 32 query
blocks per sampled head (always including block 0 and the ragged last block, and for
the HunyuanVideo-shaped config the text blocks), which the oracle computes one by one, for
both precision paths of the attention kernel.  A chained run (the GPU on its own
intermediates, two steps so that heads reuse) follows for the headline workload.
"""
import numpy as np
import pytest
import torch

import oracle
from heart_synth import make_generator
from heart_testlib import (ATTN_ATOL, OracleChain, assert_lists_equal, assert_masks_equal_up_to_threshold,
                           assert_means_close, assert_scores_close, check_attn_plan, gpu, np_gpu,
                           pooled_mean_score_shift, sample_query_blocks, u16)

pytestmark = pytest.mark.gpu

FULL = ["wan1p3b_480p", "wan14b_480p", "wan14b_720p", "hunyuan_720p"]


@pytest.fixture(scope="module")
def heart():
    import paper_2605_14513_amd as pkg

    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    pkg.load_library()
    return pkg


def attn_sample_check(name, out, st, idx, cnt, cfg, heads, qblocks, rows_ok=None, lse=None):
    """|out - oracle.attn| <= 2e-2 (and, if given, |lse - oracle's| <= 2e-2) on the sampled query
    blocks of the sampled heads; rows_ok [B,H,Nb] optionally excludes query blocks whose lists
    differ from the oracle's."""
    blk, N = cfg.block, cfg.N
    worst = 0.0
    for h in heads:
        sub = lambda x: np.ascontiguousarray(u16(x)[:, h:h + 1])
        want, wlse = oracle.attn(sub(st.q), sub(st.k), sub(st.v), blk, np.ascontiguousarray(idx[:, h:h + 1]),
                                 np.ascontiguousarray(cnt[:, h:h + 1]), qblocks=qblocks, want_lse=True)
        got = out[:, h:h + 1].float().cpu().numpy().astype(np.float64)
        glse = None if lse is None else lse[:, h:h + 1].cpu().numpy().astype(np.float64)
        for i in qblocks:
            if rows_ok is not None and not rows_ok[:, h, i].all():
                continue
            n0, n1 = i * blk, min(N, (i + 1) * blk)
            err = np.abs(got[:, :, n0:n1] - want[:, :, n0:n1]).max()
            worst = max(worst, err)
            assert err <= ATTN_ATOL, f"{name} head {h} q-block {i}: max abs err {err:.4f}"
            if glse is not None:
                lerr = np.abs(glse[:, :, n0:n1] - wlse[:, :, n0:n1]).max()
                assert lerr <= ATTN_ATOL, f"{name} head {h} q-block {i}: log-sum-exp off by {lerr:.4f}"
    return worst


@pytest.mark.parametrize("name", FULL)
def test_full_size_path_against_oracle(heart, name):
    g = make_generator(name)
    cfg = g.cfg
    B, H, N, D, Nb, blk, nt = cfg.B, cfg.H, cfg.N, cfg.D, cfg.Nb, cfg.block, cfg.n_text_blocks
    print(f"[{name}] B={B} H={H} N={N} Nb={Nb}", flush=True)
    st0, st1 = g.step(0), g.step(1)
    q0, k0, v0 = gpu(st0.q), gpu(st0.k), gpu(st0.v)

    # ---- pool: every head, every block --------------------------------------------------
    qblk, kblk, qmean, kmean = heart.heart_pool_qk(q0, k0, blk)
    torch.cuda.synchronize()
    oqb, oqm = oracle.pool(u16(st0.q), blk)
    okb, okm = oracle.pool(u16(st0.k), blk)
    amax = float(max(st0.q.float().abs().max(), st0.k.float().abs().max()))
    assert_means_close(qblk, oqb, amax, "q block means")
    assert_means_close(kblk, okb, amax, "k block means")
    assert_means_close(qmean, oqm, amax, "q token means")
    assert_means_close(kmean, okm, amax, "k token means")
    print(f"[{name}] pool ok", flush=True)

    # ---- drift over two steps on the oracle's means: bit-exact ------------------------------
    _, oqm1 = oracle.pool(u16(st1.q), blk)
    _, okm1 = oracle.pool(u16(st1.k), blk)
    oqa, oka, oha = (np.zeros((B, H, D), np.float32), np.zeros((B, H, D), np.float32),
                     np.zeros((B, H), np.uint8))
    gqa, gka, gha = np_gpu(oqa), np_gpu(oka), np_gpu(oha)
    for t, (qm, km) in enumerate(((oqm, okm), (oqm1, okm1))):
        od, orf = oracle.drift(qm, km, oqa, oka, oha, g.delta, 0.4, 0.8)
        gd, grf = heart.heart_drift(np_gpu(qm), np_gpu(km), gqa, gka, gha, np_gpu(g.delta), 0.4, 0.8)
        torch.cuda.synchronize()
        assert np.array_equal(gd.cpu().numpy().view(np.uint32), od.view(np.uint32))
        assert np.array_equal(grf.cpu().numpy(), orf)
        assert np.array_equal(gqa.cpu().numpy(), oqa) and np.array_equal(gha.cpu().numpy(), oha)
    print(f"[{name}] drift ok, refreshed at step 1: {orf.mean():.2f}", flush=True)

    # ---- scores (oracle block means in) and top-p (oracle scores in): every row ---------------
    osc = oracle.scores(oqb, okb)
    tau = g.tau  # (wan14b_720p: the stored per-head table that targets 15 % density)
    gsc = torch.empty(osc.shape, dtype=torch.float32, device="cuda")
    heart.heart_mask_topp(np_gpu(oqb), np_gpu(okb), np_gpu(tau), scores_out=gsc,
                          n_always_kv_blocks=nt, n_dense_q_blocks=nt)
    torch.cuda.synchronize()
    rel = assert_scores_close(gsc, osc, name)
    # the score stage on 8-bit slices (heart_mask_topp_ws; what the benchmark runs for long rows)
    tws = torch.empty(heart.heart_mask_topp_workspace_bytes(B, H, Nb, D), dtype=torch.uint8, device="cuda")
    gsc2 = torch.empty_like(gsc)
    heart.heart_mask_topp(np_gpu(oqb), np_gpu(okb), np_gpu(tau), scores_out=gsc2,
                          n_always_kv_blocks=nt, n_dense_q_blocks=nt, workspace=tws)
    torch.cuda.synchronize()
    rel2 = assert_scores_close(gsc2, osc, name + " (sliced)")
    print(f"[{name}] sliced score stage: max rel err {rel2:.2e}, "
          f"{int((gsc2 != gsc).sum().item())} of {gsc.numel()} scores differ in bits from the fp64 stage", flush=True)
    del tws, gsc2
    om, oi, oc = oracle.topp(osc, tau, n_always_kv=nt, n_dense_q=nt)
    gm, gi, gc = heart.heart_mask_topp(None, None, np_gpu(tau), scores_in=np_gpu(osc),
                                       n_always_kv_blocks=nt, n_dense_q_blocks=nt)
    torch.cuda.synchronize()
    assert_lists_equal(gm, gi, gc, om, oi, oc, name)
    dens = oc.sum() / (oc.size * Nb)
    print(f"[{name}] scores max rel err {rel:.2e}; masks bit-equal; density {dens:.3f}", flush=True)
    if name == "wan14b_720p":
        assert abs(dens - 0.15) < 0.005, "the stored thresholds give a global density of 15 %"

    # ---- attention on the oracle's lists: 32 sampled query blocks of 4 sampled heads ----------
    rng = np.random.default_rng(cfg.seed)
    heads = sorted(set([0, H - 1] + rng.choice(H, size=2, replace=False).tolist()))
    qblocks = sample_query_blocks(rng, Nb, nt, 32)
    for flags in (0, heart.HEART_ATTN_FOLD_SCALE):
        ws = torch.full((heart.heart_attn_workspace_bytes(q0, blk) // 4,), -1, dtype=torch.int32, device="cuda")
        lse = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
        out = heart.heart_block_sparse_attn(q0, k0, v0, blk, np_gpu(oi), np_gpu(oc), workspace=ws, flags=flags,
                                            lse=lse)
        torch.cuda.synchronize()
        check_attn_plan(ws.cpu().numpy(), oc, Nb)
        worst = attn_sample_check(name, out, st0, oi, oc, cfg, heads, qblocks, lse=lse)
        print(f"[{name}] attention (flags {flags}) ok on heads {heads}, {len(qblocks)} query blocks each, "
              f"worst err {worst:.4f}", flush=True)


@pytest.mark.parametrize("name", FULL)
def test_chained_full_size_steps_match_oracle(heart, name):
    """Every full-size workload, the GPU path on its own intermediates in the calls the benchmark
    times (pool + drift -> mask -> attention with a launch plan), steps 0 and 1 of the schedule with
    carried TMR state: decisions equal the oracle's, masks equal up to threshold rows, attention
    within tolerance on 32 sampled query blocks of 4 heads."""
    g = make_generator(name)
    cfg = g.cfg
    B, H, N, D, Nb, blk, nt = cfg.B, cfg.H, cfg.N, cfg.D, cfg.Nb, cfg.block, cfg.n_text_blocks
    dev = "cuda"
    f32 = dict(dtype=torch.float32, device=dev)
    gq, gk = torch.zeros((B, H, D), **f32), torch.zeros((B, H, D), **f32)
    gh = torch.zeros((B, H), dtype=torch.uint8, device=dev)
    gmask = torch.zeros((B, H, Nb, Nb), dtype=torch.uint8, device=dev)
    gidx = torch.zeros((B, H, Nb, Nb), dtype=torch.int32, device=dev)
    gcnt = torch.zeros((B, H, Nb), dtype=torch.int32, device=dev)
    ws = torch.empty(heart.heart_workspace_bytes(B, H, Nb, D), dtype=torch.uint8, device=dev)
    tickets = torch.zeros(heart.heart_pool_drift_workspace_bytes(B, H), dtype=torch.uint8, device=dev)
    # (as in bench.py: long rows take the score stage on 8-bit slices)
    from paper_2605_14513_amd.tmr import SLICED_SCORES_MIN_NB
    tws = None
    if Nb > SLICED_SCORES_MIN_NB:
        tws = torch.empty(heart.heart_mask_topp_workspace_bytes(B, H, Nb, D), dtype=torch.uint8, device=dev)
    chain = OracleChain(cfg, g.tau, g.delta)
    gtau, gdelta = np_gpu(g.tau), np_gpu(g.delta)
    rng = np.random.default_rng(cfg.seed + 1)
    heads = sorted(set([0, H - 1] + rng.choice(H, size=2, replace=False).tolist()))
    qblocks = sample_query_blocks(rng, Nb, nt, 32)
    for s in range(2):
        st = g.step(s)
        print(f"[{name}] chained step {s}", flush=True)
        q, k, v = gpu(st.q), gpu(st.k), gpu(st.v)
        # (the calls bench.py times: token means and drift share a launch)
        qblk, kblk, qmean, kmean, d, r = heart.heart_pool_drift(q, k, blk, gq, gk, gh, gdelta, tickets, 0.4, 0.8)
        heart.heart_mask_topp(qblk, kblk, gtau, refresh=r, n_always_kv_blocks=nt, n_dense_q_blocks=nt,
                              mask=gmask, kept_idx=gidx, kept_count=gcnt, workspace=tws)
        out = heart.heart_block_sparse_attn(q, k, v, blk, gidx, gcnt, workspace=ws)
        torch.cuda.synchronize()
        assert not tickets.any().item()
        od, orf = chain.step(st)
        assert np.array_equal(r.cpu().numpy(), orf), f"step {s}: refresh decisions differ"
        assert np.array_equal(gh.cpu().numpy(), chain.has)
        fin = np.isfinite(od)
        assert np.allclose(d.cpu().numpy()[fin], od[fin], rtol=1e-4, atol=1e-6)
        gm = gmask.cpu().numpy()
        fresh = orf.astype(bool)[:, :, None, None]
        shift = pooled_mean_score_shift(chain.scores, qblk, kblk)
        assert_masks_equal_up_to_threshold(np.where(fresh, gm, chain.mask), chain.mask, chain.scores,
                                           chain.cnt, g.tau, f"{name} step {s}", row_tol=shift)
        same = ~(gm != chain.mask).any(-1)
        worst = attn_sample_check(name, out, st, chain.idx, chain.cnt, cfg, heads, qblocks, rows_ok=same)
        print(f"[{name}] chained step {s}: refreshed {orf.mean():.2f}, {int((~same).sum())} threshold rows, "
              f"attention worst err {worst:.4f}", flush=True)
        if s == 1 and cfg.schedule == "jumps":
            assert 0.3 <= orf.mean() <= 0.7, "the schedule keeps the refreshed share inside 30-70 %"
