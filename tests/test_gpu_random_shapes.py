"""Seeded random sweeps through the C ABI against the oracle: shapes, layouts, kept lists and
flags nobody picked by hand.  Every case is deterministic (numpy PCG64 / torch generators with
fixed seeds) and is printed before it runs, so that a failure names its case."""
import numpy as np
import pytest
import torch

import oracle
from oracle import antidiag_oracle as ao
from heart_testlib import ATTN_ATOL, assert_means_close, attn_atol, np_gpu, u16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def heart():
    import paper_2605_14513_amd as pkg

    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    pkg.load_library()
    return pkg


@pytest.mark.parametrize("seed", [101, 102])
def test_attention_random_cases(heart, seed):
    rng = np.random.default_rng(seed)
    for case in range(24):
        D, blk = [(128, 128), (64, 128), (64, 64), (128, 64)][rng.integers(0, 4)]
        B, H, N = int(rng.integers(1, 3)), int(rng.integers(1, 12)), int(rng.integers(1, 1400))
        Nb = (N + blk - 1) // blk
        amp = float(rng.choice([0.3, 1.0, 1.5, 3.0]))
        pad = int(rng.choice([0, 8, 40]))
        gen = torch.Generator().manual_seed(int(rng.integers(0, 1 << 30)))
        q, k, v = ((amp * torch.randn((B, H, N, D + pad), generator=gen)).bfloat16() for _ in range(3))
        kidx = np.zeros((B, H, Nb, Nb), np.int32)
        kcnt = np.zeros((B, H, Nb), np.int32)
        for b in range(B):
            for h in range(H):
                for i in range(Nb):
                    c = [0, 1, Nb, int(rng.integers(0, Nb + 1)), min(Nb, 3)][rng.integers(0, 5)]
                    # with and without repeated entries, in any order
                    ids = rng.integers(0, Nb, size=c) if rng.random() < 0.3 else rng.permutation(Nb)[:c]
                    kidx[b, h, i, :c] = ids
                    kcnt[b, h, i] = c
        ws = "auto" if rng.random() < 0.7 else None
        print(f"attention case {seed}/{case}: B={B} H={H} N={N} D={D} block={blk} pad={pad} amp={amp} "
              f"workspace={ws}", flush=True)
        out = torch.full((B, H, N, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        heart.heart_block_sparse_attn(q.cuda()[..., :D], k.cuda()[..., :D], v.cuda()[..., :D], blk,
                                      np_gpu(kidx), np_gpu(kcnt), out=out, workspace=ws)
        torch.cuda.synchronize()
        want = oracle.attn(u16(q[..., :D].contiguous()), u16(k[..., :D].contiguous()),
                           u16(v[..., :D].contiguous()), blk, kidx, kcnt)
        got = out.float().cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        rows = np.repeat(kcnt > 0, blk, axis=2)[:, :, :N]
        assert np.all(got[~rows] == 0), "rows without kept blocks must be zero"
        if rows.any():
            # (2e-2 for outputs of unit scale, growing with the output's magnitude beyond 2)
            err = np.abs(got - want)[rows].max()
            assert err <= attn_atol(want), f"max abs err {err:.4f} > {attn_atol(want):.4f}"


@pytest.mark.parametrize("seed", [201, 202])
def test_mask_selection_random_cases(heart, seed):
    rng = np.random.default_rng(seed)
    for case in range(24):
        Nb, D, H = int(rng.integers(1, 300)), int(rng.choice([16, 32, 48, 64, 96, 128])), int(rng.integers(1, 5))
        if case % 8 == 7:
            Nb = int(rng.integers(300, 1025))
        qb = (float(rng.choice([0.5, 2.0, 6.0])) * rng.standard_normal((1, H, Nb, D))).astype(np.float32)
        kb = rng.standard_normal((1, H, Nb, D)).astype(np.float32)
        if rng.random() < 0.5:
            kb[:, :, 1::2] = kb[:, :, 0:2 * (Nb // 2):2]      # exact ties
        tau = rng.choice([0.3, 0.7, 0.9, 0.99, 1.0, 1e-8], size=H).astype(np.float32)
        kw = dict(n_always_kv=int(rng.integers(0, min(3, Nb) + 1)), n_dense_q=int(rng.integers(0, 2)),
                  min_keep=int(rng.choice([0, 1, 4, 500])))
        refresh = (rng.random((1, H)) < 0.8).astype(np.uint8)
        print(f"selection case {seed}/{case}: Nb={Nb} D={D} H={H} tau={tau.tolist()} {kw} "
              f"refresh={refresh.tolist()} workspace={bool(case % 2)}", flush=True)
        sc = torch.zeros((1, H, Nb, Nb), device="cuda")
        gm = torch.zeros((1, H, Nb, Nb), dtype=torch.uint8, device="cuda")
        gi = torch.zeros((1, H, Nb, Nb), dtype=torch.int32, device="cuda")
        gc = torch.zeros((1, H, Nb), dtype=torch.int32, device="cuda")
        # every second case with a workspace: the score stage on 8-bit slices for D = 64 / 128, and
        # exactly the plain call for every other D
        ws = None
        if case % 2:
            ws = torch.empty(heart.heart_mask_topp_workspace_bytes(1, H, Nb, D), dtype=torch.uint8, device="cuda")
        heart.heart_mask_topp(np_gpu(qb), np_gpu(kb), np_gpu(tau), refresh=np_gpu(refresh), scores_out=sc,
                              n_always_kv_blocks=kw["n_always_kv"], n_dense_q_blocks=kw["n_dense_q"],
                              min_keep=kw["min_keep"], mask=gm, kept_idx=gi, kept_count=gc, workspace=ws)
        torch.cuda.synchronize()
        s = sc.cpu().numpy()
        om, oi, oc = oracle.topp(s, tau, refresh=refresh, **kw)
        for h in range(H):
            if not refresh[0, h]:
                assert not gm[0, h].any().item() and not gc[0, h].any().item(), "reused head was written"
                continue
            assert np.array_equal(gm[0, h].cpu().numpy(), om[0, h])
            assert np.array_equal(gc[0, h].cpu().numpy(), oc[0, h])
            gin = gi[0, h].cpu().numpy()
            for i in range(Nb):
                assert np.array_equal(gin[i, :oc[0, h, i]], oi[0, h, i, :oc[0, h, i]])
            osc = oracle.scores(qb[:, h:h + 1], kb[:, h:h + 1])[0, 0]
            big = osc >= 2.0 ** -30
            if big.any():
                assert (np.abs(s[0, h] - osc)[big] / osc[big]).max() <= 1e-5


@pytest.mark.parametrize("seed", [301])
def test_pool_drift_and_estimator_random_cases(heart, seed):
    rng = np.random.default_rng(seed)
    for case in range(16):
        D, blk = [(128, 128), (64, 128), (64, 64), (128, 64)][rng.integers(0, 4)]
        B, H, N = int(rng.integers(1, 3)), int(rng.integers(1, 10)), int(rng.integers(1, 3000))
        layout = str(rng.choice(["bhnd", "bnhd", "padded"]))
        off = float(rng.choice([0.0, 0.5, 5.0]))
        gen = torch.Generator().manual_seed(int(rng.integers(0, 1 << 30)))
        print(f"pool case {seed}/{case}: B={B} H={H} N={N} D={D} block={blk} {layout} offset={off}", flush=True)

        def make():
            if layout == "bnhd":
                t = (torch.randn((B, N, H, D), generator=gen) + off).bfloat16()
                return t.permute(0, 2, 1, 3), t.cuda().permute(0, 2, 1, 3)
            if layout == "padded":
                t = (torch.randn((B, H, N, D + 16), generator=gen) + off).bfloat16()
                return t[..., :D], t.cuda()[..., :D]
            t = (torch.randn((B, H, N, D), generator=gen) + off).bfloat16()
            return t, t.cuda()

        (q, qg), (k, kg) = make(), make()
        qblk, kblk, qm, km = heart.heart_pool_qk(qg, kg, blk)
        torch.cuda.synchronize()
        oq, oqm = oracle.pool(u16(q.contiguous()), blk)
        ok, okm = oracle.pool(u16(k.contiguous()), blk)
        amax = float(max(q.float().abs().max(), k.float().abs().max()))
        assert_means_close(qblk, oq, amax, "qblk")
        assert_means_close(kblk, ok, amax, "kblk")
        assert_means_close(qm, oqm, amax, "qmean")
        assert_means_close(km, okm, amax, "kmean")
    for case in range(16):
        B, H, D = int(rng.integers(1, 4)), int(rng.integers(1, 50)), int(rng.choice([4, 16, 64, 128, 256]))
        qm = rng.standard_normal((B, H, D)).astype(np.float32)
        km = rng.standard_normal((B, H, D)).astype(np.float32)
        qa = (qm + rng.choice([0.0, 0.01, 0.1]) * rng.standard_normal((B, H, D))).astype(np.float32)
        ka = (km + rng.choice([0.0, 0.01, 0.1]) * rng.standard_normal((B, H, D))).astype(np.float32)
        has = (rng.random((B, H)) < 0.8).astype(np.uint8)
        delta = (rng.random(H) * D * 0.1).astype(np.float32)
        gate = [(0.0, 1.0), (0.4, 0.8), (0.2, 0.2)][rng.integers(0, 3)]
        print(f"drift case {seed}/{case}: B={B} H={H} D={D} gate={gate}", flush=True)
        oqa, oka, ohas = qa.copy(), ka.copy(), has.copy()
        od, orf = oracle.drift(qm, km, oqa, oka, ohas, delta, gate[0], gate[1])
        gqa, gka, ghas = np_gpu(qa), np_gpu(ka), np_gpu(has)
        gd = torch.zeros((B, H), device="cuda")
        grf = torch.zeros((B, H), dtype=torch.uint8, device="cuda")
        heart.heart_drift(np_gpu(qm), np_gpu(km), gqa, gka, ghas, np_gpu(delta), gate[0], gate[1], True, gd, grf)
        torch.cuda.synchronize()
        fin = np.isfinite(od)
        assert np.array_equal(grf.cpu().numpy(), orf)
        assert np.array_equal(gd.cpu().numpy()[fin], od[fin])
        assert np.array_equal(gqa.cpu().numpy(), oqa) and np.array_equal(gka.cpu().numpy(), oka)
        assert np.array_equal(ghas.cpu().numpy(), ohas)
    for case in range(8):
        D, blk = [(128, 128), (64, 64)][rng.integers(0, 2)]
        H, N = int(rng.integers(1, 4)), int(rng.integers(1, 6000))
        gen = torch.Generator().manual_seed(int(rng.integers(0, 1 << 30)))
        q = (2.0 * torch.randn((1, H, N, D), generator=gen)).bfloat16()
        k = (2.0 * torch.randn((1, H, N, D), generator=gen)).bfloat16()
        print(f"estimator case {seed}/{case}: H={H} N={N} D={D} block={blk}", flush=True)
        got = heart.heart_scores_antidiag(q.cuda(), k.cuda(), blk, blk // 8).cpu().numpy().astype(np.float64)
        for h in range(H):
            want = ao.antidiag_scores(q[0, h].double().numpy(), k[0, h].double().numpy(), blk, blk // 8)
            assert (np.abs(got[0, h] - want) <= 2e-3 * np.abs(want) + 1e-7).all(), f"head {h}"
