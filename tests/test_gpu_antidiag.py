"""GPU parity of heart_scores_antidiag (the antidiagonal-style importance estimator behind
heart_mask_topp's scores_in) against oracle/antidiag_oracle.py, through the C ABI.

Tolerance: inputs are the same bf16 values on both sides and bf16 products are exact in fp32,
so the GPU's error is the fp32 accumulation of S*D <= 2048 products (relative to the sum of
magnitudes about 2048 * 2^-24 ~ 1e-4 in the worst case, typically 1e-6) plus fp32 exponentials;
a logit error e changes a score by a relative e.  The bound used is 2e-3 relative + 1e-7
absolute.  Selection from these scores is the existing scores_in path and is checked bit for
bit given the GPU's scores.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import antidiag_oracle as ao
from heart_synth import make_generator
from heart_testlib import assert_lists_equal, np_gpu

pytestmark = pytest.mark.gpu

RTOL, ATOL = 2e-3, 1e-7


@pytest.fixture(scope="module")
def heart():
    import paper_2605_14513_amd as pkg

    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    pkg.load_library()
    return pkg


def oracle_scores(q, k, block, stride, heads=None):
    """q, k: CPU bf16 [B,H,N,D]; returns {(b,h): [Nb,Nb]} for the listed heads (default all)."""
    B, H = q.shape[:2]
    out = {}
    for b in range(B):
        for h in range(H):
            if heads is None or (b, h) in heads:
                out[(b, h)] = ao.antidiag_scores(q[b, h].double().numpy(), k[b, h].double().numpy(), block, stride)
    return out


def assert_close(got, want, what):
    g = got.astype(np.float64)
    err = np.abs(g - want)
    bound = RTOL * np.abs(want) + ATOL
    assert (err <= bound).all(), f"{what}: max err {err.max():.3e}, worst ratio {(err / bound).max():.2f}"
    np.testing.assert_allclose(g.sum(axis=-1), 1.0, rtol=1e-4, err_msg=what)


@pytest.mark.parametrize("name,stride", [("tiny", 8), ("small_ragged", 16), ("small_text", 16), ("small_d64", 8)])
def test_scores_match_oracle_on_synthetic_steps(heart, name, stride):
    g = make_generator(name)
    cfg, st = g.cfg, g.step(0)
    print(f"antidiag {name} N={cfg.N} D={cfg.D} block={cfg.block} stride={stride}", flush=True)
    got = heart.heart_scores_antidiag(st.q.cuda(), st.k.cuda(), cfg.block, stride)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    for (b, h), want in oracle_scores(st.q, st.k, cfg.block, stride).items():
        assert_close(got[b, h], want, f"{name} head ({b},{h})")


@pytest.mark.parametrize("B,H,N,D,block,layout", [
    (1, 2, 5000, 128, 128, "bhnd"),      # 313 reduced rows: three tiles per side, ragged in every way
    (2, 3, 2500, 64, 64, "bnhd"),        # token-major layout, stride 8
    (1, 1, 2048, 128, 128, "padded"),    # exactly one tile, padded token stride
    (1, 9, 300, 128, 128, "bhnd"),       # more heads than XCDs, a fraction of a tile
    (1, 1, 7, 64, 64, "bhnd"),           # fewer tokens than one stride
    (1, 2, 4111, 64, 64, "padded"),      # 514 reduced rows: five tiles, the last nearly empty
])
def test_scores_random_shapes_and_layouts(heart, B, H, N, D, block, layout):
    stride = block // 8
    print(f"antidiag random B={B} H={H} N={N} D={D} block={block} {layout}", flush=True)
    gen = torch.Generator().manual_seed(N + D)
    amp = 3.0
    if layout == "bnhd":
        q = (amp * torch.randn((B, N, H, D), generator=gen)).bfloat16().permute(0, 2, 1, 3)
        k = (amp * torch.randn((B, N, H, D), generator=gen)).bfloat16().permute(0, 2, 1, 3)
        qg, kg = q.permute(0, 2, 1, 3).contiguous().cuda().permute(0, 2, 1, 3), \
            k.permute(0, 2, 1, 3).contiguous().cuda().permute(0, 2, 1, 3)
    elif layout == "padded":
        q = (amp * torch.randn((B, H, N, D), generator=gen)).bfloat16()
        k = (amp * torch.randn((B, H, N, D), generator=gen)).bfloat16()
        qs = torch.full((B, H, N, D + 24), 7.0, dtype=torch.bfloat16, device="cuda")
        ks = torch.full((B, H, N, D + 8), -5.0, dtype=torch.bfloat16, device="cuda")
        qs[..., :D] = q.cuda(); ks[..., :D] = k.cuda()
        qg, kg = qs[..., :D], ks[..., :D]
    else:
        q = (amp * torch.randn((B, H, N, D), generator=gen)).bfloat16()
        k = (amp * torch.randn((B, H, N, D), generator=gen)).bfloat16()
        qg, kg = q.cuda(), k.cuda()
    Nb = (N + block - 1) // block
    scores = torch.full((B, H, Nb, Nb), float("nan"), device="cuda")
    ws = torch.empty(heart.heart_scores_antidiag_workspace_bytes(qg, block, stride) + 64, dtype=torch.uint8,
                     device="cuda").fill_(0xff)   # (NaN patterns: stale workspace contents must not matter)
    heart.heart_scores_antidiag(qg, kg, block, stride, scores=scores, workspace=ws)
    # a second call into the same buffers gives the same bits
    again = torch.empty_like(scores)
    heart.heart_scores_antidiag(qg, kg, block, stride, scores=again, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(scores, again)
    got = scores.cpu().numpy()
    assert np.isfinite(got).all()
    for (b, h), want in oracle_scores(q, k, block, stride).items():
        assert_close(got[b, h], want, f"head ({b},{h})")


def test_selection_through_the_scores_in_seam(heart):
    """Top-p on the estimator's scores: the GPU's selection equals the oracle's selection from
    the same (GPU) scores bit for bit, and the kept sets are those of the oracle's scores up to
    rows whose threshold falls within the score tolerance."""
    g = make_generator("small_text")
    cfg, st = g.cfg, g.step(0)
    nt = cfg.n_text_blocks
    sc = heart.heart_scores_antidiag(st.q.cuda(), st.k.cuda(), cfg.block, 16)
    tau = np.full(cfg.H, 0.9, np.float32)
    gm, gi, gc = heart.heart_mask_topp(None, None, np_gpu(tau), scores_in=sc, n_always_kv_blocks=nt,
                                       n_dense_q_blocks=nt)
    torch.cuda.synchronize()
    om, oi, oc = oracle.topp(sc.cpu().numpy(), tau, n_always_kv=nt, n_dense_q=nt)
    assert_lists_equal(gm, gi, gc, om, oi, oc, "selection from the estimator's scores")
    want = np.stack([np.stack([ao.antidiag_scores(st.q[b, h].double().numpy(), st.k[b, h].double().numpy(),
                                                  cfg.block, 16) for h in range(cfg.H)])
                     for b in range(cfg.B)]).astype(np.float32)
    wm, _, wc = oracle.topp(want, tau, n_always_kv=nt, n_dense_q=nt)
    differing_rows = (gm.cpu().numpy() != wm).any(axis=-1).mean()
    assert differing_rows <= 0.05, f"{differing_rows:.3f} of the rows differ from the oracle-score masks"


def test_full_size_sampled_heads(heart):
    """The benchmark's shape (wan14b_480p) in one call; three heads compared in full."""
    g = make_generator("wan14b_480p")
    cfg, st = g.cfg, g.step(0)
    print(f"antidiag full size N={cfg.N} H={cfg.H}", flush=True)
    sc = heart.heart_scores_antidiag(st.q.cuda(), st.k.cuda(), cfg.block, 16)
    torch.cuda.synchronize()
    got = sc.cpu().numpy()
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got.astype(np.float64).sum(axis=-1), 1.0, rtol=1e-4)
    heads = {(0, 0), (0, 17), (0, cfg.H - 1)}
    for (b, h), want in oracle_scores(st.q, st.k, cfg.block, 16, heads).items():
        assert_close(got[b, h], want, f"wan14b_480p head {h}")


def test_largest_shape_one_head(heart):
    """The HunyuanVideo-shaped config: 7441 reduced rows (60 records per reduced query, close to
    the limit of 64), text tokens in front; all heads in one call, one head compared in full."""
    g = make_generator("hunyuan_720p")
    cfg, st = g.cfg, g.step(0)
    print(f"antidiag largest shape N={cfg.N} H={cfg.H}", flush=True)
    sc = heart.heart_scores_antidiag(st.q.cuda(), st.k.cuda(), cfg.block, 16)
    torch.cuda.synchronize()
    got = sc.cpu().numpy()
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got.astype(np.float64).sum(axis=-1), 1.0, rtol=1e-4)
    h = 5
    want = oracle_scores(st.q, st.k, cfg.block, 16, {(0, h)})[(0, h)]
    assert_close(got[0, h], want, f"hunyuan_720p head {h}")


def test_reused_heads_are_skipped(heart):
    """With a refresh array only the marked heads are scored; the rest of `scores` is untouched."""
    g = make_generator("small_ragged")
    cfg, st = g.cfg, g.step(0)
    refresh = np.array([[1, 0, 1], [0, 0, 1]], np.uint8)
    scores = torch.full((cfg.B, cfg.H, cfg.Nb, cfg.Nb), -7.0, device="cuda")
    heart.heart_scores_antidiag(st.q.cuda(), st.k.cuda(), cfg.block, 16, scores=scores, refresh=np_gpu(refresh))
    full = heart.heart_scores_antidiag(st.q.cuda(), st.k.cuda(), cfg.block, 16)
    torch.cuda.synchronize()
    for b in range(cfg.B):
        for h in range(cfg.H):
            if refresh[b, h]:
                assert torch.equal(scores[b, h], full[b, h])
            else:
                assert (scores[b, h] == -7.0).all()


def test_argument_validation(heart):
    q = torch.zeros((1, 1, 256, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(heart.HeartError):
        heart.heart_scores_antidiag(q, q, 128, 8)        # block != 8 * stride
    ws = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(heart.HeartError):
        heart.heart_scores_antidiag(q, q, 128, 16, workspace=ws)   # workspace too small
