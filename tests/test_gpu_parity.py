"""GPU parity: every entry point of libheart, called through the C ABI (ctypes
binding), against the CPU oracle on the same seeded inputs.

Protocol (each stage is fed the ORACLE's upstream outputs so that "bit-exact given
identical scores / means" is testable; the chained test then runs the GPU path on
its own intermediates):
  P1 pool   vs oracle.pool            means within 1e-5 relative (+ cancellation floor)
  P2 drift  fed oracle means          drift, refresh, anchors bit-equal
  P3 scores fed oracle block means    within 1e-5 relative
  P4 top-p  fed oracle scores         mask / kept_idx / kept_count bit-equal
  P5 attn   fed oracle kept lists     max-abs <= 2e-2 (times max|out|/2 where outputs exceed 2)
  P6 chain  pool->drift->mask->attn   tolerances as above; mask rows that differ must
                                      be threshold ties within the score tolerance (1e-5 on
                                      the normalised cumulative mass, plus what the GPU's own
                                      block means move the oracle's scores)
"""
import numpy as np
import pytest
import torch

import oracle
from heart_synth import make_generator
from heart_testlib import (ATTN_ATOL, OracleChain, assert_lists_equal, assert_masks_equal_up_to_threshold,
                           assert_means_close, assert_scores_close, attn_atol, check_attn_plan, gpu,
                           np_gpu, pooled_mean_score_shift, u16)

pytestmark = pytest.mark.gpu

SMALL = ["tiny", "small_ragged", "small_text", "small_d64", "small_d64_b128"]


@pytest.fixture(scope="module")
def heart():
    import paper_2605_14513_amd as pkg
    from paper_2605_14513_amd import build as hb

    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    if hb.is_stale() and not __import__("os").path.exists(pkg.lib_path()):
        hb.build(force=True)
    pkg.load_library()
    return pkg


_cache = {}


def case(name, step=0):
    key = (name, step)
    if key not in _cache:
        g = _cache.get(name) or make_generator(name)
        _cache[name] = g
        _cache[key] = g.step(step)
    return _cache[name], _cache[key]


# ------------------------------------------------------------------------------ P1
@pytest.mark.parametrize("name", SMALL)
def test_pool_matches_oracle(heart, name):
    g, st = case(name)
    cfg = g.cfg
    print(f"pool {name} N={cfg.N} D={cfg.D} block={cfg.block}", flush=True)
    qblk, kblk, qmean, kmean = heart.heart_pool_qk(gpu(st.q), gpu(st.k), cfg.block)
    torch.cuda.synchronize()
    for got_b, got_m, x in ((qblk, qmean, st.q), (kblk, kmean, st.k)):
        ob, om = oracle.pool(u16(x), cfg.block)
        amax = float(x.float().abs().max())
        assert_means_close(got_b, ob, amax, f"{name} block means")
        assert_means_close(got_m, om, amax, f"{name} token means")


def test_pool_bnhd_layout_and_reproducible(heart):
    g, st = case("small_ragged")
    cfg = g.cfg
    q = gpu(st.q).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)  # [B,N,H,D] memory
    k = gpu(st.k).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert not q.is_contiguous()
    a = heart.heart_pool_qk(q, k, cfg.block)
    b = heart.heart_pool_qk(gpu(st.q), gpu(st.k), cfg.block)
    c = heart.heart_pool_qk(q, k, cfg.block)
    torch.cuda.synchronize()
    for x, y, z in zip(a, b, c):
        assert torch.equal(x, y) and torch.equal(x, z)  # same bits for both layouts, run to run


# ------------------------------------------------------------------------------ P2
def _drift_sequence(heart, qms, kms, delta, gate, B, H, D):
    """Run the same sequence of means through oracle and GPU; compare bit for bit."""
    oq, ok_, oh = (np.zeros((B, H, D), np.float32), np.zeros((B, H, D), np.float32),
                   np.zeros((B, H), np.uint8))
    gq, gk, gh = np_gpu(oq), np_gpu(ok_), np_gpu(oh)
    gdelta = np_gpu(delta)
    fracs = []
    for t, (qm, km) in enumerate(zip(qms, kms)):
        od, orf = oracle.drift(qm, km, oq, ok_, oh, delta, gate[0], gate[1])
        gd, grf = heart.heart_drift(np_gpu(qm), np_gpu(km), gq, gk, gh, gdelta, gate[0], gate[1])
        torch.cuda.synchronize()
        assert np.array_equal(gd.cpu().numpy().view(np.uint32), od.view(np.uint32)), f"step {t} drift bits"
        assert np.array_equal(grf.cpu().numpy(), orf), f"step {t} refresh"
        assert np.array_equal(gq.cpu().numpy(), oq) and np.array_equal(gk.cpu().numpy(), ok_)
        assert np.array_equal(gh.cpu().numpy(), oh)
        fracs.append(orf.mean())
    return fracs


@pytest.mark.parametrize("name", ["tiny", "small_ragged", "small_text"])
@pytest.mark.parametrize("gate", [(0.0, 1.0), (0.4, 0.8)])
def test_drift_bit_exact_on_oracle_means(heart, name, gate):
    g, _ = case(name)
    cfg = g.cfg
    qms, kms = [], []
    for s in range(cfg.steps):
        _, st = case(name, s)
        qms.append(oracle.pool(u16(st.q), cfg.block)[1])
        kms.append(oracle.pool(u16(st.k), cfg.block)[1])
    print(f"drift {name} gate={gate}", flush=True)
    _drift_sequence(heart, qms, kms, g.delta, gate, cfg.B, cfg.H, cfg.D)


@pytest.mark.parametrize("D", [4, 32, 64, 128, 256, 512])
def test_drift_random_means_all_head_dims(heart, D):
    rng = np.random.default_rng(D)
    B, H = 3, 40
    qms = [rng.standard_normal((B, H, D)).astype(np.float32)]
    kms = [rng.standard_normal((B, H, D)).astype(np.float32)]
    for t in range(5):
        step = (rng.random((B, H, 1)) < 0.5) * 0.02
        qms.append((qms[-1] + step * rng.standard_normal((B, H, D))).astype(np.float32))
        kms.append((kms[-1] + step * rng.standard_normal((B, H, D))).astype(np.float32))
    delta = np.full(H, 0.015 * D, np.float32)
    fr = _drift_sequence(heart, qms, kms, delta, (0.4, 0.8), B, H, D)
    assert fr[0] == 1.0


def test_drift_hand_example_and_commit_off(heart):
    qa = np.array([[[1.0, -0.5, 0.25, 0.0], [0.5, 0.5, -1.0, 2.0]]], np.float32)
    qb = np.array([[[1.25, -0.5, 0.0, 0.5], [0.5, 0.5, -1.0, 2.0]]], np.float32)
    ka = np.zeros((1, 2, 4), np.float32)
    kb = np.array([[[0.125, -0.125, 0.0, 0.0], [0, 0, 0, 0]]], np.float32)
    has = np.ones((1, 2), np.uint8)
    for delta, want in ((1.25, [0, 0]), (1.0, [1, 0])):
        gq, gk, gh = np_gpu(qa), np_gpu(ka), np_gpu(has)
        d, r = heart.heart_drift(np_gpu(qb), np_gpu(kb), gq, gk, gh,
                                 np_gpu(np.full(2, delta, np.float32)), 0.0, 1.0, commit=False)
        torch.cuda.synchronize()
        assert d.cpu().numpy().tolist() == [[1.25, 0.0]]
        assert r.cpu().numpy().tolist() == [want]
        assert np.array_equal(gq.cpu().numpy(), qa)  # commit off: anchors untouched


# ------------------------------------------------------------------------------ fused P1 + P2
@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("gate", [(0.0, 1.0), (0.4, 0.8)])
def test_pool_drift_equals_the_two_calls(heart, name, gate):
    """heart_pool_drift over the whole schedule with carried anchors: every output has the bits
    of heart_pool_qk followed by heart_drift, the decisions are the oracle's, and the ticket
    workspace is zero again after every call."""
    g, _ = case(name)
    cfg = g.cfg
    B, H, D = cfg.B, cfg.H, cfg.D
    dev = "cuda"
    f32 = dict(dtype=torch.float32, device=dev)
    state = [dict(qa=torch.zeros((B, H, D), **f32), ka=torch.zeros((B, H, D), **f32),
                  has=torch.zeros((B, H), dtype=torch.uint8, device=dev)) for _ in range(2)]
    ws = torch.zeros(heart.heart_pool_drift_workspace_bytes(B, H) // 4 + 2, dtype=torch.int32, device=dev)
    oq, ok_, oh = np.zeros((B, H, D), np.float32), np.zeros((B, H, D), np.float32), np.zeros((B, H), np.uint8)
    gdelta = np_gpu(g.delta)
    for s in range(cfg.steps):
        _, st = case(name, s)
        print(f"fused pool+drift {name} gate={gate} step {s}", flush=True)
        q, k = gpu(st.q), gpu(st.k)
        if s % 2:  # alternate the memory layout: [B,N,H,D] storage on odd steps
            q = q.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
            k = k.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        a, f = state
        qblk, kblk, qmean, kmean = heart.heart_pool_qk(q, k, cfg.block)
        d, r = heart.heart_drift(qmean, kmean, a["qa"], a["ka"], a["has"], gdelta, gate[0], gate[1])
        fq, fk, fqm, fkm, fd, fr = heart.heart_pool_drift(q, k, cfg.block, f["qa"], f["ka"], f["has"], gdelta,
                                                          ws, gate[0], gate[1])
        torch.cuda.synchronize()
        for x, y, what in ((fq, qblk, "qblk"), (fk, kblk, "kblk"), (fqm, qmean, "qmean"), (fkm, kmean, "kmean"),
                           (fd, d, "drift"), (fr, r, "refresh"), (f["qa"], a["qa"], "qanchor"),
                           (f["ka"], a["ka"], "kanchor"), (f["has"], a["has"], "has_anchor")):
            assert torch.equal(x, y), f"step {s}: {what} differs between the fused and the separate calls"
        assert not ws.any().item(), "the ticket workspace is zero again after the call"
        # and against the oracle: decisions exact, means within the pooling tolerance
        oqb, oqm = oracle.pool(u16(st.q), cfg.block)
        okb, okm = oracle.pool(u16(st.k), cfg.block)
        od, orf = oracle.drift(oqm, okm, oq, ok_, oh, g.delta, gate[0], gate[1])
        assert np.array_equal(fr.cpu().numpy(), orf) and np.array_equal(f["has"].cpu().numpy(), oh)
        amax = float(max(st.q.float().abs().max(), st.k.float().abs().max()))
        assert_means_close(fqm, oqm, amax, "q token means")
        assert_means_close(fkm, okm, amax, "k token means")
        assert_means_close(fq, oqb, amax, "q block means")


def test_pool_drift_commit_off_and_validation(heart):
    g, st = case("small_d64")
    cfg = g.cfg
    B, H, D = cfg.B, cfg.H, cfg.D
    q, k = gpu(st.q), gpu(st.k)
    qa = torch.ones((B, H, D), device="cuda"); ka = torch.ones((B, H, D), device="cuda")
    has = torch.ones((B, H), dtype=torch.uint8, device="cuda")
    ws = torch.zeros(heart.heart_pool_drift_workspace_bytes(B, H), dtype=torch.uint8, device="cuda")
    out = heart.heart_pool_drift(q, k, cfg.block, qa, ka, has, np_gpu(np.full(H, 1e-3, np.float32)), ws,
                                 0.0, 1.0, commit=False)
    torch.cuda.synchronize()
    assert out[5].all().item()                     # far from the anchors: every head refreshes
    assert (qa == 1).all().item() and (ka == 1).all().item()  # commit off: anchors untouched
    assert not ws.any().item()
    with pytest.raises(heart.HeartError):
        heart.heart_pool_drift(q, k, cfg.block, qa, ka, has, np_gpu(g.delta), ws[:-1])


# ------------------------------------------------------------------------------ P3
def _topp_workspace(heart, shape, sliced):
    """A workspace for heart_mask_topp (score stage on 8-bit slices of the block means), or None."""
    if not sliced:
        return None
    B, H, Nb, D = shape
    return torch.empty(heart.heart_mask_topp_workspace_bytes(B, H, Nb, D), dtype=torch.uint8, device="cuda")


@pytest.mark.parametrize("sliced", [False, True])
@pytest.mark.parametrize("name", SMALL)
def test_scores_match_oracle(heart, name, sliced):
    g, st = case(name)
    cfg = g.cfg
    qblk, _ = oracle.pool(u16(st.q), cfg.block)
    kblk, _ = oracle.pool(u16(st.k), cfg.block)
    want = oracle.scores(qblk, kblk)
    out = torch.empty(want.shape, dtype=torch.float32, device="cuda")
    print(f"scores {name} Nb={cfg.Nb} sliced={sliced}", flush=True)
    heart.heart_mask_topp(np_gpu(qblk), np_gpu(kblk), np_gpu(g.tau), scores_out=out,
                          workspace=_topp_workspace(heart, qblk.shape, sliced))
    torch.cuda.synchronize()
    assert_scores_close(out, want, name)


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("Nb", [1, 17, 100, 300, 600])
def test_scores_from_slices_wide_dynamic_range(heart, D, Nb):
    """The score stage on 8-bit slices: block means whose entries span many binades inside one
    block and from block to block, zero blocks, denormal entries, a lone large entry, partial
    refresh (reused heads are neither sliced nor written) -- scores against the oracle, and the
    kept lists against the oracle's selection from the scores the kernel reports."""
    rng = np.random.default_rng(7 * Nb + D)
    B, H = 2, 3
    mag = 2.0 ** rng.integers(-12, 3, size=(B, H, Nb, D))           # entry-wise binades
    qblk = (rng.standard_normal((B, H, Nb, D)) * mag).astype(np.float32)
    blockmag = 2.0 ** rng.integers(-6, 2, size=(B, H, Nb, 1))        # block-wise binades
    kblk = (rng.standard_normal((B, H, Nb, D)) * blockmag).astype(np.float32)
    kblk[0, 0, 0] = 0.0                                              # a zero block
    qblk[0, 1, Nb // 2] = 0.0
    kblk[1, 2, Nb - 1, : D // 2] = np.float32(1e-41)                 # denormal entries
    kblk[1, 0, Nb // 3] = 0.0
    kblk[1, 0, Nb // 3, 5] = 3.0                                     # a lone large entry
    qblk[1, 0, :, 5] += 1.5
    tau = np.array([0.9, 0.6, 0.97], np.float32)
    want = oracle.scores(qblk, kblk)
    ws = _topp_workspace(heart, qblk.shape, True)
    out = torch.zeros(want.shape, dtype=torch.float32, device="cuda")
    print(f"sliced scores Nb={Nb} D={D}", flush=True)
    gm, gi, gc = heart.heart_mask_topp(np_gpu(qblk), np_gpu(kblk), np_gpu(tau), scores_out=out, workspace=ws)
    torch.cuda.synchronize()
    assert_scores_close(out, want, f"slices Nb={Nb} D={D}")
    om, oi, oc = oracle.topp(out.cpu().numpy(), tau)
    assert_lists_equal(gm, gi, gc, om, oi, oc, f"slices Nb={Nb} D={D}")
    # partial refresh: the same call on poisoned outputs writes refreshed heads only, same bits
    refresh = np.array([[1, 0, 1], [0, 1, 0]], np.uint8)
    m2 = torch.full_like(gm, 7); i2 = torch.full_like(gi, -5); c2 = torch.full_like(gc, -3)
    ws.fill_(0xAB)
    heart.heart_mask_topp(np_gpu(qblk), np_gpu(kblk), np_gpu(tau), refresh=np_gpu(refresh), mask=m2,
                          kept_idx=i2, kept_count=c2, workspace=ws)
    torch.cuda.synchronize()
    r = torch.from_numpy(refresh.astype(bool)).cuda()
    assert torch.equal(m2[r], gm[r]) and torch.equal(c2[r], gc[r])
    assert bool((m2[~r] == 7).all()) and bool((i2[~r] == -5).all()) and bool((c2[~r] == -3).all())


@pytest.mark.parametrize("sliced", [False, True])
def test_scores_large_logits_and_many_blocks(heart, sliced):
    # Nb = 600 (10 slots per lane), logits up to about +-30
    rng = np.random.default_rng(0)
    B, H, Nb, D = 1, 2, 600, 128
    base = rng.standard_normal((B, H, 6, D))
    sel = rng.integers(0, 6, size=(B, H, Nb))
    qblk = (np.take_along_axis(base, sel[..., None], 2) * 1.6
            + 0.05 * rng.standard_normal((B, H, Nb, D))).astype(np.float32)
    kblk = (np.take_along_axis(base, sel[..., None], 2) * 1.6
            + 0.05 * rng.standard_normal((B, H, Nb, D))).astype(np.float32)
    want = oracle.scores(qblk, kblk)
    out = torch.empty(want.shape, dtype=torch.float32, device="cuda")
    heart.heart_mask_topp(np_gpu(qblk), np_gpu(kblk), np_gpu(np.array([0.9, 0.5], np.float32)),
                          scores_out=out, workspace=_topp_workspace(heart, qblk.shape, sliced))
    torch.cuda.synchronize()
    assert_scores_close(out, want, "large logits")


# ------------------------------------------------------------------------------ P4
def _topp_both(heart, scores, tau, refresh=None, **kw):
    o = oracle.topp(scores, tau, refresh=refresh, **kw)
    gm, gi, gc = heart.heart_mask_topp(None, None, np_gpu(tau), scores_in=np_gpu(scores),
                                       refresh=None if refresh is None else np_gpu(refresh), **{
                                           "n_always_kv_blocks": kw.get("n_always_kv", 0),
                                           "n_dense_q_blocks": kw.get("n_dense_q", 0),
                                           "min_keep": kw.get("min_keep", 1)})
    torch.cuda.synchronize()
    return (gm, gi, gc), o


@pytest.mark.parametrize("name", SMALL)
def test_topp_bit_exact_on_oracle_scores(heart, name):
    g, st = case(name)
    cfg = g.cfg
    qblk, _ = oracle.pool(u16(st.q), cfg.block)
    kblk, _ = oracle.pool(u16(st.k), cfg.block)
    scores = oracle.scores(qblk, kblk)
    nt = cfg.n_text_blocks
    print(f"topp {name} Nb={cfg.Nb}", flush=True)
    (gm, gi, gc), (om, oi, oc) = _topp_both(heart, scores, g.tau, n_always_kv=nt, n_dense_q=nt)
    assert_lists_equal(gm, gi, gc, om, oi, oc, name)


@pytest.mark.parametrize("Nb", [1, 2, 63, 64, 65, 200, 256, 257, 511, 931, 1024])
def test_topp_adversarial_rows(heart, Nb):
    """Ties, uniform rows, one-hot rows, zeros, sub-quantum scores, thresholds at
    exact mass boundaries -- at every lane-slot width including the maximum Nb."""
    rng = np.random.default_rng(Nb)
    rows = []
    r = rng.random(Nb).astype(np.float32) ** 8
    rows.append(r / r.sum())
    rows.append(np.full(Nb, np.float32(1.0 / 1024)))                       # all tied
    oh = np.zeros(Nb, np.float32); oh[Nb // 2] = 1.0; rows.append(oh)       # one-hot
    q = np.round(rng.random(Nb) * 8) / 8 / Nb; rows.append(q.astype(np.float32))  # many ties + zeros
    rows.append(np.zeros(Nb, np.float32))                                   # no mass at all
    tiny = np.full(Nb, np.float32(2.0 ** -31)); tiny[0] = 0.5; rows.append(tiny)  # sub-quantum tail
    dy = (2.0 ** -np.minimum(np.arange(Nb) + 1, 40)).astype(np.float32); rows.append(dy)  # dyadic
    while len(rows) < Nb:
        r = rng.random(Nb).astype(np.float32) ** rng.integers(1, 12)
        rows.append((r / r.sum()).astype(np.float32))
    scores = np.stack(rows[:Nb])[None, None]
    scores = np.concatenate([scores, scores[:, :, ::-1]], axis=1)  # second head: rows reversed
    scores = np.ascontiguousarray(scores)
    for tau in (0.5, 0.75, 0.9, 0.999, 1.0, 2.0 ** -20):
        t = np.array([tau, min(1.0, tau + 0.05)], np.float32)
        (gm, gi, gc), (om, oi, oc) = _topp_both(heart, scores, t)
        assert_lists_equal(gm, gi, gc, om, oi, oc, f"Nb={Nb} tau={tau}")
    (gm, gi, gc), (om, oi, oc) = _topp_both(heart, scores, np.array([0.3, 0.6], np.float32),
                                            n_always_kv=min(2, Nb), n_dense_q=1,
                                            min_keep=min(5, Nb))
    assert_lists_equal(gm, gi, gc, om, oi, oc, f"Nb={Nb} extras")


@pytest.mark.parametrize("Nb", [1, 2, 31, 33, 64, 65, 100, 255, 256, 257, 511, 600, 931, 1024])
def test_topp_from_own_scores_ties_floors_and_flags(heart, Nb):
    """The selection that follows the kernel's own score stage (two rows per wavefront, at every
    lane-slot width): exact ties from duplicated key blocks, uniform rows
    from identical key blocks, a threshold that truncates to zero mass, the floor on the number
    of kept blocks, always-kept columns and dense rows, tau >= 1 -- each compared bit for bit
    with the oracle's selection from the scores the kernel reports."""
    B, H, D = 1, 3, 32
    rng = np.random.default_rng(1000 + Nb)
    qblk = (2.0 * rng.standard_normal((B, H, Nb, D))).astype(np.float32)
    kblk = (2.0 * rng.standard_normal((B, H, Nb, D))).astype(np.float32)
    kblk[0, 0, 1::2] = kblk[0, 0, 0:2 * (Nb // 2):2]   # head 0: key blocks in identical pairs
    kblk[0, 1, :] = kblk[0, 1, 0]                        # head 1: all key blocks identical
    qg, kg = np_gpu(qblk), np_gpu(kblk)
    cases = [((0.9, 0.5, 0.95), {}), ((1e-9, 1e-9, 1e-9), {}), ((0.6, 0.6, 0.6), dict(min_keep=5)),
             ((0.3, 0.3, 0.3), dict(min_keep=300)), ((0.8, 0.8, 0.8), dict(n_always_kv=min(2, Nb), n_dense_q=1)),
             ((1.0, 0.7, 1.5), {})]
    for taus, kw in cases:
        tau = np.array(taus, np.float32)
        sc = torch.empty((B, H, Nb, Nb), dtype=torch.float32, device="cuda")
        gm, gi, gc = heart.heart_mask_topp(qg, kg, np_gpu(tau), scores_out=sc,
                                           n_always_kv_blocks=kw.get("n_always_kv", 0),
                                           n_dense_q_blocks=kw.get("n_dense_q", 0),
                                           min_keep=kw.get("min_keep", 1))
        torch.cuda.synchronize()
        s = sc.cpu().numpy()
        if Nb >= 2:
            assert np.array_equal(s[0, 0, :, 0], s[0, 0, :, 1]), "duplicated key blocks must tie exactly"
        om, oi, oc = oracle.topp(s, tau, **kw)
        assert_lists_equal(gm, gi, gc, om, oi, oc, f"Nb={Nb} tau={taus} {kw}")


def test_topp_reused_heads_are_untouched(heart):
    rng = np.random.default_rng(1)
    B, H, Nb = 2, 3, 70
    s = rng.random((B, H, Nb, Nb)).astype(np.float32) ** 5
    s /= s.sum(-1, keepdims=True)
    tau = np.array([0.8, 0.9, 0.95], np.float32)
    refresh = np.array([[1, 0, 1], [0, 0, 1]], np.uint8)
    mask = torch.full((B, H, Nb, Nb), 7, dtype=torch.uint8, device="cuda")
    kidx = torch.full((B, H, Nb, Nb), -5, dtype=torch.int32, device="cuda")
    kcnt = torch.full((B, H, Nb), -3, dtype=torch.int32, device="cuda")
    heart.heart_mask_topp(None, None, np_gpu(tau), scores_in=np_gpu(s), refresh=np_gpu(refresh),
                          mask=mask, kept_idx=kidx, kept_count=kcnt)
    torch.cuda.synchronize()
    om, oi, oc = oracle.topp(s, tau)
    for b in range(B):
        for h in range(H):
            if refresh[b, h]:
                assert np.array_equal(mask[b, h].cpu().numpy(), om[b, h])
                assert np.array_equal(kcnt[b, h].cpu().numpy(), oc[b, h])
            else:
                assert (mask[b, h] == 7).all() and (kidx[b, h] == -5).all() and (kcnt[b, h] == -3).all()


# ------------------------------------------------------------------------------ P5
def _attn_case(heart, name, tau_override=None, lse=False):
    g, st = case(name)
    cfg = g.cfg
    qblk, _ = oracle.pool(u16(st.q), cfg.block)
    kblk, _ = oracle.pool(u16(st.k), cfg.block)
    scores = oracle.scores(qblk, kblk)
    tau = g.tau if tau_override is None else np.full(cfg.H, tau_override, np.float32)
    nt = cfg.n_text_blocks
    om, oi, oc = oracle.topp(scores, tau, n_always_kv=nt, n_dense_q=nt)
    want = oracle.attn(u16(st.q), u16(st.k), u16(st.v), cfg.block, oi, oc, want_lse=lse)
    glse = torch.empty((cfg.B, cfg.H, cfg.N), dtype=torch.float32, device="cuda") if lse else None
    print(f"attn {name} N={cfg.N} density={oc.sum() / (oc.size * cfg.Nb):.3f}", flush=True)
    out = heart.heart_block_sparse_attn(gpu(st.q), gpu(st.k), gpu(st.v), cfg.block, np_gpu(oi),
                                        np_gpu(oc), lse=glse)
    torch.cuda.synchronize()
    return out, glse, want, (st, cfg)


@pytest.mark.parametrize("name", SMALL)
def test_attn_matches_oracle_on_oracle_lists(heart, name):
    out, _, want, _ = _attn_case(heart, name)
    err = (out.float().cpu().numpy().astype(np.float64) - want).__abs__().max()
    assert err <= ATTN_ATOL, f"{name}: max abs err {err:.4f}"


def test_attn_dense_value_equals_dense_attention_and_lse(heart):
    # tau = 1 keeps every block: sparse attention must equal brute-force dense attention
    out, glse, (want, wlse), (st, cfg) = _attn_case(heart, "tiny", tau_override=1.0, lse=True)
    dense = oracle.dense_attn(u16(st.q), u16(st.k), u16(st.v))
    got = out.float().cpu().numpy().astype(np.float64)
    assert np.abs(got - dense).max() <= ATTN_ATOL
    assert np.abs(got - want).max() <= ATTN_ATOL
    assert np.abs(glse.cpu().numpy() - wlse).max() <= 2e-2


def test_attn_strided_layout_unsorted_lists_and_empty_rows(heart):
    g, st = case("small_ragged")
    cfg = g.cfg
    rng = np.random.default_rng(5)
    Nb = cfg.Nb
    # random kept lists in random (non-ascending) order; some rows empty
    idx = np.zeros((cfg.B, cfg.H, Nb, Nb), np.int32)
    cnt = rng.integers(0, Nb + 1, size=(cfg.B, cfg.H, Nb)).astype(np.int32)
    for b in range(cfg.B):
        for h in range(cfg.H):
            for i in range(Nb):
                idx[b, h, i, :cnt[b, h, i]] = rng.permutation(Nb)[:cnt[b, h, i]]
    cnt[0, 0, 1] = 0
    want = oracle.attn(u16(st.q), u16(st.k), u16(st.v), cfg.block,
                       idx, np.maximum(cnt, 0))
    def bnhd(x):
        return gpu(x).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    q, k, v = bnhd(st.q), bnhd(st.k), bnhd(st.v)
    out = torch.empty_like(q)  # preserves the [B,N,H,D] memory layout
    assert out.stride() == q.stride()
    heart.heart_block_sparse_attn(q, k, v, cfg.block, np_gpu(idx), np_gpu(cnt), out=out)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    empty = cnt == 0
    rows_empty = np.repeat(empty, cfg.block, axis=2)[:, :, :cfg.N]
    assert np.all(got[rows_empty] == 0.0)  # empty rows give zeros
    err = np.abs(got - want)[~rows_empty].max()
    assert err <= ATTN_ATOL, f"max abs err {err:.4f}"


def test_attn_launch_plan_and_same_bits_with_and_without_it(heart):
    # the workspace receives the launch plan (heads assigned to XCDs, rows of a head longest
    # first); the output bits do not depend on it
    g, st = case("small_ragged")
    cfg = g.cfg
    rng = np.random.default_rng(9)
    Nb = cfg.Nb
    cnt = rng.integers(0, Nb + 1, size=(cfg.B, cfg.H, Nb)).astype(np.int32)
    cnt[0, 1] //= 3  # heads of different weight
    idx = np.zeros((cfg.B, cfg.H, Nb, Nb), np.int32)
    for b in range(cfg.B):
        for h in range(cfg.H):
            for i in range(Nb):
                idx[b, h, i, :cnt[b, h, i]] = np.sort(rng.permutation(Nb)[:cnt[b, h, i]])
    q, k, v = gpu(st.q), gpu(st.k), gpu(st.v)
    n = cfg.B * cfg.H * Nb
    words = heart.heart_attn_workspace_bytes(q, cfg.block) // 4
    assert words == 24 + 2 * cfg.B * cfg.H + n
    ws = torch.full((words + 3,), -7, dtype=torch.int32, device="cuda")
    out_planned = heart.heart_block_sparse_attn(q, k, v, cfg.block, np_gpu(idx), np_gpu(cnt), workspace=ws)
    out_natural = heart.heart_block_sparse_attn(q, k, v, cfg.block, np_gpu(idx), np_gpu(cnt), workspace=None)
    torch.cuda.synchronize()
    plan = ws.cpu().numpy()
    assert (plan[words:] == -7).all()  # nothing written past the stated size
    check_attn_plan(plan[:words], cnt, Nb)
    assert torch.equal(out_planned, out_natural)
    with pytest.raises(heart.HeartError):
        heart.heart_block_sparse_attn(q, k, v, cfg.block, np_gpu(idx), np_gpu(cnt), workspace=ws[:words - 1])


# ------------------------------------------------------------------------------ P6
@pytest.mark.parametrize("name", ["tiny", "small_ragged", "small_text"])
def test_chained_steps_match_oracle(heart, name):
    g, _ = case(name)
    cfg = g.cfg
    B, H, D, Nb, nt = cfg.B, cfg.H, cfg.D, cfg.Nb, cfg.n_text_blocks
    dev = "cuda"
    # caller-owned state: the GPU's, and the oracle's inside OracleChain
    gq = torch.zeros((B, H, D), device=dev); gk = torch.zeros((B, H, D), device=dev)
    gh = torch.zeros((B, H), dtype=torch.uint8, device=dev)
    gmask = torch.zeros((B, H, Nb, Nb), dtype=torch.uint8, device=dev)
    gidx = torch.zeros((B, H, Nb, Nb), dtype=torch.int32, device=dev)
    gcnt = torch.zeros((B, H, Nb), dtype=torch.int32, device=dev)
    chain = OracleChain(cfg, g.tau, g.delta)
    gtau, gdelta = np_gpu(g.tau), np_gpu(g.delta)
    for s in range(cfg.steps):
        _, st = case(name, s)
        print(f"chain {name} step {s}", flush=True)
        q, k, v = gpu(st.q), gpu(st.k), gpu(st.v)
        qblk, kblk, qmean, kmean = heart.heart_pool_qk(q, k, cfg.block)
        d, r = heart.heart_drift(qmean, kmean, gq, gk, gh, gdelta, 0.4, 0.8)
        heart.heart_mask_topp(qblk, kblk, gtau, refresh=r, n_always_kv_blocks=nt,
                              n_dense_q_blocks=nt, mask=gmask, kept_idx=gidx, kept_count=gcnt)
        out = heart.heart_block_sparse_attn(q, k, v, cfg.block, gidx, gcnt)
        torch.cuda.synchronize()
        od, orf = chain.step(st)
        oout = oracle.attn(u16(st.q), u16(st.k), u16(st.v), cfg.block, chain.idx, chain.cnt)
        # decisions: a GPU/oracle disagreement is only legitimate if the drift sits
        # within rounding of delta; the synthetic schedules keep clear of it
        assert np.array_equal(r.cpu().numpy(), orf), f"step {s}: refresh decisions differ"
        gd = d.cpu().numpy()
        fin = np.isfinite(od)
        assert np.allclose(gd[fin], od[fin], rtol=1e-4, atol=1e-6)
        # masks of the heads refreshed at this step: rows may differ only where the cumulative
        # mass passes within the score tolerance of the threshold (reused heads keep masks that
        # were checked at the step that made them)
        shift = pooled_mean_score_shift(chain.scores, qblk, kblk)
        fresh = orf.astype(bool)[:, :, None]
        gm = gmask.cpu().numpy()
        assert_masks_equal_up_to_threshold(
            np.where(fresh[..., None], gm, chain.mask), chain.mask, chain.scores, chain.cnt, g.tau,
            f"{name} step {s}", row_tol=shift)
        same = ~(gm != chain.mask).any(-1)
        got = out.float().cpu().numpy().astype(np.float64)
        rows_same = np.repeat(same, cfg.block, axis=2)[:, :, :cfg.N]
        err = np.abs(got - oout)[rows_same].max()
        assert err <= attn_atol(oout), f"step {s}: attention max abs err {err:.4f}"


# ------------------------------------------------------------------------------ precision
@pytest.mark.parametrize("amp", [0.5, 1.0, 2.0, 3.0])
@pytest.mark.parametrize("fold", [False, True])
def test_attn_error_against_input_magnitude(heart, amp, fold):
    """Precision contract of the attention kernel on iid N(0, amp^2) inputs (logits of standard
    deviation amp^2: +-27 at amp = 3, nearly one-hot rows; outputs of magnitude up to ~4 amp).
    Default path: logits scaled in fp32, so the error is the bf16 rounding of the weights and of
    the output and the bound follows the output's magnitude, 2e-2 * max(1, max|out| / 2), at
    every amplitude.  With HEART_ATTN_FOLD_SCALE the query carries one more bf16 rounding, whose
    effect grows with the cube of the input scale: the same bound is required up to amp = 2
    (logits of +-12) and at amp = 3 the path is only required to stay finite and within its
    documented cube law."""
    B, H, N, D, blk = 1, 2, 700, 128, 128
    Nb = (N + blk - 1) // blk
    gen = torch.Generator().manual_seed(int(amp * 10))
    q, k, v = ((amp * torch.randn((B, H, N, D), generator=gen)).bfloat16() for _ in range(3))
    idx = np.broadcast_to(np.arange(Nb, dtype=np.int32), (B, H, Nb, Nb)).copy()
    cnt = np.full((B, H, Nb), Nb, np.int32)
    flags = heart.HEART_ATTN_FOLD_SCALE if fold else 0
    out = heart.heart_block_sparse_attn(gpu(q), gpu(k), gpu(v), blk, np_gpu(idx), np_gpu(cnt), flags=flags)
    torch.cuda.synchronize()
    want = oracle.attn(u16(q), u16(k), u16(v), blk, idx, cnt)
    got = out.float().cpu().numpy().astype(np.float64)
    err = np.abs(got - want).max()
    bound = attn_atol(want)
    print(f"amp {amp} fold={fold}: max abs err {err:.4f}, bound {bound:.4f} "
          f"(outputs up to {np.abs(want).max():.1f})", flush=True)
    if fold and amp > 2.0:
        assert np.isfinite(got).all() and err <= ATTN_ATOL * amp ** 3
    else:
        assert err <= bound


@pytest.mark.parametrize("fold", [False, True])
def test_attn_both_scale_paths_on_the_synthetic_fields(heart, fold):
    # the workloads' own value range (logits spanning ~8): both paths inside the plain 2e-2
    g, st = case("small_ragged")
    cfg = g.cfg
    qblk, _ = oracle.pool(u16(st.q), cfg.block)
    kblk, _ = oracle.pool(u16(st.k), cfg.block)
    _, oi, oc = oracle.topp(oracle.scores(qblk, kblk), g.tau)
    want = oracle.attn(u16(st.q), u16(st.k), u16(st.v), cfg.block, oi, oc)
    out = heart.heart_block_sparse_attn(gpu(st.q), gpu(st.k), gpu(st.v), cfg.block, np_gpu(oi), np_gpu(oc),
                                        flags=heart.HEART_ATTN_FOLD_SCALE if fold else 0)
    torch.cuda.synchronize()
    err = np.abs(out.float().cpu().numpy().astype(np.float64) - want).max()
    print(f"fold={fold}: max abs err {err:.4f}", flush=True)
    assert err <= ATTN_ATOL


@pytest.mark.parametrize("B,H,N,D,blk", [
    (1, 1, 33, 128, 128),     # one ragged block, a single head: 7 of the 8 XCD lists are empty
    (1, 1, 100, 64, 64),      # two blocks, the second ragged
    (1, 3, 128, 64, 128),     # exactly one full block per head
    (2, 2, 1, 128, 128),      # a single token
    (1, 5, 700, 128, 128),    # fewer heads than XCDs
    (1, 9, 330, 64, 64),      # more heads than XCDs, uneven lists
    (1, 2, 4100, 64, 128),    # 33 blocks, last one with 4 tokens
    (1, 3, 333, 128, 64),     # D = 128 with blocks of 64 tokens, ragged last block
    (2, 2, 64, 128, 64),      # the same pair, exactly one block
])
def test_attn_small_and_odd_shapes(heart, B, H, N, D, blk):
    # random bf16 tensors, random kept lists with duplicates and out-of-order entries;
    # K/V rows padded (row stride larger than D) to exercise the strides
    rng = np.random.default_rng(B * 1000 + H * 100 + N)
    Nb = (N + blk - 1) // blk
    def rand():
        full = torch.randn((B, H, N, D + 16), generator=torch.Generator().manual_seed(int(rng.integers(1 << 30)))).to(torch.bfloat16)
        return full
    qf_, kf_, vf_ = rand(), rand(), rand()
    qc, kc, vc = (x[..., :D] for x in (qf_, kf_, vf_))          # CPU views
    q, k, v = (x.cuda()[..., :D] for x in (qf_, kf_, vf_))       # strided GPU views (token stride D+16)
    cnt = rng.integers(0, Nb + 1, size=(B, H, Nb)).astype(np.int32)
    idx = rng.integers(0, Nb, size=(B, H, Nb, Nb)).astype(np.int32)  # duplicates allowed
    want = oracle.attn(u16(qc.contiguous()), u16(kc.contiguous()), u16(vc.contiguous()), blk, idx, cnt)
    for ws in ("auto", None):
        out = torch.full((B, H, N, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        heart.heart_block_sparse_attn(q, k, v, blk, np_gpu(idx), np_gpu(cnt), out=out, workspace=ws)
        torch.cuda.synchronize()
        got = out.float().cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all(), "every output row is written"
        rows_empty = np.repeat(cnt == 0, blk, axis=2)[:, :, :N]
        assert np.all(got[rows_empty] == 0.0)  # rows without kept blocks give zeros
        if (~rows_empty).any():
            err = np.abs(got - want)[~rows_empty].max()
            assert err <= ATTN_ATOL, f"workspace={ws}: max abs err {err:.4f}"
