"""Pins for the CPU oracle: closed forms, invariants, brute force, library special
cases and the hand example.  None of these re-types the oracle's own formula in
the same shape; each would fail for a plausible mistake in it (dropped term,
wrong sign or index, transposed operand, off-by-one at the threshold)."""
import itertools
import json
import os

import numpy as np
import pytest
import torch

import oracle
from heart_synth import as_u16, make_generator

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_example.json")))


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float array -> bf16 bit patterns via torch's round-to-nearest-even."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return as_u16(t).copy().reshape(x.shape)


def bf16_vals(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------- pool
def test_pool_partial_block_pitfall():
    # N=3, block=2, tokens [1,3,5]: block means [2,5]; token mean 3 (not 3.5)
    x = np.array([1.0, 3.0, 5.0], dtype=np.float32).reshape(1, 1, 3, 1).repeat(4, axis=3)
    blk, mean = oracle.pool(bf16_bits(x), block=2)
    assert blk.shape == (1, 1, 2, 4)
    assert np.array_equal(blk[0, 0, :, 0], np.array([2.0, 5.0], dtype=np.float32))
    assert np.array_equal(mean[0, 0], np.full(4, 3.0, dtype=np.float32))


def test_pool_ramp_closed_form():
    # x[n, d] = n + d (all exactly representable in bf16 up to 256)
    N, D, block = 250, 8, 64
    n = np.arange(N, dtype=np.float32)[:, None]
    x = (n % 128 + np.arange(D, dtype=np.float32)[None, :]).reshape(1, 1, N, D)
    bits = bf16_bits(x)
    assert np.array_equal(bf16_vals(bits), x.astype(np.float64))
    blk, mean = oracle.pool(bits, block)
    for i in range(4):
        n0, n1 = i * block, min(N, (i + 1) * block)
        # mean of an arithmetic ramp = midpoint of first and last element
        expect = ((n0 % 128) + ((n1 - 1) % 128)) / 2.0 + np.arange(D)
        assert np.allclose(blk[0, 0, i], expect, rtol=0, atol=0)
    tot = x[0, 0].astype(np.float64).sum(axis=0) / N
    assert np.allclose(mean[0, 0], tot, rtol=1e-7)


def test_pool_matches_numpy_and_strided_layout():
    rng = np.random.default_rng(5)
    B, H, N, D, block = 2, 3, 300, 16, 128
    bits = bf16_bits(rng.standard_normal((B, H, N, D)).astype(np.float32))
    blk, mean = oracle.pool(bits, block)
    v = bf16_vals(bits)
    assert np.allclose(mean, v.mean(axis=2), rtol=1e-6, atol=1e-7)
    assert np.allclose(blk[:, :, 0], v[:, :, :128].mean(axis=2), rtol=1e-6, atol=1e-7)
    assert np.allclose(blk[:, :, 2], v[:, :, 256:].mean(axis=2), rtol=1e-6, atol=1e-7)
    # the same numbers held as [B,N,H,D] in memory must pool identically
    bnhd = np.ascontiguousarray(bits.transpose(0, 2, 1, 3))
    blk2, mean2 = oracle.pool(bnhd.transpose(0, 2, 1, 3), block)
    assert np.array_equal(blk, blk2) and np.array_equal(mean, mean2)


def test_pooled_cache_size_matches_paper():
    c = GOLD["cache_size"]
    per = c["L"] * c["H"] * c["D"] * c["bytes_per_elem"] * c["cfg_branches"] * 2  # Q and K
    assert abs(per / 2**20 - c["pooled_MB"]) < 0.01  # one D-vector per head for Q and K
    assert abs(per * c["N"] / 2**30 - c["token_level_GB"]) < 0.1


# --------------------------------------------------------------------------- drift
def _state(B, H, D):
    return (np.zeros((B, H, D), np.float32), np.zeros((B, H, D), np.float32),
            np.zeros((B, H), np.uint8))


def test_drift_hand_example():
    g = GOLD["drift"]
    D = g["D"]
    for dec in g["decisions"]:
        qa, ka, has = _state(1, 2, D)
        qb = np.zeros((1, 2, D), np.float32)
        kb = np.zeros((1, 2, D), np.float32)
        for h, key in enumerate(("head0", "head1")):
            qa[0, h], qb[0, h] = g[key]["qa"], g[key]["qb"]
            ka[0, h], kb[0, h] = g[key]["ka"], g[key]["kb"]
        has[:] = 1
        d, r = oracle.drift(qb, kb, qa, ka, has, np.full(2, dec["delta"], np.float32),
                            gate_lo=0.0, gate_hi=1.0)
        assert d[0, 0] == np.float32(g["head0"]["drift"])
        assert d[0, 1] == np.float32(g["head1"]["drift"])
        assert r[0, 0] == dec["refresh_head0"]
        assert r[0, 1] == 0  # identical features reuse for any delta >= 0
        if dec["refresh_head0"]:
            assert np.array_equal(qa[0, 0], qb[0, 0]) and np.array_equal(ka[0, 0], kb[0, 0])
        else:
            assert np.array_equal(qa[0, 0], np.array(g["head0"]["qa"], np.float32))


def test_drift_zero_for_identical_steps_even_with_delta_zero():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((2, 5, 64)).astype(np.float32)
    k = rng.standard_normal((2, 5, 64)).astype(np.float32)
    qa, ka, has = q.copy(), k.copy(), np.ones((2, 5), np.uint8)
    d, r = oracle.drift(q, k, qa, ka, has, np.zeros(5, np.float32), 0.0, 1.0)
    assert np.all(d == 0.0) and np.all(r == 0)


def test_drift_no_anchor_always_refreshes_and_commits():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((1, 3, 8)).astype(np.float32)
    k = rng.standard_normal((1, 3, 8)).astype(np.float32)
    qa, ka, has = _state(1, 3, 8)
    d, r = oracle.drift(q, k, qa, ka, has, np.full(3, 1e9, np.float32), 0.4, 0.8)
    assert np.all(r == 1) and np.all(has == 1) and np.all(np.isinf(d))
    assert np.array_equal(qa, q) and np.array_equal(ka, k)
    # commit=False leaves the state alone
    qa, ka, has = _state(1, 3, 8)
    d, r = oracle.drift(q, k, qa, ka, has, np.full(3, 1e9, np.float32), 0.4, 0.8, commit=False)
    assert np.all(r == 1) and np.all(has == 0) and np.all(qa == 0)


def test_drift_is_l1_sum_of_both_terms():
    # independent formulation via numpy in fp64; catches a dropped K term, an
    # averaged (not summed) norm or an L2 norm
    rng = np.random.default_rng(3)
    B, H, D = 2, 4, 128
    q, k, qa, ka = (rng.standard_normal((B, H, D)).astype(np.float32) for _ in range(4))
    has = np.ones((B, H), np.uint8)
    d, _ = oracle.drift(q, k, qa.copy(), ka.copy(), has, np.zeros(H, np.float32), 0.0, 1.0,
                        commit=False)
    ref = np.abs(qa.astype(np.float64) - q).sum(-1) + np.abs(ka.astype(np.float64) - k).sum(-1)
    assert np.allclose(d, ref, rtol=1e-6)
    # triangle inequality a->c <= a->b + b->c
    q2, k2 = q + 0.1, k - 0.2
    dab = ref
    dbc = np.abs(q2.astype(np.float64) - q).sum(-1) + np.abs(k2.astype(np.float64) - k).sum(-1)
    dac, _ = oracle.drift(q2, k2, qa.copy(), ka.copy(), has, np.zeros(H, np.float32), 0.0, 1.0,
                          commit=False)
    assert np.all(dac <= (dab + dbc) * (1 + 1e-6))


def test_drift_anchor_stays_fixed_until_refresh():
    # Alg. 1 trace: slow cumulative drift is measured against the ANCHOR, so it
    # eventually trips delta; after the refresh the anchor is the current step.
    D = 4
    qa, ka, has = _state(1, 1, D)
    delta = np.array([1.0], np.float32)
    refreshed = []
    for t in range(6):
        q = np.full((1, 1, D), 0.125 * t, np.float32)  # step-to-step drift 0.5
        k = np.zeros((1, 1, D), np.float32)
        d, r = oracle.drift(q, k, qa, ka, has, delta, 0.0, 1.0)
        refreshed.append(int(r[0, 0]))
        if t in (1, 2):
            assert d[0, 0] == np.float32(0.5 * t)  # vs anchor at t=0
    # t=0 no anchor; t=1 (0.5), t=2 (1.0 == delta: reuse); t=3 (1.5 > 1) refresh;
    # t=4 (0.5), t=5 (1.0) reuse
    assert refreshed == [1, 0, 0, 1, 0, 0]


@pytest.mark.parametrize("case", GOLD["gate"])
def test_gate_boundaries(case):
    H, marks = case["H"], case["marks"]
    D = 2
    qa, ka, has = _state(1, H, D)
    has[:] = 1
    q = np.zeros((1, H, D), np.float32)
    q[0, :marks, 0] = 2.0  # drift 2 > delta 1 for the first `marks` heads
    k = np.zeros((1, H, D), np.float32)
    d, r = oracle.drift(q, k, qa, ka, has, np.ones(H, np.float32), 0.4, 0.8)
    if case["outcome"] == "headwise":
        assert r[0].tolist() == [1] * marks + [0] * (H - marks)
    elif case["outcome"] == "all_reuse":
        assert not r.any() and np.all(qa == 0)  # forced reuse leaves anchors unchanged
    else:
        assert r.all() and np.array_equal(qa, q)


def test_gate_forced_reuse_never_applies_to_heads_without_anchor():
    H, D = 5, 2
    qa, ka, has = _state(1, H, D)
    has[0, 1:] = 1  # head 0 has no anchor -> marked; 1/5 < 0.4 -> layer reuses
    q = np.zeros((1, H, D), np.float32)
    k = np.zeros((1, H, D), np.float32)
    d, r = oracle.drift(q, k, qa, ka, has, np.ones(H, np.float32), 0.4, 0.8)
    assert r[0].tolist() == [1, 0, 0, 0, 0]


# --------------------------------------------------------------------------- scores
def test_scores_uniform_when_keys_equal():
    rng = np.random.default_rng(0)
    B, H, Nb, D = 1, 2, 16, 64
    q = rng.standard_normal((B, H, Nb, D)).astype(np.float32)
    k = np.broadcast_to(rng.standard_normal((B, H, 1, D)).astype(np.float32), (B, H, Nb, D))
    p = oracle.scores(q, k)
    assert np.all(p == np.float32(1.0 / Nb))


def test_scores_shift_invariance_rowsum_and_library_softmax():
    from scipy.special import softmax

    rng = np.random.default_rng(1)
    B, H, Nb, D = 2, 2, 37, 128
    q = rng.standard_normal((B, H, Nb, D)).astype(np.float32)
    k = rng.standard_normal((B, H, Nb, D)).astype(np.float32)
    p = oracle.scores(q, k)
    assert np.allclose(p.sum(-1), 1.0, atol=1e-6)
    ref = softmax(np.einsum("bhid,bhjd->bhij", q.astype(np.float64), k.astype(np.float64))
                  / np.sqrt(D), axis=-1)
    assert np.allclose(p, ref, rtol=1e-6, atol=1e-12)
    # a transposed operand (K.Q^T) would fail the line above; a missing 1/sqrt(D)
    # too.  Adding one vector c to every key shifts each row's logits equally.
    c = rng.standard_normal((B, H, 1, D)).astype(np.float32)
    p2 = oracle.scores(q, k + c)
    assert np.allclose(p, p2, rtol=2e-5, atol=1e-9)


def test_scores_peaks_on_aligned_key():
    D, Nb = 64, 8
    q = np.zeros((1, 1, Nb, D), np.float32)
    k = np.zeros((1, 1, Nb, D), np.float32)
    q[..., 0] = 1.0
    k[0, 0, 3, 0] = 400.0  # logit 400/8 = 50 against 0 for the rest
    p = oracle.scores(q, k)
    assert np.all(p[0, 0, :, 3] == 1.0) and np.all(p[0, 0, :, 0] < 1e-20)


# --------------------------------------------------------------------------- top-p
def _topp_row(scores, tau, **kw):
    s = np.asarray(scores, np.float32).reshape(1, 1, 1, -1)
    Nb = s.shape[-1]
    full = np.tile(s, (1, 1, Nb, 1))
    m, idx, cnt = oracle.topp(full, np.array([tau], np.float32), **kw)
    return m, idx, cnt


@pytest.mark.parametrize("case", GOLD["topp"])
def test_topp_hand_example(case):
    tau = case["tau"]
    if isinstance(tau, str):
        tau = np.nextafter(np.float32(0.5), np.float32(1.0))
    m, idx, cnt = _topp_row(case["scores"], tau)
    for row in range(4):
        assert m[0, 0, row].tolist() == case["mask"]
        c = cnt[0, 0, row]
        assert c == sum(case["mask"])
        assert idx[0, 0, row, :c].tolist() == [j for j, v in enumerate(case["mask"]) if v]


def test_topp_tau_one_keeps_all_and_monotone_in_tau():
    rng = np.random.default_rng(7)
    Nb = 50
    s = rng.random((1, 3, Nb, Nb)).astype(np.float32) ** 4
    s /= s.sum(-1, keepdims=True)
    prev = None
    for tau in (0.1, 0.3, 0.5, 0.7, 0.9, 0.97, 1.0):
        m, _, cnt = oracle.topp(s, np.full(3, tau, np.float32))
        if prev is not None:
            assert np.all(m >= prev)  # kept(tau1) subset of kept(tau2)
        prev = m
    assert np.all(prev == 1) and np.all(cnt == Nb)


def test_topp_uniform_and_onehot():
    Nb = 40
    s = np.full((1, 1, Nb, Nb), 1.0 / 64, np.float32)
    for tau, want in ((0.5, 20), (0.51, 21), (0.9, 36), (0.26, 11)):
        m, idx, cnt = oracle.topp(s, np.array([tau], np.float32))
        assert np.all(cnt == want)  # ceil(tau * Nb)
        assert np.all(m[..., :want] == 1) and np.all(m[..., want:] == 0)  # lowest indices
    s = np.zeros((1, 1, Nb, Nb), np.float32)
    s[0, 0, np.arange(Nb), (np.arange(Nb) * 7) % Nb] = 1.0
    m, idx, cnt = oracle.topp(s, np.array([0.9], np.float32))
    assert np.all(cnt == 1)
    assert np.array_equal(idx[0, 0, :, 0], (np.arange(Nb) * 7) % Nb)


def test_topp_minimal_by_brute_force():
    # Eq. 1: minimal set whose mass reaches tau.  For Nb <= 8 enumerate every
    # subset: no smaller subset may reach the target, and the kept set must.
    rng = np.random.default_rng(11)
    for Nb in (3, 5, 8):
        for trial in range(20):
            p = rng.random(Nb) ** 3
            p = (np.round(p / p.sum() * 4096) / 4096).astype(np.float32)  # dyadic -> exact sums
            p[p == 0] = 1 / 4096
            tau = np.float32(rng.choice([0.5, 0.75, 0.9, 0.95, 0.8125]))
            m, idx, cnt = _topp_row(p, tau)
            kept = np.flatnonzero(m[0, 0, 0])
            total = float(p.astype(np.float64).sum())
            target = float(tau) * total
            assert p[kept].astype(np.float64).sum() >= target
            k = len(kept)
            for sub in itertools.combinations(range(Nb), k - 1):
                assert p[list(sub)].astype(np.float64).sum() < target
            # and it is the top-k under (score desc, index asc)
            order = sorted(range(Nb), key=lambda j: (-p[j], j))
            assert sorted(order[:k]) == kept.tolist()


def test_topp_always_kept_dense_rows_min_keep_and_refresh():
    rng = np.random.default_rng(3)
    Nb = 12
    s = rng.random((2, 2, Nb, Nb)).astype(np.float32) ** 6
    s /= s.sum(-1, keepdims=True)
    tau = np.array([0.5, 0.6], np.float32)
    base, _, _ = oracle.topp(s, tau)
    m, idx, cnt = oracle.topp(s, tau, n_always_kv=2, n_dense_q=1)
    assert np.all(m[:, :, 0] == 1) and np.all(m[..., :2] == 1)
    assert np.array_equal(m[:, :, 1:, 2:], base[:, :, 1:, 2:])  # top-p itself unchanged
    assert np.array_equal(cnt, m.sum(-1))
    m5, _, c5 = oracle.topp(s, tau, min_keep=5)
    assert np.all(c5 >= 5) and np.all(m5 >= base)
    # reused heads keep whatever the buffers held
    mask = np.full((2, 2, Nb, Nb), 7, np.uint8)
    kidx = np.full((2, 2, Nb, Nb), -5, np.int32)
    kcnt = np.full((2, 2, Nb), -3, np.int32)
    refresh = np.array([[1, 0], [0, 1]], np.uint8)
    oracle.topp(s, tau, refresh=refresh, mask=mask, kept_idx=kidx, kept_count=kcnt)
    assert np.all(mask[0, 1] == 7) and np.all(kidx[1, 0] == -5) and np.all(kcnt[0, 1] == -3)
    assert np.array_equal(mask[0, 0], base[0, 0]) and np.array_equal(mask[1, 1], base[1, 1])


# --------------------------------------------------------------------------- attention
def _np_attention(q, k, v, keep_tok=None):
    """Textbook softmax(QK^T/sqrt(D))V in float64 with an optional token mask."""
    D = q.shape[-1]
    s = np.einsum("bhnd,bhmd->bhnm", q, k) / np.sqrt(D)
    if keep_tok is not None:
        s = np.where(keep_tok, s, -np.inf)
    s = s - s.max(-1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(-1, keepdims=True)
    return np.einsum("bhnm,bhmd->bhnd", p, v)


def _rand_qkv(rng, B, H, N, D, scale=1.0):
    return [bf16_bits((rng.standard_normal((B, H, N, D)) * scale).astype(np.float32))
            for _ in range(3)]


def test_attn_all_blocks_equals_dense_bruteforce_and_numpy():
    g = make_generator("tiny")
    st = g.step(0)
    q, k, v = as_u16(st.q), as_u16(st.k), as_u16(st.v)
    cfg = g.cfg
    qblk, _ = oracle.pool(q, cfg.block)
    kblk, _ = oracle.pool(k, cfg.block)
    p = oracle.scores(qblk, kblk)
    m, idx, cnt = oracle.topp(p, np.ones(cfg.H, np.float32))  # p = 1.0: the dense value
    assert np.all(m == 1)
    out = oracle.attn(q, k, v, cfg.block, idx, cnt)
    dense = oracle.dense_attn(q, k, v)
    assert np.allclose(out, dense, rtol=1e-6, atol=1e-7)
    ref = _np_attention(bf16_vals(q), bf16_vals(k), bf16_vals(v))
    assert np.allclose(dense, ref, rtol=1e-5, atol=1e-6)


def test_attn_masked_matches_numpy_on_ragged_blocks():
    rng = np.random.default_rng(4)
    B, H, N, D, block = 1, 2, 150, 32, 64  # blocks of 64, 64, 22 tokens
    q, k, v = _rand_qkv(rng, B, H, N, D)
    Nb = 3
    mask = np.array([[[1, 0, 1], [0, 1, 0], [1, 1, 0]], [[0, 0, 1], [1, 1, 1], [0, 1, 1]]],
                    np.uint8).reshape(B, H, Nb, Nb)
    idx = np.zeros((B, H, Nb, Nb), np.int32)
    cnt = mask.sum(-1).astype(np.int32)
    for h in range(H):
        for i in range(Nb):
            js = np.flatnonzero(mask[0, h, i])
            idx[0, h, i, :len(js)] = js
    out, lse = oracle.attn(q, k, v, block, idx, cnt, want_lse=True)
    tok = np.repeat(np.repeat(mask, block, axis=2), block, axis=3)[:, :, :N, :N].astype(bool)
    ref = _np_attention(bf16_vals(q), bf16_vals(k), bf16_vals(v), tok)
    assert np.allclose(out, ref, rtol=1e-5, atol=1e-6)
    s = np.einsum("bhnd,bhmd->bhnm", bf16_vals(q), bf16_vals(k)) / np.sqrt(D)
    s = np.where(tok, s, -np.inf)
    ref_lse = np.log(np.exp(s - s.max(-1, keepdims=True)).sum(-1)) + s.max(-1)
    assert np.allclose(lse, ref_lse, rtol=1e-5, atol=1e-5)
    # rows are convex combinations of V rows
    vv = bf16_vals(v)
    assert np.all(out <= vv.max(axis=2, keepdims=True) + 1e-6)
    assert np.all(out >= vv.min(axis=2, keepdims=True) - 1e-6)


def test_attn_single_block_and_qblock_subset():
    rng = np.random.default_rng(9)
    B, H, N, D, block = 1, 1, 128, 16, 32
    q, k, v = _rand_qkv(rng, B, H, N, D)
    Nb = 4
    idx = np.zeros((B, H, Nb, Nb), np.int32)
    idx[..., 0] = 2  # every query block sees key block 2 only
    cnt = np.ones((B, H, Nb), np.int32)
    out = oracle.attn(q, k, v, block, idx, cnt)
    ref = _np_attention(bf16_vals(q), bf16_vals(k)[:, :, 64:96], bf16_vals(v)[:, :, 64:96])
    assert np.allclose(out, ref, rtol=1e-5, atol=1e-6)
    sub = oracle.attn(q, k, v, block, idx, cnt, qblocks=[1, 3])
    assert np.array_equal(sub[:, :, 32:64], out[:, :, 32:64])
    assert np.array_equal(sub[:, :, 96:], out[:, :, 96:])
    assert np.all(np.isnan(sub[:, :, :32])) and np.all(np.isnan(sub[:, :, 64:96]))


def test_attn_custom_scale():
    rng = np.random.default_rng(10)
    q, k, v = _rand_qkv(rng, 1, 1, 64, 16)
    idx = np.zeros((1, 1, 1, 1), np.int32)
    cnt = np.ones((1, 1, 1), np.int32)
    out = oracle.attn(q, k, v, 64, idx, cnt, scale=0.5)
    # scale 0.5 with D=16 equals default scale on Q multiplied by 2 (exact in bf16)
    q2 = bf16_bits(bf16_vals(q).astype(np.float32) * 2)
    out2 = oracle.attn(q2, k, v, 64, idx, cnt)
    assert np.allclose(out, out2, rtol=1e-6, atol=1e-7)


# --------------------------------------------------------------------------- whole path
def test_tiny_config_end_to_end_sanity():
    """Reuse on the quiet head, refresh on the noisy one (with delta = 0.3; under
    the config's own delta = 0.05 both heads refresh, as the summed L1 predicts)."""
    g = make_generator("tiny")
    cfg = g.cfg
    s0, s1 = g.step(0), g.step(1)
    means = []
    for st in (s0, s1):
        _, qm = oracle.pool(as_u16(st.q), cfg.block)
        _, km = oracle.pool(as_u16(st.k), cfg.block)
        means.append((qm, km))
    for delta, want in ((0.05, [1, 1]), (0.3, [0, 1])):
        qa, ka, has = _state(1, 2, cfg.D)
        oracle.drift(means[0][0], means[0][1], qa, ka, has, np.full(2, delta, np.float32), 0.0, 1.0)
        d, r = oracle.drift(means[1][0], means[1][1], qa, ka, has,
                            np.full(2, delta, np.float32), 0.0, 1.0)
        assert r[0].tolist() == want, (delta, d)


def test_pooled_drift_against_the_full_token_drift_of_the_appendix():
    """App. query-key stability: the full-token drift d (mean over tokens of the L1 change of q
    plus that of k) bounds the mean change of the scaled logits by max(B_q, B_k) / sqrt(D) * d
    (Hoelder), and the online proxy (L1 distance of the token means) can only be smaller than d
    (triangle inequality) -- with equality when every token moves by the same vector.  Pins
    pool + drift together against quantities computed token by token in numpy."""
    rng = np.random.default_rng(5)
    N, D, blk = 300, 64, 64
    qa = bf16_vals(bf16_bits(rng.standard_normal((1, 1, N, D))))
    ka = bf16_vals(bf16_bits(rng.standard_normal((1, 1, N, D))))
    qb = bf16_vals(bf16_bits(qa + 0.25 * rng.standard_normal((1, 1, N, D))))
    kb = bf16_vals(bf16_bits(ka + 0.25 * rng.standard_normal((1, 1, N, D))))

    def proxy(q0, k0, q1, k1):
        _, qm0 = oracle.pool(bf16_bits(q0), blk)
        _, km0 = oracle.pool(bf16_bits(k0), blk)
        _, qm1 = oracle.pool(bf16_bits(q1), blk)
        _, km1 = oracle.pool(bf16_bits(k1), blk)
        has = np.ones((1, 1), np.uint8)
        d, _ = oracle.drift(qm1, km1, qm0.copy(), km0.copy(), has, np.zeros(1, np.float32), 0.0, 1.0,
                            commit=False)
        return float(d[0, 0])

    dq, dk = qb - qa, kb - ka
    full = np.abs(dq[0, 0]).sum(axis=1).mean() + np.abs(dk[0, 0]).sum(axis=1).mean()
    d_proxy = proxy(qa, ka, qb, kb)
    assert 0.0 < d_proxy <= full * (1 + 1e-6)
    assert d_proxy < 0.5 * full          # iid changes average out in the token mean
    # the Hoelder bound on the mean logit change (ties the full-token drift to what it is for)
    ga = qa[0, 0] @ ka[0, 0].T / np.sqrt(D)
    gb = qb[0, 0] @ kb[0, 0].T / np.sqrt(D)
    bq = max(np.abs(qa).max(), np.abs(qb).max())
    bk = max(np.abs(ka).max(), np.abs(kb).max())
    assert np.abs(gb - ga).mean() <= max(bq, bk) / np.sqrt(D) * full
    # a common offset: proxy == full-token drift (values chosen exactly representable in bf16)
    cq = np.zeros(D); cq[::2] = 0.5; cq[1::4] = -0.25
    ck = np.zeros(D); ck[::3] = 1.0
    q0 = np.round(qa * 8) / 8
    k0 = np.round(ka * 8) / 8
    q1, k1 = q0 + cq, k0 + ck
    full_c = np.abs(cq).sum() + np.abs(ck).sum()
    assert abs(proxy(q0, k0, q1, k1) - full_c) <= 1e-5 * full_c
    # and it is the SUM of the two terms: moving only the keys gives only the key term
    assert abs(proxy(q0, k0, q0, k1) - np.abs(ck).sum()) <= 1e-5 * full_c


def test_drift_and_mask_stability_are_negatively_related():
    """Sec. 4.1 / 4.2 (the observation TMR rests on): heads whose pooled Q/K features have drifted
    more from the anchor step have masks that overlap less with the anchor mask.  Sign only:
    Spearman rank correlation between drift and mask IoU over (head, step) pairs is negative."""
    import dataclasses

    from scipy.stats import spearmanr

    from heart_synth import CONFIGS, HeartInputGenerator

    cfg = dataclasses.replace(CONFIGS["small_ragged"], name="small_ragged_obs", steps=6, H=6, seed=21)
    g = HeartInputGenerator(cfg)
    st0 = g.step(0)
    qb0, qm0 = oracle.pool(as_u16(st0.q), cfg.block)
    kb0, km0 = oracle.pool(as_u16(st0.k), cfg.block)
    m0, _, _ = oracle.topp(oracle.scores(qb0, kb0), g.tau)
    drifts, ious = [], []
    for s in range(1, cfg.steps):
        st = g.step(s)
        qb, qm = oracle.pool(as_u16(st.q), cfg.block)
        kb, km = oracle.pool(as_u16(st.k), cfg.block)
        has = np.ones((cfg.B, cfg.H), np.uint8)
        d, _ = oracle.drift(qm, km, qm0.copy(), km0.copy(), has, g.delta, 0.0, 1.0, commit=False)
        m, _, _ = oracle.topp(oracle.scores(qb, kb), g.tau)
        inter = (m & m0).sum(axis=(2, 3)).astype(np.float64)
        union = (m | m0).sum(axis=(2, 3)).astype(np.float64)
        drifts.append(d.reshape(-1))
        ious.append((inter / union).reshape(-1))
    rho, _ = spearmanr(np.concatenate(drifts), np.concatenate(ious))
    assert rho < -0.3, rho
