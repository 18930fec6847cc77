"""heart_ebc_band_error (GPU, transform-free) against the oracle's 3D-FFT definition of Eq. 6,
on tensors shaped like latent velocities (channels x frames x height x width) with odd, even
and ragged axis lengths, and the end-to-end calibration of per-head thresholds on the tiny
workload: errors measured with the library's own sparse attention, thresholds selected under
the sparsity budget of the shared threshold."""
import numpy as np
import pytest
import torch

import oracle
from oracle import ebc_oracle as eo
from heart_synth import make_generator
from heart_testlib import gpu, np_gpu, u16

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape", [(1, 4, 4, 4), (3, 5, 6, 7), (16, 21, 30, 52), (2, 1, 9, 8), (2, 8, 1, 3), (1, 33, 45, 80)])
def test_band_error_matches_fft_definition(shape):
    import paper_2605_14513_amd as heart

    rng = np.random.default_rng(sum(shape))
    C, T, Y, X = shape
    t, y, x = np.meshgrid(np.arange(T), np.arange(Y), np.arange(X), indexing="ij")
    # smooth structure plus noise, so that every band carries energy of a different size
    dense = (np.sin(2 * np.pi * (t / T + 2 * y / Y)) + 0.3 * rng.standard_normal(shape)).astype(np.float32)
    err = (0.05 * np.cos(2 * np.pi * (x / X + t / T)) + 0.01 * rng.standard_normal(shape)).astype(np.float32)
    got = heart.heart_ebc_band_error(np_gpu(err), np_gpu(dense)).cpu().numpy()
    want_bands = eo.band_energies(err)
    want = eo.band_error(err, dense)
    tot = want_bands.sum()
    assert np.allclose(got[1:5], want_bands, rtol=1e-9, atol=1e-12 * tot), (got[1:5], want_bands)
    assert np.isclose(got[0], want, rtol=1e-9), (got[0], want)
    assert np.isclose(got[5], T * Y * X * (dense.astype(np.float64) ** 2).sum(), rtol=1e-12)
    # other weights and epsilon; reproducible bits
    w = (0.3, 2.0, 1.0, 0.0)
    got2 = heart.heart_ebc_band_error(np_gpu(err), np_gpu(dense), weights=w, epsilon=3.0).cpu().numpy()
    assert np.isclose(got2[0], eo.band_error(err, dense, weights=w, epsilon=3.0), rtol=1e-9)
    again = heart.heart_ebc_band_error(np_gpu(err), np_gpu(dense)).cpu().numpy()
    assert np.array_equal(again, got)


def test_band_error_single_frequencies_and_zero_reference():
    import paper_2605_14513_amd as heart

    T, Y, X = 8, 8, 12
    t, y, x = np.meshgrid(np.arange(T), np.arange(Y), np.arange(X), indexing="ij")
    zero = torch.zeros((1, T, Y, X), device="cuda")
    for (ft, fy, fx), band in (((1, 2, 3), 0), ((0, 0, 4), 1), ((3, 0, 0), 2), ((4, 0, 6), 3)):
        wave = np.cos(2 * np.pi * (ft * t / T + fy * y / Y + fx * x / X)).astype(np.float32)[None]
        got = heart.heart_ebc_band_error(np_gpu(wave), zero, epsilon=1.0).cpu().numpy()
        e = got[1:5]
        # (the fp32 rounding of the wave leaks about 1e-7 of its energy into the other bands)
        assert abs(e.sum() - e[band]) < 1e-6 * e.sum()
        assert np.isclose(got[0], np.dot(eo.BAND_WEIGHTS, e) / 1.0, rtol=1e-12)
        assert np.allclose(e, eo.band_energies(wave), rtol=1e-9, atol=1e-12 * e.sum())


def test_thresholds_calibrated_on_the_tiny_workload():
    """Sec. 4.3 end to end on synthetic tensors: per head and candidate threshold, the sparse
    attention output (this library) minus the dense one plays the sparse-induced error; its
    frequency-weighted error and realised sparsity fill the tables; the selection under the
    budget of the shared threshold never has more error than the shared threshold."""
    import paper_2605_14513_amd as heart

    g = make_generator("tiny")
    cfg = g.cfg
    st = g.step(0)
    B, H, N, D, Nb, blk = cfg.B, cfg.H, cfg.N, cfg.D, cfg.Nb, cfg.block
    T, Yg, Xg = cfg.grid
    q, k, v = gpu(st.q), gpu(st.k), gpu(st.v)
    qblk, kblk, _, _ = heart.heart_pool_qk(q, k, blk)
    cands = np.array([0.5, 0.7, 0.8, 0.9, 0.95, 1.0], np.float32)
    dense_tau = torch.ones(H, device="cuda")
    _, didx, dcnt = heart.heart_mask_topp(qblk, kblk, dense_tau)
    dense = heart.heart_block_sparse_attn(q, k, v, blk, didx, dcnt).float()
    E = np.zeros((H, len(cands))); S = np.zeros((H, len(cands)))
    oE = np.zeros_like(E)
    for ci, tau_c in enumerate(cands):
        tau = torch.full((H,), float(tau_c), device="cuda")
        _, idx, cnt = heart.heart_mask_topp(qblk, kblk, tau)
        out = heart.heart_block_sparse_attn(q, k, v, blk, idx, cnt).float()
        for h in range(H):
            # [B, N, D] of head h -> channels D (and B) over the (T, Y, X) token grid
            err_h = (out[:, h] - dense[:, h]).permute(0, 2, 1).reshape(B * D, T, Yg, Xg).contiguous()
            den_h = dense[:, h].permute(0, 2, 1).reshape(B * D, T, Yg, Xg).contiguous()
            E[h, ci] = heart.heart_ebc_band_error(err_h, den_h)[0].item()
            oE[h, ci] = eo.band_error(err_h.cpu().numpy(), den_h.cpu().numpy())
            S[h, ci] = 1.0 - cnt[:, h].float().sum().item() / (B * Nb * Nb)
    assert np.allclose(E, oE, rtol=1e-7, atol=1e-18)
    assert (E[:, -1] == 0).all() and (S[:, -1] == 0).all()     # p = 1 is the dense value
    assert (np.diff(S, axis=1) <= 1e-12).all()                  # larger threshold, less sparsity
    shared = 3  # the shared threshold 0.9
    budget = S[:, shared].mean()
    choice, total = heart.heart_ebc_select(E, S, budget)
    assert S[np.arange(H), choice].mean() >= budget - 1e-12
    assert total <= E[:, shared].sum() + 1e-15
    want_c, want_e = eo.select_bruteforce(E, S, budget)
    assert np.isclose(total, want_e, rtol=1e-12, atol=1e-18)
    print("calibrated thresholds", cands[choice], "error", total, "vs shared", E[:, shared].sum(), flush=True)
