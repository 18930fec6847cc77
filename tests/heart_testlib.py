"""Helpers shared by the GPU parity tests (no method arithmetic here)."""
import numpy as np
import torch

from heart_synth import as_u16

SCORE_RTOL = 1e-5          # spec tolerance on block scores (relative)
SCORE_QUANTUM = 2.0 ** -30  # mass quantum of the top-p fixed point
ATTN_ATOL = 2e-2           # spec tolerance on attention outputs (max-abs, bf16 I/O)
MEAN_RTOL = 1e-5
# fp32 accumulation of <= 128 bf16 values plus 32 partial sums: error below
# 2^-24 * (8 + 32) * mean|x| < 3e-6 * max|x|; used as the absolute floor where a
# mean cancels to (nearly) zero and a relative bound is meaningless
MEAN_ATOL_FACTOR = 3e-6


def gpu(t: torch.Tensor) -> torch.Tensor:
    return t.to("cuda", non_blocking=False)


def np_gpu(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def assert_means_close(got: torch.Tensor, want: np.ndarray, x_absmax: float, what: str):
    g = got.detach().cpu().numpy().astype(np.float64)
    w = want.astype(np.float64)
    err = np.abs(g - w)
    bound = MEAN_RTOL * np.abs(w) + MEAN_ATOL_FACTOR * x_absmax
    bad = err > bound
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, max err {err.max():.3e}"


def assert_scores_close(got: torch.Tensor, want: np.ndarray, what: str):
    g = got.detach().cpu().numpy().astype(np.float64)
    w = want.astype(np.float64)
    big = w >= SCORE_QUANTUM
    rel = np.abs(g - w)[big] / w[big]
    assert rel.size == 0 or rel.max() <= SCORE_RTOL, f"{what}: max rel err {rel.max():.3e}"
    assert np.all(g[~big] < 2 * SCORE_QUANTUM), f"{what}: sub-quantum score too large"
    return float(rel.max()) if rel.size else 0.0


def assert_lists_equal(mask, kept_idx, kept_count, o_mask, o_idx, o_cnt, what: str, heads=None):
    """Bit-exact comparison of mask, counts and the valid prefix of the index lists."""
    m = mask.cpu().numpy()
    ki = kept_idx.cpu().numpy()
    kc = kept_count.cpu().numpy()
    if heads is not None:
        sel = np.zeros(m.shape[:2], bool)
        sel[heads] = True
    else:
        sel = np.ones(m.shape[:2], bool)
    assert np.array_equal(m[sel], o_mask[sel]), f"{what}: mask differs"
    assert np.array_equal(kc[sel], o_cnt[sel]), f"{what}: kept_count differs"
    Nb = m.shape[-1]
    valid = np.arange(Nb)[None, None, None, :] < o_cnt[..., None]
    valid &= sel[:, :, None, None]
    assert np.array_equal(ki[valid], o_idx[valid]), f"{what}: kept_idx differs"


def u16(t: torch.Tensor) -> np.ndarray:
    return as_u16(t.cpu())
