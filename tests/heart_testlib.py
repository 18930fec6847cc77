"""Helpers shared by the GPU parity tests (no method arithmetic here: every expected value
comes from the `oracle` package)."""
import numpy as np
import torch

import oracle
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


def check_attn_plan(ws, cnt, Nb):
    """Validate the launch plan heart_block_sparse_attn leaves in its workspace.

    ws: int32 workspace after the call (numpy); cnt: kept counts [B,H,Nb].  Layout: 8 cursors,
    8 list lengths (items), 8 offsets into the head table, the head table (heads of XCD 0 in
    the order it walks them, then XCD 1, ...), the total kept count per head, then per head its
    items in launch order.  Heads go to the least loaded XCD, heaviest first (load = kept count
    + Nb per head); inside a head the items are sorted by count class, longest first, stable."""
    BH = cnt.shape[0] * cnt.shape[1]
    n = BH * Nb
    c = np.clip(cnt.reshape(BH, Nb).astype(np.int64), 0, Nb)
    w = c.sum(1)
    order = sorted(range(BH), key=lambda h: (-w[h], h))
    load = [0] * 8
    shift = 0
    while (BH * Nb * (Nb + 1)) >> shift > 0x3fffffff:
        shift += 1
    heads = [[] for _ in range(8)]
    for h in order:
        x = min(range(8), key=lambda x: (load[x], x))
        heads[x].append(h)
        load[x] += (int(w[h]) + Nb) >> shift
    lens = np.array([len(hs) * Nb for hs in heads])
    offs = np.concatenate([[0], np.cumsum([len(hs) for hs in heads])[:-1]])
    assert np.array_equal(ws[8:16], lens), "list lengths"
    assert np.array_equal(ws[16:24], offs), "head table offsets"
    assert (ws[0:8] >= lens).all(), "every list was drained"
    assert np.array_equal(ws[24:24 + BH], np.concatenate([np.array(hs, np.int64) for hs in heads])), "head table"
    assert np.array_equal(ws[24 + BH:24 + 2 * BH], w), "head totals"
    seq = ws[24 + 2 * BH:24 + 2 * BH + n]
    mult = (31 << 16) // Nb
    classes = 31 - ((c * mult) >> 16)
    for h in range(BH):
        want = h * Nb + np.argsort(classes[h], kind="stable")
        assert np.array_equal(seq[h * Nb:(h + 1) * Nb], want), f"items of head {h}"


def attn_atol(want: np.ndarray) -> float:
    """Bound on |out - exact| for bf16 outputs: the 2e-2 of unit-scale outputs, growing with the
    output's magnitude beyond 2 (an output of magnitude m is rounded to bf16 with an error of up
    to 2^-9 m, and the rounded softmax weights contribute as much again)."""
    return ATTN_ATOL * max(1.0, float(np.nanmax(np.abs(want))) / 2.0)


def sample_query_blocks(rng, Nb: int, n_text_blocks: int, n: int = 32):
    """At least n query blocks (all of them when Nb <= n): block 0, the (possibly ragged) last
    block, the text blocks, and seeded random ones."""
    fixed = sorted(set([0, Nb - 1] + list(range(min(n_text_blocks, Nb)))))
    if Nb <= n:
        return list(range(Nb))
    rest = [i for i in rng.permutation(Nb).tolist() if i not in fixed]
    return sorted(fixed + rest[:n - len(fixed)])


def pooled_mean_score_shift(osc: np.ndarray, qblk_gpu, kblk_gpu) -> np.ndarray:
    """How far the GPU's own block means (equal to the oracle's within the pooling tolerance)
    can move the scores of a row: the largest relative change, per row [B,H,Nb], between the
    oracle's scores on the oracle's block means (osc) and the oracle's scores on the GPU's."""
    osc2 = oracle.scores(qblk_gpu.detach().cpu().numpy(), kblk_gpu.detach().cpu().numpy())
    big = osc >= SCORE_QUANTUM
    rel = np.where(big, np.abs(osc2.astype(np.float64) - osc) / np.where(big, osc, 1.0), 0.0)
    return rel.max(-1)


def assert_masks_equal_up_to_threshold(gmask, omask, osc, ocnt, tau, what: str,
                                       tol: float = SCORE_RTOL, row_tol=None):
    """GPU-chained masks may differ from the oracle's only in rows whose cumulative mass passes
    within the score tolerance of the threshold: every score agrees within `tol` relative, so
    a normalised cumulative mass (a sum of scores) moves by at most `tol`.  `row_tol` [B,H,Nb]
    adds what the caller has measured on the oracle's side for inputs that are themselves only
    equal within a tolerance (pooled_mean_score_shift).  Returns the boolean [B,H,Nb] 'row is
    equal'."""
    gmask = gmask.cpu().numpy() if isinstance(gmask, torch.Tensor) else gmask
    B, H, Nb, _ = omask.shape
    diff = (gmask != omask).any(-1)
    for (b, h, i) in np.argwhere(diff):
        p = osc[b, h, i].astype(np.float64)
        order = np.argsort(-p, kind="stable")
        cum = np.cumsum(p[order]) / p.sum()
        kk = min(int(ocnt[b, h, i]), Nb) - 1
        t = tol + (0.0 if row_tol is None else float(row_tol[b, h, i]))
        assert abs(cum[kk] - tau[h]) < t or abs(cum[max(kk - 1, 0)] - tau[h]) < t, \
            (f"{what}: mask row {(b, h, i)} differs away from the threshold "
             f"(mass {cum[kk]:.7f} / {cum[max(kk - 1, 0)]:.7f}, tau {tau[h]:.7f}, tolerance {t:.1e})")
    assert diff.sum() <= max(1, 0.01 * B * H * Nb), f"{what}: {diff.sum()} rows differ"
    return ~diff


class OracleChain:
    """The oracle's side of a chained run: caller-owned TMR state (anchors, cached mask and
    lists) carried from step to step through the oracle's single-step functions, in the order
    of Alg. 1."""

    def __init__(self, cfg, tau, delta, gate=(0.4, 0.8)):
        B, H, D, Nb = cfg.B, cfg.H, cfg.D, cfg.Nb
        self.cfg, self.tau, self.delta, self.gate = cfg, tau, delta, gate
        self.qa = np.zeros((B, H, D), np.float32)
        self.ka = np.zeros((B, H, D), np.float32)
        self.has = np.zeros((B, H), np.uint8)
        self.mask = np.zeros((B, H, Nb, Nb), np.uint8)
        self.idx = np.zeros((B, H, Nb, Nb), np.int32)
        self.cnt = np.zeros((B, H, Nb), np.int32)

    def step(self, st):
        """st: StepInputs (CPU bf16).  Returns drift, refresh and the scores of this step; mask,
        idx, cnt are updated in place for refreshed heads."""
        cfg = self.cfg
        nt = cfg.n_text_blocks
        self.qblk, qm = oracle.pool(u16(st.q), cfg.block)
        self.kblk, km = oracle.pool(u16(st.k), cfg.block)
        d, r = oracle.drift(qm, km, self.qa, self.ka, self.has, self.delta, *self.gate)
        self.scores = oracle.scores(self.qblk, self.kblk)
        oracle.topp(self.scores, self.tau, refresh=r, n_always_kv=nt, n_dense_q=nt, mask=self.mask,
                    kept_idx=self.idx, kept_count=self.cnt)
        return d, r
