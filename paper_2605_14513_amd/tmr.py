"""Multi-step, multi-layer Temporal Mask Reuse on top of the four libheart calls.

The library is stateless; the state of TMR -- anchor features, `has_anchor`, the cached block
mask and its kept-block lists -- belongs to the caller, one set per (layer, classifier-free-
guidance branch) as in the paper's cache (Sec. 4.2).  This module owns that state for a stack
of attention layers and sequences the calls of one attention invocation:

    heart   pool + drift, token means and drift sharing a launch (reuse rule + layer gate, Alg. 1) -> mask for refreshed heads -> attention
    always  pool -> mask for every head -> attention              (no reuse)
    interval:k   every head refreshes on every k-th sparse step, otherwise every head reuses
                 (the shared fixed-interval schedule the paper compares with, Sec. 5 ablations)
    warmup:w     every head refreshes during the first w sparse steps, then every head reuses
                 (the shared "switch to reuse after a preset step" schedule, same ablation)

The first `dense_steps` denoising steps run dense attention (Experimental Setup: all
experiments keep the first five steps dense); they neither read nor write the cache.

Block importance comes from the pooled scores inside heart_mask_topp (`estimator="pooled"`) or
from the antidiagonal-style estimator (`estimator="antidiag"`: heart_scores_antidiag, then
heart_mask_topp on its scores); the latter is computed for refreshed heads only, so what a
reused mask saves includes the estimator.

Only call sequencing and the shared schedules live here; every array operation of the path is
a libheart kernel.  Policies other than `heart` skip pooling on steps where nothing refreshes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import torch

from . import binding as _b

# Above this many key blocks per row heart_mask_topp is called with a workspace (measured on
# MI355X: 42 against 38 us at Nb = 256, 113 against 139 at 591, 150 against 249 at 931).
SLICED_SCORES_MIN_NB = 256

__all__ = ["TmrConfig", "TmrState", "TmrDriver"]


@dataclass
class TmrConfig:
    B: int
    H: int
    N: int
    D: int
    block: int
    tau: torch.Tensor            # [H] fp32 on the GPU: per-head top-p thresholds
    delta: torch.Tensor          # [H] fp32 on the GPU: drift thresholds
    policy: str = "heart"        # "heart" | "always" | "interval:<k>" | "warmup:<w>"
    estimator: str = "pooled"    # "pooled" | "antidiag" (stride = block / 8)
    gate: Tuple[float, float] = (0.4, 0.8)
    dense_steps: int = 5
    n_always_kv_blocks: int = 0
    n_dense_q_blocks: int = 0
    min_keep: int = 1

    @property
    def Nb(self) -> int:
        return (self.N + self.block - 1) // self.block


@dataclass
class TmrState:
    """Cache of one (layer, branch): anchors and the cached mask in its three forms."""
    qanchor: torch.Tensor
    kanchor: torch.Tensor
    has_anchor: torch.Tensor
    refresh: torch.Tensor        # decision of the last sparse call, uint8 [B,H]
    drift: torch.Tensor
    mask: torch.Tensor
    kept_idx: torch.Tensor
    kept_count: torch.Tensor
    sparse_calls: int = 0        # sparse (non-warm-up) calls seen so far


@dataclass
class TmrCallRecord:
    layer: int
    branch: int
    step: int
    kind: str                    # "dense" | "refresh" | "reuse" | "heart"
    refresh: Optional[torch.Tensor] = None   # device copy of the per-head decisions
    events: List[torch.cuda.Event] = field(default_factory=list)  # pool, drift, mask, attn bounds


class TmrDriver:
    def __init__(self, cfg: TmrConfig, n_layers: int, n_branches: int = 2, device="cuda",
                 record: bool = False, time_kernels: bool = False):
        _b.load_library()
        self.cfg = cfg
        self.device = torch.device(device)
        self.record = record
        self.time_kernels = time_kernels
        self.records: List[TmrCallRecord] = []
        B, H, D, Nb = cfg.B, cfg.H, cfg.D, cfg.Nb
        f32 = dict(dtype=torch.float32, device=self.device)
        self.policy, self.policy_arg = self._parse_policy(cfg.policy)
        # scratch shared by all layers (a call consumes it before the next one starts)
        self.qblk = torch.empty((B, H, Nb, D), **f32)
        self.kblk = torch.empty((B, H, Nb, D), **f32)
        self.qmean = torch.empty((B, H, D), **f32)
        self.kmean = torch.empty((B, H, D), **f32)
        self.workspace: Optional[torch.Tensor] = None
        # completion tickets of the fused pooling + drift launch (zero now, zero after every call)
        self.tickets = torch.zeros(_b.heart_pool_drift_workspace_bytes(B, H), dtype=torch.uint8,
                                   device=self.device)
        if cfg.estimator not in ("pooled", "antidiag"):
            raise ValueError(f"unknown importance estimator {cfg.estimator!r}")
        # workspace of heart_mask_topp_ws (score stage on 8-bit slices of the block means): one
        # launch more and a several times faster score stage, which pays for long rows only
        self.topp_ws: Optional[torch.Tensor] = None
        if cfg.estimator == "pooled" and Nb > SLICED_SCORES_MIN_NB and D in (64, 128):
            self.topp_ws = torch.empty(_b.heart_mask_topp_workspace_bytes(B, H, Nb, D),
                                       dtype=torch.uint8, device=self.device)
        # scores and records of the antidiagonal-style estimator, shared by all layers
        self.scores: Optional[torch.Tensor] = None
        self.estimator_ws: Optional[torch.Tensor] = None
        if cfg.estimator == "antidiag":
            self.scores = torch.zeros((B, H, Nb, Nb), **f32)
        # dense lists for the warm-up steps, shared by all layers
        ar = torch.arange(Nb, dtype=torch.int32, device=self.device)
        self.dense_idx = ar.expand(B, H, Nb, Nb).contiguous()
        self.dense_cnt = torch.full((B, H, Nb), Nb, dtype=torch.int32, device=self.device)
        self.states: Dict[Tuple[int, int], TmrState] = {}
        for layer in range(n_layers):
            for br in range(n_branches):
                self.states[(layer, br)] = TmrState(
                    qanchor=torch.zeros((B, H, D), **f32), kanchor=torch.zeros((B, H, D), **f32),
                    has_anchor=torch.zeros((B, H), dtype=torch.uint8, device=self.device),
                    refresh=torch.zeros((B, H), dtype=torch.uint8, device=self.device),
                    drift=torch.zeros((B, H), **f32),
                    mask=torch.zeros((B, H, Nb, Nb), dtype=torch.uint8, device=self.device),
                    kept_idx=torch.zeros((B, H, Nb, Nb), dtype=torch.int32, device=self.device),
                    kept_count=torch.zeros((B, H, Nb), dtype=torch.int32, device=self.device))

    @staticmethod
    def _parse_policy(p: str) -> Tuple[str, int]:
        if p in ("heart", "always"):
            return p, 0
        name, _, arg = p.partition(":")
        if name in ("interval", "warmup") and arg.isdigit() and int(arg) >= 1:
            return name, int(arg)
        raise ValueError(f"unknown TMR policy {p!r}")

    def reset(self) -> None:
        """Forget every cache (start of a new generation)."""
        for st in self.states.values():
            st.has_anchor.zero_()
            st.sparse_calls = 0
        self.records.clear()

    def _shared_schedule_refreshes(self, sparse_call: int) -> bool:
        if self.policy == "always":
            return True
        if self.policy == "interval":
            return sparse_call % self.policy_arg == 0
        if self.policy == "warmup":
            return sparse_call < self.policy_arg
        raise AssertionError(self.policy)

    def attention(self, layer: int, branch: int, step: int, q, k, v, out=None):
        """One attention call of `layer` / `branch` at denoising step `step` (0-based)."""
        cfg = self.cfg
        st = self.states[(layer, branch)]
        if out is None:
            out = torch.empty_like(q)
        if self.workspace is None:
            self.workspace = torch.empty(_b.heart_attn_workspace_bytes(q, cfg.block),
                                         dtype=torch.uint8, device=self.device)
        if self.scores is not None and self.estimator_ws is None:
            self.estimator_ws = torch.empty(
                _b.heart_scores_antidiag_workspace_bytes(q, cfg.block, cfg.block // 8),
                dtype=torch.uint8, device=self.device)
        ev: List[torch.cuda.Event] = []

        def refresh_mask(refresh):
            """Importance scores and top-p lists of the heads in `refresh` (None = all)."""
            if self.scores is None:
                _b.heart_mask_topp(self.qblk, self.kblk, cfg.tau, refresh=refresh,
                                   n_always_kv_blocks=cfg.n_always_kv_blocks,
                                   n_dense_q_blocks=cfg.n_dense_q_blocks, min_keep=cfg.min_keep,
                                   mask=st.mask, kept_idx=st.kept_idx, kept_count=st.kept_count,
                                   workspace=self.topp_ws)
            else:
                _b.heart_scores_antidiag(q, k, cfg.block, cfg.block // 8, scores=self.scores,
                                         workspace=self.estimator_ws, refresh=refresh)
                _b.heart_mask_topp(None, None, cfg.tau, scores_in=self.scores, refresh=refresh,
                                   n_always_kv_blocks=cfg.n_always_kv_blocks,
                                   n_dense_q_blocks=cfg.n_dense_q_blocks, min_keep=cfg.min_keep,
                                   mask=st.mask, kept_idx=st.kept_idx, kept_count=st.kept_count)

        def mark():
            if self.time_kernels:
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                ev.append(e)

        rec_refresh = None
        mark()
        if step < cfg.dense_steps:
            kind = "dense"
            mark(); mark(); mark()
            _b.heart_block_sparse_attn(q, k, v, cfg.block, self.dense_idx, self.dense_cnt, out=out,
                                       workspace=self.workspace)
        else:
            if self.policy == "heart":
                kind = "heart"
                # pooling pass, then token means + drift + reuse rule + gate in one launch
                _b.heart_pool_drift(q, k, cfg.block, st.qanchor, st.kanchor, st.has_anchor, cfg.delta,
                                    self.tickets, cfg.gate[0], cfg.gate[1], True, self.qblk, self.kblk,
                                    self.qmean, self.kmean, st.drift, st.refresh)
                mark()
                mark()
                refresh_mask(st.refresh)
                mark()
                if self.record:
                    rec_refresh = st.refresh.clone()
            elif self._shared_schedule_refreshes(st.sparse_calls):
                kind = "refresh"
                if self.scores is None:  # (the antidiagonal estimator reads q and k itself)
                    _b.heart_pool_qk(q, k, cfg.block, self.qblk, self.kblk, self.qmean, self.kmean)
                mark(); mark()
                refresh_mask(None)
                mark()
            else:
                kind = "reuse"
                mark(); mark(); mark()
            st.sparse_calls += 1
            _b.heart_block_sparse_attn(q, k, v, cfg.block, st.kept_idx, st.kept_count, out=out,
                                       workspace=self.workspace)
        mark()
        if self.record or self.time_kernels:
            self.records.append(TmrCallRecord(layer, branch, step, kind, rec_refresh, ev))
        return out

    # ---- reporting (synchronises) ---------------------------------------------------------
    def summary(self) -> dict:
        """Refresh counts and kernel times over the recorded calls."""
        torch.cuda.synchronize()
        H, B = self.cfg.H, self.cfg.B
        sparse = [r for r in self.records if r.kind != "dense"]
        refreshed_heads = 0.0
        for r in sparse:
            if r.kind == "heart":
                refreshed_heads += float(r.refresh.float().sum().item()) if r.refresh is not None else 0.0
            elif r.kind == "refresh":
                refreshed_heads += B * H
        out = {
            "policy": self.cfg.policy,
            "calls": len(self.records),
            "dense_calls": len(self.records) - len(sparse),
            "sparse_calls": len(sparse),
            "refreshed_head_fraction": refreshed_heads / max(1, len(sparse) * B * H),
        }
        if self.time_kernels and self.records:
            names = ["pool_us", "drift_us", "mask_us", "attn_us"]
            tot = {n: 0.0 for n in names}
            for r in sparse:
                for i, n in enumerate(names):
                    tot[n] += r.events[i].elapsed_time(r.events[i + 1]) * 1e3
            for n in names:
                out[n + "_per_sparse_call"] = tot[n] / max(1, len(sparse))
            out["mask_refresh_us_per_sparse_call"] = (tot["pool_us"] + tot["drift_us"] + tot["mask_us"]) / max(1, len(sparse))
            dense = [r for r in self.records if r.kind == "dense"]
            if dense:
                out["dense_attn_us_per_call"] = sum(
                    r.events[3].elapsed_time(r.events[4]) * 1e3 for r in dense) / len(dense)
        return out
