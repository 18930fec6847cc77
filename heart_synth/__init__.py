"""Seeded synthetic inputs for the HEART sparse-attention hot path.

This module is shared by the CPU oracle's tests and by the HIP path's tests and
benchmark.  It holds *no* arithmetic of the method (no pooling, drift, scoring,
top-p or attention): it only manufactures bf16 Q/K/V tensors, per-head
thresholds and a per-step perturbation schedule with the shapes of the video
diffusion workloads the paper evaluates (Experimental Setup: Wan2.1 at 81
frames, HunyuanVideo at 129 frames; block size 128 from the appendix on
baseline configurations).  The tensors stand in for real activations, which
need model weights and prompts that are not available offline.

Recipe (all configs):
  token n of a (T, Hg, W) latent grid sits at (t, y, x); per head h four
  sinusoids r = 0..3 with integer frequency triples, phases and unit-scale
  directions u_r in R^D are drawn from numpy PCG64([seed, h]).  Q and K share
  the directions (so q.k is large where the phases agree, giving spatially and
  temporally structured attention), V uses directions of its own:
      X[n, :] = gain * sum_r sin(2 pi (f_t t/T + f_y y/Hg + f_x x/W) / ell_h + phi_r) u_r
                + N(0, 0.1^2)
  ell_h ("locality scale") stretches the field per head.  Values are rounded
  once to bf16; both the oracle and the GPU path consume those bf16 bits.
  Optional text tokens (HunyuanVideo-shaped config) are iid N(0, 0.3^2) rows
  prepended to the grid tokens.

Multi-step schedules: step s adds, per head, a common offset vector (which is
what moves the token mean) of scheduled L1 size, directed within the span of the
head's own sinusoid directions (so that it also changes the head's block scores), plus noise_std[s, h] times one
fixed iid N(0,1) field per (tensor, head).

The "jumps" schedule is laid out so that the share of heads whose features move far
from where they last jumped is between 40 % and 70 % at every step after the first:
inside the 30-70 % band the Wan2.1-14B-shaped benchmark configuration asks for, and
never below the 40 % at which the layer-level gate of the method (Sec. 4.2) would
turn a step into reuse for every head, so the same schedule serves runs with the gate
on and off.  `planned_jumps[s, h]` records the layout (step 0: every head, nothing is
cached yet); it is bookkeeping of this generator, not a decision of the method.

Per-head thresholds are drawn uniformly, except for the Wan2.1-14B-shaped 720P
configuration, which asks for a global kept-block density of 15 % "via per-head tau":
its thresholds are a stored table (wan14b_720p_tau.json beside this file, written by
oracle/make_density_tau.py from the CPU oracle's scores and top-p rule on step 0).
"""
from __future__ import annotations

import json
import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np
import torch

__all__ = [
    "HeartConfig",
    "CONFIGS",
    "get_config",
    "StepInputs",
    "make_generator",
    "HeartInputGenerator",
    "as_u16",
]


@dataclass(frozen=True)
class HeartConfig:
    """Shape and schedule of one synthetic workload."""

    name: str
    B: int
    H: int
    D: int
    grid: Tuple[int, int, int]  # (T, Hg, W) latent grid
    block: int
    seed: int
    n_text: int = 0  # text tokens prepended (always-kept blocks)
    steps: int = 2
    gain: float = 8.0
    # how per-head thresholds are drawn: ("list", [...]), ("uniform", lo, hi), or
    # ("file", name, lo, hi): a stored table beside this module (made from uniform draws
    # in [lo, hi] by the script the file names)
    tau_spec: tuple = ("uniform", 0.85, 0.98)
    delta: float = 1.0
    # schedule kind: "tiny" (iid noise per head), "loguniform" (one later step,
    # per-head magnitude log-uniform), "jumps" (per step a random 30-70 % of
    # heads receive a large offset, the rest a tiny one)
    schedule: str = "jumps"
    locality: Tuple[float, float] = (0.5, 4.0)

    @property
    def N(self) -> int:
        t, h, w = self.grid
        return self.n_text + t * h * w

    @property
    def Nb(self) -> int:
        return (self.N + self.block - 1) // self.block

    @property
    def n_text_blocks(self) -> int:
        return self.n_text // self.block


CONFIGS: Dict[str, HeartConfig] = {
    # the five benchmark configurations, smallest first: (1) tiny
    "tiny": HeartConfig(
        name="tiny", B=1, H=2, D=64, grid=(4, 16, 16), block=64, seed=0, steps=2,
        gain=6.0, tau_spec=("list", (0.9, 0.95)), delta=0.05, schedule="tiny",
        locality=(1.0, 1.0),
    ),
    # (2) Wan2.1-1.3B at 480P
    "wan1p3b_480p": HeartConfig(
        name="wan1p3b_480p", B=1, H=12, D=128, grid=(21, 30, 52), block=128, seed=1,
        steps=2, tau_spec=("uniform", 0.85, 0.98), delta=0.01, schedule="loguniform",
    ),
    # (3) Wan2.1-14B at 480P: the shape the headline metric is quoted on
    "wan14b_480p": HeartConfig(
        name="wan14b_480p", B=1, H=40, D=128, grid=(21, 30, 52), block=128, seed=2,
        steps=10, tau_spec=("uniform", 0.85, 0.98), delta=1.0, schedule="jumps",
    ),
    # (4) Wan2.1-14B at 720P
    "wan14b_720p": HeartConfig(
        name="wan14b_720p", B=1, H=40, D=128, grid=(21, 45, 80), block=128, seed=3,
        steps=2, tau_spec=("file", "wan14b_720p_tau.json", 0.85, 0.98), delta=1.0,
        schedule="jumps",
    ),
    # (5) HunyuanVideo-shaped, 720P, with text tokens in front
    "hunyuan_720p": HeartConfig(
        name="hunyuan_720p", B=1, H=24, D=128, grid=(33, 45, 80), block=128, seed=4,
        n_text=256, steps=10, tau_spec=("uniform", 0.80, 0.98), delta=1.0,
        schedule="jumps",
    ),
    # reduced shapes for parity tests that the oracle finishes in seconds and
    # that still span several tiles and a ragged last block
    "small_ragged": HeartConfig(
        name="small_ragged", B=2, H=3, D=128, grid=(3, 10, 23), block=128, seed=11,
        steps=3, tau_spec=("uniform", 0.7, 0.98), delta=1.0, schedule="jumps",
    ),
    "small_text": HeartConfig(
        name="small_text", B=1, H=4, D=128, grid=(5, 9, 16), block=128, seed=12,
        n_text=256, steps=3, tau_spec=("uniform", 0.8, 0.98), delta=1.0,
        schedule="jumps",
    ),
    "small_d64": HeartConfig(
        name="small_d64", B=1, H=3, D=64, grid=(3, 11, 13), block=64, seed=13,
        steps=2, tau_spec=("uniform", 0.8, 0.98), delta=1.0, schedule="jumps",
    ),
    "small_d64_b128": HeartConfig(
        name="small_d64_b128", B=2, H=2, D=64, grid=(4, 9, 17), block=128, seed=14,
        steps=2, tau_spec=("uniform", 0.8, 0.98), delta=1.0, schedule="jumps",
    ),
}


def get_config(name: str) -> HeartConfig:
    return CONFIGS[name]


@dataclass
class StepInputs:
    """bf16 tensors of one simulated denoising step, layout [B, H, N, D]."""

    q: torch.Tensor
    k: torch.Tensor
    v: torch.Tensor


def as_u16(t: torch.Tensor) -> np.ndarray:
    """View a CPU bf16 tensor's bits as a uint16 numpy array (no copy)."""
    assert t.dtype == torch.bfloat16 and t.device.type == "cpu"
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


_WORKERS = 8  # generator threads; results do not depend on this number


def _head_rng(seed: int, *stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, *stream]))


def _torch_gen(seed: int, *stream: int) -> torch.Generator:
    s = seed
    for x in stream:
        s = (s * 1000003 + x + 12345) % (2**62)
    return torch.Generator().manual_seed(s)


class HeartInputGenerator:
    """Produces the per-step bf16 tensors and per-head parameters of a config.

    The base fields are built once (fp32, CPU); `step(s)` returns the tensors of
    simulated denoising step s.  Everything is a pure function of (config,
    step), so the oracle and the GPU path can be fed identical bits.
    """

    def __init__(self, cfg: HeartConfig, heads: Optional[List[int]] = None):
        self.cfg = cfg
        # `heads` restricts generation to a subset of heads (same values those
        # heads have in the full tensor) so that sampled oracle checks at full
        # sequence length stay cheap.
        self.heads = list(range(cfg.H)) if heads is None else list(heads)
        self._build_params()
        self._build_base()

    # ---- per-head parameters -------------------------------------------------
    def _build_params(self) -> None:
        cfg = self.cfg
        rng = _head_rng(cfg.seed, 9001)
        if cfg.tau_spec[0] == "list":
            tau = np.asarray(cfg.tau_spec[1], dtype=np.float32)
            assert tau.shape == (cfg.H,)
        else:
            lo_t, hi_t = cfg.tau_spec[-2:]
            tau = rng.uniform(lo_t, hi_t, size=cfg.H).astype(np.float32)
        # (the uniform draw is kept for every spec so that the random stream below is the same)
        self.tau_drawn = tau
        if cfg.tau_spec[0] == "file":
            path = os.path.join(os.path.dirname(os.path.abspath(__file__)), cfg.tau_spec[1])
            if os.path.exists(path):
                with open(path) as f:
                    table = json.load(f)
                assert table["config"] == cfg.name and len(table["tau"]) == cfg.H
                tau = np.asarray(table["tau"], dtype=np.float32)
            # (absent only while the script that writes it runs)
        self.tau = tau
        self.delta = np.full((cfg.H,), cfg.delta, dtype=np.float32)
        lo, hi = cfg.locality
        self.locality = rng.uniform(lo, hi, size=cfg.H) if hi > lo else np.full(cfg.H, lo)

        S, H, D = cfg.steps, cfg.H, cfg.D
        # offsets[s, h] = L1 size of the common offset added (cumulatively) at step s
        inc = np.zeros((S, H), dtype=np.float64)
        noise = np.zeros((S, H), dtype=np.float64)  # std of iid noise at step s vs step 0
        planned = np.zeros((S, H), dtype=bool)
        if cfg.schedule == "tiny":
            # tiny configuration: step 2 = step 1 + N(0, 0.02) on head 0, N(0, 0.5) on head 1
            sig = [0.02, 0.5]
            for s in range(1, S):
                for h in range(H):
                    noise[s, h] = sig[h % 2] * math.sqrt(s)
        elif cfg.schedule == "loguniform":
            mag = np.exp(rng.uniform(math.log(1e-3), math.log(1e-1), size=H))
            for s in range(1, S):
                inc[s] = mag
                noise[s] = mag * 0.1
        elif cfg.schedule == "jumps":
            planned[0] = True
            for s in range(1, S):
                n_lo = math.ceil(0.4 * H - 1e-9)
                n_hi = max(n_lo, math.floor(0.7 * H + 1e-9))
                n_jump = int(rng.integers(n_lo, n_hi + 1))
                jump = rng.permutation(H)[:n_jump]
                inc[s] = 0.01 * cfg.delta
                inc[s, jump] = 4.0 * cfg.delta
                noise[s] = 0.002 * s
                planned[s, jump] = True
        else:
            raise ValueError(cfg.schedule)
        self.planned_jumps = planned  # [S, H] bool, "jumps" schedule only
        self.offset_l1 = np.cumsum(inc, axis=0)  # [S, H]
        self.noise_std = noise
        # Fixed per-head offset directions (unit L1 norm), separate for Q and K.  They lie in
        # the span of the head's own field directions: an offset of Q then adds a term to the
        # logits that varies with the key position, so a head that drifts more also has a
        # block mask that changes more (the relation TMR relies on, Sec. 4.1-4.2).
        self.dir_q = np.zeros((H, D), dtype=np.float32)
        self.dir_k = np.zeros((H, D), dtype=np.float32)
        for h in range(H):
            r = _head_rng(cfg.seed, 9002, h)
            _, _, u_qk, _ = self._field_params(h)
            for arr in (self.dir_q, self.dir_k):
                v = r.standard_normal(4) @ u_qk
                arr[h] = (v / np.abs(v).sum()).astype(np.float32)

    # ---- base fields -----------------------------------------------------------
    def _field_params(self, h: int):
        """Frequencies, phases and directions of head h's four sinusoids (deterministic)."""
        D = self.cfg.D
        rng = _head_rng(self.cfg.seed, 100, h)
        freqs = np.zeros((4, 3), dtype=np.float64)
        # Sinusoids 0..2 vary over (t, y) only, so they survive pooling over a
        # block of consecutive tokens (a block spans whole rows of the grid);
        # sinusoid 3 also varies along x: token-level detail that block means lose.
        for r in range(4):
            while True:
                f = np.array([rng.integers(0, 4), rng.integers(0, 5),
                              0 if r < 3 else rng.integers(1, 4)])
                if f[:2].any():
                    break
            freqs[r] = f
        phase = rng.uniform(0.0, 2.0 * math.pi, size=4)
        u_qk = rng.standard_normal((4, D)) / math.sqrt(D)  # rows of about unit norm
        u_v = rng.standard_normal((4, D)) / math.sqrt(D)
        return freqs, phase, u_qk, u_v

    def _field(self, h: int) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
        cfg = self.cfg
        T, Hg, W = cfg.grid
        D = cfg.D
        freqs, phase, u_qk, u_v = self._field_params(h)
        n = np.arange(T * Hg * W)
        t = n // (Hg * W)
        y = (n // W) % Hg
        x = n % W
        pos = np.stack([t / T, y / Hg, x / W], axis=1)  # [Ng, 3]
        arg = 2.0 * math.pi * (pos @ freqs.T) / self.locality[h] + phase  # [Ng, 4]
        s = torch.from_numpy(np.sin(arg).astype(np.float32))
        # cfg.gain is the intended span of the logits q.k/sqrt(D): the sum of
        # four sine products ranges over about +-2, so amp^2 * 2 / sqrt(D) = gain
        amp = math.sqrt(cfg.gain * math.sqrt(D) / 2.0)
        fq = s @ torch.from_numpy((amp * u_qk).astype(np.float32))
        fv = s @ torch.from_numpy(u_v.astype(np.float32))
        out = []
        for ti, f in enumerate((fq, fq, fv)):
            g = _torch_gen(cfg.seed, 200, ti, h)
            x0 = f + 0.1 * torch.randn(f.shape, generator=g)
            if cfg.n_text:
                txt = 0.3 * torch.randn((cfg.n_text, D), generator=g)
                x0 = torch.cat([txt, x0], dim=0)
            out.append(x0)
        return out[0], out[1], out[2]

    def _build_base(self) -> None:
        cfg = self.cfg
        nh = len(self.heads)
        self.base_q = torch.empty((nh, cfg.N, cfg.D), dtype=torch.float32)
        self.base_k = torch.empty_like(self.base_q)
        self.base_v = torch.empty_like(self.base_q)

        # One fixed unit-variance noise field per (tensor, head): the iid noise of
        # step s is noise_std[s, h] times this field (a smooth trajectory across
        # steps, and it keeps the per-step cost at one fused multiply-add pass).
        need_noise = bool((self.noise_std != 0.0).any())
        self.noise = None
        if need_noise:
            self.noise = [torch.empty((nh, cfg.N, cfg.D), dtype=torch.bfloat16) for _ in range(3)]

        def work(i: int) -> None:
            h = self.heads[i]
            q, k, v = self._field(h)
            self.base_q[i], self.base_k[i], self.base_v[i] = q, k, v
            if need_noise:
                for ti in range(3):
                    g = _torch_gen(cfg.seed, 300, ti, h)
                    self.noise[ti][i] = torch.randn((cfg.N, cfg.D), generator=g).to(torch.bfloat16)

        with ThreadPoolExecutor(max_workers=_WORKERS) as ex:
            list(ex.map(work, range(nh)))

    # ---- per-step tensors --------------------------------------------------------
    def step(self, s: int) -> StepInputs:
        """bf16 tensors of step s, layout [B, len(heads), N, D] (contiguous)."""
        cfg = self.cfg
        assert 0 <= s < cfg.steps
        nh = len(self.heads)
        outs = [torch.empty((cfg.B, nh, cfg.N, cfg.D), dtype=torch.bfloat16) for _ in range(3)]
        bases = (self.base_q, self.base_k, self.base_v)
        dirs = (self.dir_q, self.dir_k, None)

        def work(job: Tuple[int, int, int]) -> None:
            b, i, ti = job
            h = self.heads[i]
            x = bases[ti][i].clone()
            if b > 0:
                # batch items (e.g. the two guidance branches) differ slightly
                g = _torch_gen(cfg.seed, 301, ti, h, b)
                x += 0.05 * torch.randn(x.shape, generator=g)
            if s > 0:
                if dirs[ti] is not None and self.offset_l1[s, h] != 0.0:
                    off = torch.from_numpy(dirs[ti][h] * np.float32(0.5 * self.offset_l1[s, h]))
                    x += off
                if self.noise_std[s, h] != 0.0:
                    x.add_(self.noise[ti][i].float(), alpha=float(self.noise_std[s, h]))
            outs[ti][b, i] = x.to(torch.bfloat16)

        jobs = [(b, i, ti) for b in range(cfg.B) for i in range(nh) for ti in range(3)]
        with ThreadPoolExecutor(max_workers=_WORKERS) as ex:
            list(ex.map(work, jobs))
        return StepInputs(q=outs[0], k=outs[1], v=outs[2])

    def tau_for_heads(self) -> np.ndarray:
        return self.tau[self.heads].copy()

    def delta_for_heads(self) -> np.ndarray:
        return self.delta[self.heads].copy()


def make_generator(name: str, heads: Optional[List[int]] = None) -> HeartInputGenerator:
    return HeartInputGenerator(get_config(name), heads)
