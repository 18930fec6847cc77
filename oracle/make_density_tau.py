#!/usr/bin/env python3
"""Writes heart_synth/wan14b_720p_tau.json: the per-head top-p thresholds of the
Wan2.1-14B-shaped 720P configuration, which asks for a global kept-block density of
15 % "via per-head tau".  Test infrastructure: this script calls only the CPU oracle
(block means, block scores, top-p rule of Sec. 3.2 / Eq. 1) and the seeded input
generator; nothing of the HIP path.

Recipe.  The generator's uniform draw tau0_h ~ U(0.85, 0.98) gives each head a natural
density d0_h on step 0 (heads differ in how peaked their block scores are).  The target
of head h is d_h = 0.15 * d0_h / mean(d0): the heads keep their relative densities and
the global density is 15 %.  tau_h is then found by bisection on the oracle's top-p
selection until the head's density brackets d_h; the stored value is the float32 at the
end of 24 halvings.

Run from the repository root:  python oracle/make_density_tau.py
"""
from __future__ import annotations

import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from heart_synth import as_u16, make_generator  # noqa: E402

NAME = "wan14b_720p"
TARGET = 0.15


def main() -> None:
    g = make_generator(NAME)
    cfg = g.cfg
    st = g.step(0)
    qb, _ = oracle.pool(as_u16(st.q), cfg.block)
    kb, _ = oracle.pool(as_u16(st.k), cfg.block)
    sc = oracle.scores(qb, kb)
    nt = cfg.n_text_blocks
    B, H, Nb = cfg.B, cfg.H, cfg.Nb

    def density(tau):
        _, _, cnt = oracle.topp(sc, tau.astype(np.float32), n_always_kv=nt, n_dense_q=nt)
        return cnt.sum(axis=(0, 2)) / float(B * Nb * Nb)

    d0 = density(g.tau_drawn)
    want = TARGET * d0 / d0.mean()
    lo = np.full(H, 0.01, np.float32)
    hi = np.full(H, 0.9999, np.float32)
    for _ in range(24):
        mid = ((lo.astype(np.float64) + hi) / 2).astype(np.float32)
        d = density(mid)
        hi = np.where(d > want, mid, hi).astype(np.float32)
        lo = np.where(d > want, lo, mid).astype(np.float32)
    tau = lo
    d = density(tau)
    out = {
        "config": NAME,
        "written_by": "oracle/make_density_tau.py",
        "target_global_density": TARGET,
        "global_density": float(d.mean()),
        "tau": [float(np.float32(x)) for x in tau],
        "density_per_head": [round(float(x), 5) for x in d],
        "density_per_head_at_drawn_tau": [round(float(x), 5) for x in d0],
    }
    path = os.path.join(ROOT, "heart_synth", NAME + "_tau.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print(f"{path}: global density {d.mean():.4f} (drawn thresholds gave {d0.mean():.4f})")


if __name__ == "__main__":
    main()
