"""CPU checks of the synthetic input recipe (heart_synth): what the benchmark configurations
ask of the schedules and thresholds holds by construction, for every config, without
generating any tensor."""
import json
import os

import numpy as np
import pytest

from heart_synth import CONFIGS, HeartInputGenerator

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def params(name):
    g = HeartInputGenerator.__new__(HeartInputGenerator)
    g.cfg = CONFIGS[name]
    g.heads = list(range(g.cfg.H))
    g._build_params()
    return g


@pytest.mark.parametrize("name", [n for n, c in CONFIGS.items() if c.schedule == "jumps"])
def test_jump_schedule_keeps_the_planned_refresh_share_in_band(name):
    """30-70 % of heads per step (the Wan2.1-14B-shaped configuration), and never below the 40 %
    at which the layer gate would turn a step into reuse for every head."""
    g = params(name)
    cfg = g.cfg
    frac = g.planned_jumps.mean(axis=1)
    assert frac[0] == 1.0  # nothing is cached at step 0
    assert np.all(frac[1:] >= 0.4 - 1e-9) and np.all(frac[1:] <= 0.7 + 1e-9), frac
    # a planned head jumps by 4 delta, the others creep by 0.01 delta per step: far from delta
    inc = np.diff(g.offset_l1, axis=0)
    assert np.allclose(inc[g.planned_jumps[1:]], 4.0 * cfg.delta)
    assert np.allclose(inc[~g.planned_jumps[1:]], 0.01 * cfg.delta)
    assert 0.01 * cfg.delta * cfg.steps < 0.5 * cfg.delta


def test_stored_threshold_table_of_the_720p_configuration():
    g = params("wan14b_720p")
    path = os.path.join(ROOT, "heart_synth", "wan14b_720p_tau.json")
    table = json.load(open(path))
    assert table["config"] == "wan14b_720p" and table["written_by"] == "oracle/make_density_tau.py"
    assert abs(table["global_density"] - 0.15) < 0.005 and table["target_global_density"] == 0.15
    tau = np.asarray(table["tau"], np.float32)
    assert tau.shape == (g.cfg.H,) and np.all(tau > 0) and np.all(tau < 1)
    assert np.array_equal(g.tau, tau)          # the generator hands out the stored table
    assert not np.array_equal(g.tau_drawn, tau)  # ... not the uniform draw it was made from
    # heads keep their relative densities: the table's per-head densities are proportional to
    # those of the uniform draw
    d, d0 = np.asarray(table["density_per_head"]), np.asarray(table["density_per_head_at_drawn_tau"])
    assert np.allclose(d / d.mean(), d0 / d0.mean(), atol=0.02)


def test_thresholds_and_shapes_of_the_five_benchmark_configurations():
    want = {"tiny": (1, 2, 64, 1024, 64), "wan1p3b_480p": (1, 12, 128, 32760, 128),
            "wan14b_480p": (1, 40, 128, 32760, 128), "wan14b_720p": (1, 40, 128, 75600, 128),
            "hunyuan_720p": (1, 24, 128, 118800 + 256, 128)}
    for name, (B, H, D, N, blk) in want.items():
        c = CONFIGS[name]
        assert (c.B, c.H, c.D, c.N, c.block) == (B, H, D, N, blk), name
    assert params("tiny").tau.tolist() == pytest.approx([0.9, 0.95])
    for name, lo, hi in (("wan1p3b_480p", 0.85, 0.98), ("wan14b_480p", 0.85, 0.98), ("hunyuan_720p", 0.80, 0.98)):
        t = params(name).tau
        assert np.all(t >= lo) and np.all(t <= hi)
    assert CONFIGS["hunyuan_720p"].n_text_blocks == 2 and CONFIGS["wan14b_480p"].steps == 10
