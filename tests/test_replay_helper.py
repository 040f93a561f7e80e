"""The free-run replay helper of the GPU tests (tests/_gpu.py), exercised on the CPU with stand-ins for the GPU side:
a stepper that rounds its states to fp32 at every window (what the library does) must either stay on the oracle's
path or leave it at a near tie that the rounding explains; a stepper with a planted wrong decision must be caught."""
import numpy as np
import pytest

import workloads as W
from oracle import philox
from oracle import speculative as S
from oracle.denoisers import GMMDenoiser

from _gpu import first_divergence_is_a_near_tie


def _steppers(cfg, den, sabotage_window=None):
    def ostep(state, n, cid):
        r, *_ = S.window(cfg.schedule, den, state[0][None], np.array([n]), np.array([cid], dtype=np.int64), cfg.K, seed=cfg.seed)
        return (r.y_out[0],), int(r.adv[0]), r.logratio[0], r.logu[0]

    calls = {"w": 0}

    def fake_gpu_step(state, n, cid):
        out, adv, _, _ = ostep((state[0].astype(np.float32).astype(np.float64),), n, cid)
        if sabotage_window is not None and calls["w"] == sabotage_window and adv > 1:
            adv -= 1                                   # a wrong decision nothing explains
        calls["w"] += 1
        return (out[0].astype(np.float32).astype(np.float64),), adv

    return ostep, fake_gpu_step


def test_fp32_rounded_replay_stays_on_the_path_or_parts_at_a_near_tie():
    cfg = W.make_config("c1", B=16, T=60)
    den = GMMDenoiser(cfg.params, cfg.schedule.alpha_bar_state)
    for cid in range(cfg.B):
        ostep, gstep = _steppers(cfg, den)
        y0 = philox.initial_state(cfg.seed, np.array([cid], dtype=np.int64), cfg.d)[0]
        found = first_divergence_is_a_near_tie(gstep, ostep, (y0.astype(np.float32).astype(np.float64),), (y0,), cid, cfg.T)
        assert found is None or found[1] <= found[2] + 1e-6


def test_a_decision_nothing_explains_is_caught():
    cfg = W.make_config("c1", B=4, T=60)
    den = GMMDenoiser(cfg.params, cfg.schedule.alpha_bar_state)
    caught = 0
    for cid in range(cfg.B):
        ostep, gstep = _steppers(cfg, den, sabotage_window=2)
        y0 = philox.initial_state(cfg.seed, np.array([cid], dtype=np.int64), cfg.d)[0]
        try:
            first_divergence_is_a_near_tie(gstep, ostep, (y0,), (y0,), cid, cfg.T)
        except AssertionError:
            caught += 1
    assert caught == cfg.B
