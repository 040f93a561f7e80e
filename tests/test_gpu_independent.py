"""GPU parity of the independent draft model (Sec. 3.1): a cheaper network called at every window
position (``sd_draft_step`` between the calls), one batched target call, ``sd_verify`` in EXPLICIT
mode with the window-start prediction kept as its own array.  The oracle side is
``oracle.speculative.window / sample`` with ``drafter="independent"``.
"""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import philox
from oracle import speculative as S
from oracle.denoisers import GMMDenoiser, LowRankDenoiser

from _gpu import as_f32_f64, decisions_match, dev, f32, host, rel_err

pytestmark = pytest.mark.gpu

TOL = 1e-5


def _ragged_states(cfg, rng, scale):
    B = cfg.B
    n = rng.integers(0, cfg.T, size=B)
    n[:8] = cfg.T - 1 - (np.arange(8) % cfg.K)            # chains inside the last window
    y = (rng.standard_normal((B, cfg.d)) * scale).astype(np.float32)
    return y, n.astype(np.int64)


def _load(smp, y, n, ids):
    b = smp.buf
    B = n.size
    b.y[:B].copy_(torch.from_numpy(y)); b.n[:B].copy_(dev(n, torch.int32)); b.chain_id[:B].copy_(dev(ids, torch.int64))


@pytest.mark.parametrize("d", [64, 37])                    # vectorised and scalar (d % 4 != 0) kernels
def test_draft_step_rollout_and_window_match_oracle_gmm(d):
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config("c2", B=192, d=d, T=60)
    dp = W.draft_params(cfg)
    D = GMMDenoiser(cfg.params, cfg.schedule.alpha_bar_state)
    Dd = GMMDenoiser(dp, cfg.schedule.alpha_bar_state)
    rng = np.random.default_rng(5)
    y, n = _ragged_states(cfg, rng, 3.0)
    ids = rng.permutation(1000)[:cfg.B].astype(np.int64)
    smp = make_sampler(cfg, drafter="independent", draft_params=dp)
    _load(smp, y, n, ids)
    K = cfg.K
    lr = torch.zeros(cfg.B, K, device="cuda"); lu = torch.zeros(cfg.B, K, device="cuda")
    smp.window(cfg.B, (lr, lu))
    b = smp.buf
    res, Ytil, Dq, D0, krow, calls = S.window(cfg.schedule, D, y.astype(np.float64), n, ids, K, seed=cfg.seed,
                                              drafter="independent", D_draft=Dd)
    _, mp, _ = S.draft_independent(cfg.schedule, Dd, y.astype(np.float64), n, ids, K, cfg.seed)
    assert np.array_equal(host(b.krow), krow)
    assert rel_err(host(b.mp), mp) < TOL
    assert rel_err(host(b.Ytilde), Ytil) < TOL
    assert rel_err(host(b.D0), D0) < TOL
    mask = np.zeros((cfg.B, K), dtype=bool); mask[:, 1:] = krow[:, :K - 1] >= 0
    assert rel_err(host(b.Dq)[mask], Dq[mask]) < 2 * TOL
    Kt = np.minimum(K, cfg.T - n)
    adv = host(b.adv)
    assert np.all(adv >= 1) and np.all(adv <= Kt)
    # the draft differs from the target, so position 1 is no longer accepted for certain
    assert (res.adv == 1).sum() > 0 and res.rejected.mean() > 0.2
    nbad, near = decisions_match(adv, res, band=1e-4)
    print(f"[independent gmm d={d}] oracle mean adv {res.adv.mean():.2f}, rejected {res.rejected.mean():.2f}, "
          f"mismatches {nbad} (near ties {near})")
    assert nbad == near
    same = adv == res.adv
    assert np.array_equal(host(b.rejected)[same].astype(bool), res.rejected[same])
    assert rel_err(host(b.y_out)[same], res.y_out[same]) < 5 * TOL
    inwin = np.arange(K)[None, :] < Kt[:, None]
    assert np.max(np.abs(host(lr)[inwin] - res.logratio[inwin]) / np.maximum(1.0, np.abs(res.logratio[inwin]))) < 1e-3


def test_verify_reads_start_prediction_from_its_own_array():
    """EXPLICIT mode with the window-start prediction in a separate [B,d] array gives the same
    result as with that prediction stored in row 0 of Dq."""
    from paper_2501_05370_amd.binding import SD_DRAFT_EXPLICIT
    from _gpu import make_context
    cfg = W.make_config("c2", B=96, d=64, T=60)
    dp = W.draft_params(cfg)
    D = GMMDenoiser(cfg.params, cfg.schedule.alpha_bar_state)
    Dd = GMMDenoiser(dp, cfg.schedule.alpha_bar_state)
    rng = np.random.default_rng(6)
    y, n = _ragged_states(cfg, rng, 3.0)
    y64 = y.astype(np.float64)
    ids = np.arange(cfg.B, dtype=np.int64)
    K = cfg.K
    Ytil, mp, krow = S.draft_independent(cfg.schedule, Dd, y64, n, ids, K, cfg.seed)
    Ytil, mp = as_f32_f64(Ytil), as_f32_f64(mp)
    D0 = as_f32_f64(D(y64, n))
    Dq = as_f32_f64(S.target_predictions(cfg.schedule, D, Ytil, krow, D0))
    ctx = make_context(cfg.schedule, cfg.d, K, seed=cfg.seed, mode=SD_DRAFT_EXPLICIT)
    outs = []
    for separate in (False, True):
        gDq = f32(Dq)
        gD0 = f32(D0)
        if separate:
            gDq[:, 0] = 1e30                                # must not be read
            ctx.sd_set_start_prediction(gD0)
        y_out = torch.zeros(cfg.B, cfg.d, device="cuda"); adv = torch.zeros(cfg.B, dtype=torch.int32, device="cuda")
        rej = torch.zeros(cfg.B, dtype=torch.uint8, device="cuda")
        ctx.sd_verify(cfg.B, f32(y), dev(n, torch.int32), dev(ids, torch.int64), f32(mp), gDq, f32(Ytil), y_out, adv, rej)
        outs.append((host(y_out).copy(), host(adv).copy(), host(rej).copy()))
    ctx.sd_set_start_prediction(None)
    for a, c in zip(outs[0], outs[1]):
        assert np.array_equal(a, c)
    res = S.verify(cfg.schedule, y64, n, ids, Ytil, Dq, K, cfg.seed, mp=mp)
    nbad, near = decisions_match(outs[1][1], res)
    assert nbad == near
    same = outs[1][1] == res.adv
    assert rel_err(outs[1][0][same], res.y_out[same]) < TOL


def test_independent_free_running_sampler_lowrank():
    """Whole run with a low-rank-Gaussian target and a coarser low-rank draft: final states of the
    chains that stayed on the oracle's decision path agree; step bookkeeping is exact."""
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config("c3", B=48, d=256, r=32, K=6, T=40)
    dp = W.draft_params(cfg)
    D = LowRankDenoiser(cfg.params, cfg.schedule.alpha_bar_state)
    Dd = LowRankDenoiser(dp, cfg.schedule.alpha_bar_state)
    smp = make_sampler(cfg, drafter="independent", draft_params=dp)
    out, counters = smp.run(torch.arange(cfg.B, dtype=torch.int64, device="cuda"))
    ref, st = S.sample(cfg.schedule, D, cfg.B, cfg.d, cfg.K, seed=cfg.seed, drafter="independent", D_draft=Dd)
    got = host(out)
    err = np.max(np.abs(got - ref) / np.maximum(1.0, np.abs(ref).max(axis=1, keepdims=True)), axis=1)
    diverged = int((err > 1e-3).sum())
    print(f"[independent lowrank run] GPU counters {counters}, oracle steps {st.steps} chain-windows {st.chain_windows} "
          f"rejections {st.rejections}, mean advance {st.mean_advance:.2f}; chains off the oracle path: {diverged}")
    assert counters[0] == cfg.B * cfg.T
    from _gpu import explain_divergent_chains, gpu_chain_stepper
    from oracle import philox

    def ostep(state, n, cid):
        r, *_ = S.window(cfg.schedule, D, state[0][None], np.array([n]), np.array([cid], dtype=np.int64), cfg.K, seed=cfg.seed,
                         drafter="independent", D_draft=Dd)
        return (r.y_out[0],), int(r.adv[0]), r.logratio[0], r.logu[0]
    ostart = lambda cid: (philox.initial_state(cfg.seed, np.array([cid], dtype=np.int64), cfg.d)[0],)
    assert explain_divergent_chains(err, np.arange(cfg.B), *gpu_chain_stepper(cfg, drafter="independent", draft_params=dp),
                                    ostart, ostep, cfg.T, "independent lowrank run") == diverged
    if diverged == 0:
        assert counters[1] == st.chain_windows and counters[2] == st.rejections
    assert np.max(err[err <= 1e-3]) < 1e-4
