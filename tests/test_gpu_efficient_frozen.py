"""GPU parity of the efficient frozen drafter (App. on extending the draft models): draft mean frozen
on the prediction carried over from the previous window, one batched target call on the start
state and all drafts, the carried prediction moved by ``sd_advance``.  Oracle side:
``oracle.speculative.window_efficient / sample_efficient``.
"""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import speculative as S
from oracle.denoisers import GMMDenoiser, LowRankDenoiser

from _gpu import as_f32_f64, decisions_match, dev, f32, host, rel_err

pytestmark = pytest.mark.gpu

TOL = 1e-5


_DRAFTER = {"draft": "efficient_frozen", "last_accepted": "efficient_frozen_last_accepted"}


@pytest.mark.parametrize("carry", ["draft", "last_accepted"])
@pytest.mark.parametrize("d", [64, 30])
def test_window_and_carry_match_oracle(d, carry):
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config("c2", B=160, d=d, T=50)
    D = GMMDenoiser(cfg.params, cfg.schedule.alpha_bar_state)
    rng = np.random.default_rng(8)
    B, K, T = cfg.B, cfg.K, cfg.T
    n = rng.integers(0, T, size=B).astype(np.int64)
    n[:10] = T - 1 - (np.arange(10) % K)
    y = (rng.standard_normal((B, d)) * 3.0).astype(np.float32)
    ids = rng.permutation(500)[:B].astype(np.int64)
    # a stale frozen vector: the exact prediction plus a perturbation
    Dfz = as_f32_f64(D(y.astype(np.float64), n) + 0.3 * rng.standard_normal((B, d)))
    smp = make_sampler(cfg, out_rows=500, drafter=_DRAFTER[carry])        # finished chains land in out[chain id]
    b = smp.buf
    b.y.copy_(torch.from_numpy(y)); b.n.copy_(dev(n, torch.int32)); b.chain_id.copy_(dev(ids, torch.int64))
    b.Dfz.copy_(f32(Dfz))
    lr = torch.zeros(B, K, device="cuda"); lu = torch.zeros(B, K, device="cuda")
    smp.window(B, (lr, lu))
    res, Ytil, Dq_ext, krow_ext, Dnext = S.window_efficient(cfg.schedule, D, y.astype(np.float64), n, ids, Dfz, K, cfg.seed,
                                                            carry=carry)
    X = host(b.X_ext)
    assert np.array_equal(X[:, 0], y)
    assert rel_err(X[:, 1:], Ytil) < TOL
    assert np.array_equal(host(b.krow_ext), krow_ext)
    ev = krow_ext >= 0
    assert rel_err(host(b.Dq_ext)[ev], Dq_ext[ev]) < 2 * TOL
    Kt = np.minimum(K, T - n)
    adv = host(b.adv).copy()
    assert np.all(adv >= 1) and np.all(adv <= Kt)
    assert (res.adv == 1).sum() > 0                          # position 1 can be rejected now
    nbad, near = decisions_match(adv, res, band=1e-4)
    print(f"[efficient frozen d={d} carry={carry}] oracle mean adv {res.adv.mean():.2f}, rejected {res.rejected.mean():.2f}, "
          f"mismatches {nbad} (near ties {near})")
    assert nbad == near
    same = adv == res.adv
    assert rel_err(host(b.y_out)[same], res.y_out[same]) < 5 * TOL
    inwin = np.arange(K)[None, :] < Kt[:, None]
    assert np.max(np.abs(host(lr)[inwin] - res.logratio[inwin]) / np.maximum(1.0, np.abs(res.logratio[inwin]))) < 1e-3
    # advance: the carried prediction follows the surviving chains
    from _gpu import check_advance_on_matching_chains
    assert check_advance_on_matching_chains(smp, T, n, ids, res, adv, 5 * TOL, carry_ref=Dnext) == int(same.sum())


@pytest.mark.parametrize("carry", ["draft", "last_accepted"])
def test_free_running_sampler_matches_oracle_lowrank(carry):
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config("c3", B=40, d=256, r=32, K=6, T=45)
    D = LowRankDenoiser(cfg.params, cfg.schedule.alpha_bar_state)
    smp = make_sampler(cfg, drafter=_DRAFTER[carry])
    out, counters = smp.run(torch.arange(cfg.B, dtype=torch.int64, device="cuda"))
    ref, st = S.sample_efficient(cfg.schedule, D, cfg.B, cfg.d, cfg.K, seed=cfg.seed, carry=carry)
    got = host(out)
    err = np.max(np.abs(got - ref) / np.maximum(1.0, np.abs(ref).max(axis=1, keepdims=True)), axis=1)
    diverged = int((err > 1e-3).sum())
    print(f"[efficient frozen run, carry {carry}] GPU counters {counters}, oracle steps {st.steps} chain-windows {st.chain_windows} "
          f"rejections {st.rejections}, mean advance {st.mean_advance:.2f}; chains off the oracle path: {diverged}")
    assert counters[0] == cfg.B * cfg.T
    from _gpu import explain_divergent_chains, gpu_chain_stepper
    from oracle import philox

    def ostep(state, n, cid):
        r, _, Dq_ext, _, Dnext = S.window_efficient(cfg.schedule, D, state[0][None], np.array([n]), np.array([cid], dtype=np.int64),
                                                    state[1][None], cfg.K, cfg.seed, carry=carry)
        return (r.y_out[0], Dnext[0]), int(r.adv[0]), r.logratio[0], r.logu[0]

    def ostart(cid):
        y0 = philox.initial_state(cfg.seed, np.array([cid], dtype=np.int64), cfg.d)
        return (y0[0], D(y0, np.zeros(1, dtype=np.int64))[0])
    assert explain_divergent_chains(err, np.arange(cfg.B), *gpu_chain_stepper(cfg, drafter=_DRAFTER[carry]), ostart, ostep,
                                    cfg.T, f"efficient frozen run, carry {carry}") == diverged
    if diverged == 0:
        assert counters[1] == st.chain_windows and counters[2] == st.rejections and counters[3] == st.windows
    assert np.max(err[err <= 1e-3]) < 1e-4


def test_plain_frozen_mode_unchanged_by_the_stride_parameters():
    """The ordinary frozen window still matches the oracle after the kernels learnt the K+1 layout
    (regression guard for the shared draft / verify kernels)."""
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config("c2", B=96, d=64, T=40)
    D = GMMDenoiser(cfg.params, cfg.schedule.alpha_bar_state)
    rng = np.random.default_rng(9)
    n = rng.integers(0, cfg.T, size=cfg.B).astype(np.int64)
    y = (rng.standard_normal((cfg.B, cfg.d)) * 3.0).astype(np.float32)
    ids = np.arange(cfg.B, dtype=np.int64)
    smp = make_sampler(cfg)
    b = smp.buf
    b.y.copy_(torch.from_numpy(y)); b.n.copy_(dev(n, torch.int32)); b.chain_id.copy_(dev(ids, torch.int64))
    smp.window(cfg.B)
    res, Ytil, Dq, D0, krow, _ = S.window(cfg.schedule, D, y.astype(np.float64), n, ids, cfg.K, seed=cfg.seed)
    assert rel_err(host(b.Ytilde), Ytil) < TOL and np.array_equal(host(b.krow), krow)
    nbad, near = decisions_match(host(b.adv), res)
    assert nbad == near


def test_last_accepted_rule_needs_the_rejected_array():
    """With the last-accepted rule sd_advance reads `rejected`; leaving it out is an argument error raised on the
    host before anything is launched."""
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config("c2", B=8, d=16, T=20)
    smp = make_sampler(cfg, drafter="efficient_frozen_last_accepted")
    b = smp.buf
    smp.start(torch.arange(cfg.B, dtype=torch.int64, device="cuda"))
    smp.window(cfg.B)
    with pytest.raises(Exception, match="rejected"):
        smp.ctx.sd_advance(cfg.B, b.y_out, b.adv, None, b.y, b.n, b.chain_id, b.out, b.B_active, b.counters)
    with pytest.raises(Exception, match="rule"):
        smp.ctx.sd_set_carry_rule(2)
