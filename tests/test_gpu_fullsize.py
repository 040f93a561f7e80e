"""GPU parity at the full sizes of the five configurations, in the launch configuration the
benchmark times (full batch B, full d, K, T): the GPU runs one whole window for all chains from
seeded synthetic states; the oracle recomputes the window for a sample of the chains (chains are
independent and their random streams are keyed by chain id, so a sample is exact), and every
sampled output is compared element by element.

Tolerances as in the stage tests: fp32 1e-5 relative (row scale, floor 1), bf16 MLP 2e-2;
accepted-prefix lengths exact outside the near-tie band (hits are counted and printed).
"""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import langevin as L
from oracle import speculative as S
from oracle.denoisers import GMMDenoiser, GMMScore, LowRankDenoiser, MLPDenoiser

from _gpu import (as_f32_f64, check_advance_on_matching_chains, decisions_match, dev, explain_divergent_chains, f32,
                  gpu_chain_stepper, host, rel_err, ula_oracle_stepper)

pytestmark = pytest.mark.gpu


def _states(cfg, rng, scale):
    """Ragged positions (a few chains inside the last window) and states of the right magnitude."""
    B, T, K = cfg.B, cfg.T, cfg.K
    n = rng.integers(0, T, size=B)
    n[:16] = T - 1 - (np.arange(16) % min(K, T))
    y = (rng.standard_normal((B, cfg.d)) * scale).astype(np.float32)
    return y, n.astype(np.int64)


def _run_gpu_window(cfg, y, n, ids, diagnostics=False):
    from paper_2501_05370_amd.runner import make_sampler
    smp = make_sampler(cfg)
    b = smp.buf
    b.y.copy_(torch.from_numpy(y)); b.n.copy_(dev(n, torch.int32)); b.chain_id.copy_(dev(ids, torch.int64))
    smp.lr = smp.lu = None
    if diagnostics:
        smp.lr = torch.zeros(cfg.B, cfg.K, device="cuda"); smp.lu = torch.zeros(cfg.B, cfg.K, device="cuda")
        smp.window(cfg.B, (smp.lr, smp.lu))
    else:
        smp.window(cfg.B)
    torch.cuda.synchronize()
    return smp


def _compare_window(cfg, D, smp, y, n, ids, sample, tol, band, check_decisions=True):
    """band None: the tie band of the decision comparison is derived from this very run -- four times the largest
    difference between the GPU's and the oracle's log-ratio over the sampled chains (printed), at least 1e-6."""
    b = smp.buf
    sel = torch.as_tensor(sample, device="cuda")
    ys = y[sample].astype(np.float64)
    res, Ytil, Dq, D0, krow, _ = S.window(cfg.schedule, D, ys, n[sample], ids[sample], cfg.K, seed=cfg.seed)
    K = cfg.K
    assert rel_err(host(b.D0[sel]), D0) < tol
    assert rel_err(host(b.Ytilde[sel]), Ytil) < tol
    assert np.array_equal(host(b.krow[sel]), krow)
    mask = np.zeros((len(sample), K), dtype=bool); mask[:, 1:] = krow[:, :K - 1] >= 0
    assert rel_err(host(b.Dq[sel])[mask], Dq[mask]) < 2 * tol
    adv = host(b.adv[sel])
    Kt = np.minimum(K, cfg.T - n[sample])
    assert np.all(adv >= np.minimum(2, Kt)) and np.all(adv <= Kt)
    dl = None
    if smp.lr is not None:
        inwin = np.arange(K)[None, :] < Kt[:, None]
        dl = float(np.max(np.abs(host(smp.lr[sel])[inwin] - res.logratio[inwin])))
        assert np.max(np.abs(host(smp.lu[sel])[inwin] - res.logu[inwin])) < 1e-5
    if band is None:
        band = max(1e-6, 4.0 * dl)
    nbad, near = decisions_match(adv, res, band=band)
    same = adv == res.adv
    print(f"[{cfg.name} full size] sampled {len(sample)} of {cfg.B} chains: oracle mean adv {res.adv.mean():.2f}, "
          f"rejected {res.rejected.mean():.2f}, decision mismatches {nbad} (near ties {near} in a band of {band:.1e}"
          + (f"; largest |log-ratio GPU - oracle| {dl:.2e})" if dl is not None else ")"))
    if check_decisions:
        assert nbad == near
    assert same.mean() > 0.5
    assert rel_err(host(b.y_out[sel])[same], res.y_out[same]) < 5 * tol
    return res


def _verify_on_oracle_inputs(cfg, D, smp, y, n, ids, sample, tol):
    """Decision parity at the 1e-6 band of the contract, at full size: the oracle builds the verify inputs of the
    sampled chains (its own predictions, rounded to fp32), their rows in the GPU's window tensors are overwritten
    with them, and sd_verify runs on the FULL batch.  (The GPU's own window tensors are never oracle input.)"""
    b = smp.buf
    ys = y[sample].astype(np.float64)
    D0 = as_f32_f64(D(ys, n[sample]))
    Ytil, krow = S.draft_frozen(cfg.schedule, ys, n[sample], ids[sample], D0, cfg.K, cfg.seed)
    Ytil = as_f32_f64(Ytil)
    Dq = as_f32_f64(S.target_predictions(cfg.schedule, D, Ytil, krow, D0))
    res = S.verify(cfg.schedule, ys, n[sample], ids[sample], Ytil, Dq, cfg.K, cfg.seed, D0=D0)
    sel = torch.as_tensor(sample, device="cuda")
    b.D0[sel] = f32(D0); b.Ytilde[sel] = f32(Ytil); b.Dq[sel] = f32(Dq)
    outs = []
    for diag in (True, False):                      # with the per-position diagnostics, and in the form the sampler runs
        lr = torch.zeros(cfg.B, cfg.K, device="cuda"); lu = torch.zeros(cfg.B, cfg.K, device="cuda")
        smp.ctx.sd_verify(cfg.B, b.y, b.n, b.chain_id, b.D0, b.Dq, b.Ytilde, b.y_out, b.adv, b.rejected,
                          lr if diag else None, lu if diag else None)
        outs.append((host(b.adv[sel]).copy(), host(b.y_out[sel]).copy(), host(lr[sel]).copy()))
    adv = outs[0][0]
    nbad, near = decisions_match(adv, res)
    print(f"[{cfg.name} full size verify on the oracle's inputs] {len(sample)} chains, oracle mean adv {res.adv.mean():.2f}, "
          f"rejected {res.rejected.mean():.2f}, mismatches {nbad} (near ties {near} at 1e-6)")
    assert nbad == near
    same = adv == res.adv
    assert rel_err(outs[0][1][same], res.y_out[same]) < tol
    assert np.max(np.abs(outs[0][2] - res.logratio) / np.maximum(1.0, np.abs(res.logratio))) < 1e-5
    assert np.array_equal(outs[1][0], adv) and np.array_equal(outs[1][1], outs[0][1])


def test_c2_full_size_all_chains():
    cfg = W.make_config("c2")
    rng = np.random.default_rng(20)
    y, n = _states(cfg, rng, 3.0)
    ids = rng.permutation(cfg.B).astype(np.int64)
    smp = _run_gpu_window(cfg, y, n, ids)
    D = GMMDenoiser(cfg.params, cfg.schedule.alpha_bar_state)
    _compare_window(cfg, D, smp, y, n, ids, np.arange(cfg.B), 1e-5, 1e-6)
    # and the bookkeeping of the whole batch
    res, *_ = S.window(cfg.schedule, D, y.astype(np.float64), n, ids, cfg.K, seed=cfg.seed)
    checked = check_advance_on_matching_chains(smp, cfg.T, n, ids, res, host(smp.buf.adv).copy(), 5e-5)
    assert checked >= cfg.B - 2


def test_c3_full_size_sampled_chains():
    cfg = W.make_config("c3")
    rng = np.random.default_rng(30)
    y, n = _states(cfg, rng, 1.0)
    ids = np.arange(cfg.B, dtype=np.int64)
    smp = _run_gpu_window(cfg, y, n, ids, diagnostics=True)
    sample = np.concatenate([np.arange(8), rng.choice(np.arange(16, cfg.B), 88, replace=False)])
    D = LowRankDenoiser(cfg.params, cfg.schedule.alpha_bar_state)
    # end to end the predictions differ by the fp32 rounding of two GEMMs over d = 3072, which moves the log-ratio:
    # the tie band of this comparison is four times the largest shift measured in this run (printed) ...
    _compare_window(cfg, D, smp, y, n, ids, sample, 1e-5, None)
    # ... and the decisions are held to the contract's 1e-6 on identical inputs
    _verify_on_oracle_inputs(cfg, D, smp, y, n, ids, sample, 1e-5)


def test_c4_full_size_sampled_chains():
    cfg = W.make_config("c4")
    rng = np.random.default_rng(40)
    y, n = _states(cfg, rng, 1.0)
    ids = np.arange(cfg.B, dtype=np.int64)
    smp = _run_gpu_window(cfg, y, n, ids)
    sample = np.unique(np.concatenate([[0, 3, 17, 511], rng.choice(np.arange(18, 500), 30, replace=False)]))   # 34 chains
    D = MLPDenoiser(cfg.params)
    # bf16 predictions move the log-ratio by O(0.1): decisions are compared on identical inputs below
    _compare_window(cfg, D, smp, y, n, ids, sample, 2e-2, 1e-6, check_decisions=False)
    _verify_on_oracle_inputs(cfg, D, smp, y, n, ids, sample, 1e-5)


def test_c5_full_size_sampled_chains():
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config("c5")
    rng = np.random.default_rng(50)
    p = cfg.params
    B, d, K, T = cfg.B, cfg.d, cfg.K, cfg.T
    comp = rng.integers(0, p.means.shape[0], size=B)
    y = (p.means[comp] * rng.uniform(0.5, 1.0, size=(B, 1)) + rng.standard_normal((B, d))).astype(np.float32)
    n = rng.integers(0, T, size=B).astype(np.int64)
    n[:16] = T - 1 - np.arange(16)
    ids = np.arange(B, dtype=np.int64)
    smp = make_sampler(cfg)
    b = smp.buf
    b.y.copy_(torch.from_numpy(y)); b.n.copy_(dev(n, torch.int32)); b.chain_id.copy_(dev(ids, torch.int64))
    lr = torch.zeros(B, K, device="cuda"); lu = torch.zeros(B, K, device="cuda")
    smp.window(B, lr, lu)
    torch.cuda.synchronize()
    sample = np.concatenate([np.arange(8), rng.choice(np.arange(16, B), 56, replace=False)])
    xo, adv, rej, olr, olu = L.ula_window(GMMScore(p), y[sample].astype(np.float64), n[sample], ids[sample], K, T,
                                          cfg.gamma, seed=cfg.seed)
    sel = torch.as_tensor(sample, device="cuda")

    class R:
        pass
    R.adv, R.logu, R.logratio = adv, olu, olr
    gadv = host(b.adv[sel])
    nbad, near = decisions_match(gadv, R)
    print(f"[c5 full size] sampled {len(sample)} of {B} chains: mean adv {adv.mean():.2f}, rejected {rej.mean():.2f}, "
          f"mismatches {nbad} (near ties {near})")
    assert nbad == near
    same = gadv == adv
    assert np.array_equal(host(b.rejected[sel])[same].astype(bool), rej[same])
    assert rel_err(host(b.y_out[sel])[same], xo[same]) < 1e-5


def test_phi4_full_size_sampled_chains():
    """The phi^4 lattice window at the benchmark's size (16384 chains of 8 x 8 sites, K = 20) in the launch
    configuration bench.py times; sampled chains against the oracle's window on the same states."""
    from oracle.langevin import Phi4Energy
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config("phi4")
    rng = np.random.default_rng(60)
    B, d, K, T = cfg.B, cfg.d, cfg.K, cfg.T
    Lside = cfg.params.L
    y = (rng.choice([-1.0, 1.0], size=(B, 1)) + 0.15 * rng.standard_normal((B, d))).astype(np.float32)
    n = rng.integers(0, T, size=B).astype(np.int64)
    n[:16] = T - 1 - np.arange(16)
    ids = np.arange(B, dtype=np.int64)
    smp = make_sampler(cfg)
    b = smp.buf
    b.y.copy_(torch.from_numpy(y)); b.n.copy_(dev(n, torch.int32)); b.chain_id.copy_(dev(ids, torch.int64))
    smp.window(B)
    torch.cuda.synchronize()
    sample = np.concatenate([np.arange(16), rng.choice(np.arange(16, B), 112, replace=False)])
    xo, adv, rej, olr, olu = L.ula_window(Phi4Energy(Lside, cfg.params.beta), y[sample].astype(np.float64), n[sample],
                                          ids[sample], K, T, cfg.gamma, seed=cfg.seed)
    sel = torch.as_tensor(sample, device="cuda")

    class R:
        pass
    R.adv, R.logu, R.logratio = adv, olu, olr
    gadv = host(b.adv[sel])
    nbad, near = decisions_match(gadv, R)
    print(f"[phi4 full size] sampled {len(sample)} of {B} chains: mean adv {adv.mean():.2f}, rejected {rej.mean():.2f}, "
          f"mismatches {nbad} (near ties {near})")
    assert nbad == near
    same = gadv == adv
    assert same.mean() > 0.9
    assert np.array_equal(host(b.rejected[sel])[same].astype(bool), rej[same])
    assert rel_err(host(b.y_out[sel])[same], xo[same]) < 1e-5
    # advance at this size: the scan's single pass of 16 chunks
    n_next = n + host(b.adv).astype(np.int64)
    smp.advance(B)
    Ba = int(host(b.B_active)[0])
    assert Ba == int((n_next < T).sum())
    assert np.array_equal(host(b.n)[:Ba], n_next[n_next < T])
    assert np.array_equal(host(b.chain_id)[:Ba], ids[n_next < T])


@pytest.mark.parametrize("name,T", [("c5", 160), ("phi4", 400)])
def test_langevin_full_size_run_equals_the_window_loop(name, T):
    """The one-launch form (sd_langevin_run / sd_langevin_run_phi4) that bench.py times for c5 and phi4, at
    the benchmark's batch and state size (the chain length is cut to keep the test short): final states
    and counters equal those of the launch-per-window loop bit for bit; sampled chains are compared with the
    oracle's sampler, which carries its states in fp64 (tolerance as in the small free-run tests)."""
    from oracle.langevin import Phi4Energy
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config(name, T=T)
    B = cfg.B
    ids = torch.arange(B, dtype=torch.int64, device="cuda")
    smp = make_sampler(cfg)
    out, cw = smp.run(ids, windows_per_sync=4)
    xw = out[:B].clone()
    smp2 = make_sampler(cfg)
    out2, cf = smp2.run_fused(ids)
    assert torch.equal(xw, out2[:B])
    assert [cf[i] for i in (0, 1, 2, 4)] == [cw[i] for i in (0, 1, 2, 4)] and cf[0] == B * T
    assert bool((smp2.buf.n[:B] == T).all())
    sample = np.sort(np.random.default_rng(61).choice(B, 24, replace=False))
    grad = Phi4Energy(cfg.params.L, cfg.params.beta) if name == "phi4" else GMMScore(cfg.params)
    ref, _, _ = L.ula_sample(grad, len(sample), cfg.d, cfg.K, T, cfg.gamma, seed=cfg.seed,
                             chain_ids=sample.astype(np.int64))
    got = host(out2[torch.as_tensor(sample, device="cuda")])
    err = np.max(np.abs(got - ref), axis=1) / np.maximum(1.0, np.abs(ref).max(axis=1))
    diverged = int((err > 1e-3).sum())
    print(f"[{name} one launch, {B} chains, T={T}] counters {cf}; {len(sample)} chains against the oracle: "
          f"max err {err.max():.2e}, off-path {diverged}")
    assert explain_divergent_chains(err, sample, *gpu_chain_stepper(cfg), *ula_oracle_stepper(grad, cfg, cfg.seed), T,
                                    f"{name} one launch") == diverged
