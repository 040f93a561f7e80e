"""GPU parity of whole runs: the window loop fed window by window with the oracle's state, the
free-running sampler against the oracle's trajectories, and the fused Langevin window.
"""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import langevin as L
from oracle import speculative as S
from oracle.denoisers import GMMDenoiser, GMMScore

from _gpu import explain_divergent_chains, gpu_chain_stepper, ula_oracle_stepper, as_f32_f64, decisions_match, dev, f32, host, make_context, rel_err

pytestmark = pytest.mark.gpu

TOL = 1e-5


def test_c1_window_by_window_and_free_running():
    """Config 1 (toy DDPM, d=2, 64 chains, 100 steps, K=4, seed 0), all windows.
    (a) every window of the oracle's run is replayed on the GPU from the oracle's state;
    (b) the GPU sampler runs by itself; chains whose decisions never hit a near tie must end
        within tolerance of the oracle's final state."""
    from paper_2501_05370_amd.binding import Denoiser
    from paper_2501_05370_amd.sampler import DiffusionSampler
    from oracle import philox
    cfg = W.make_config("c1")
    den = GMMDenoiser(cfg.params, cfg.schedule.alpha_bar_state)
    B, K, d, T = cfg.B, cfg.K, cfg.d, cfg.T
    ctx = make_context(cfg.schedule, d, K, seed=cfg.seed)
    g = Denoiser.sdden_gmm_create(cfg.params.means, cfg.params.stds, cfg.params.logw, cfg.schedule.alpha_bar_state)
    smp = DiffusionSampler(ctx, g, B)
    b = smp.buf

    ids = np.arange(B, dtype=np.int64)
    y = as_f32_f64(philox.initial_state(cfg.seed, ids, d))
    n = np.zeros(B, dtype=np.int64)
    out_ref = np.zeros((B, d))
    windows = mism = ties = 0
    worst = 0.0
    while n.size:
        res, *_ = S.window(cfg.schedule, den, y, n, ids, K, seed=cfg.seed)
        Bc = n.size
        b.y[:Bc].copy_(f32(y)); b.n[:Bc].copy_(dev(n, torch.int32)); b.chain_id[:Bc].copy_(dev(ids, torch.int64))
        smp.window(Bc)
        nb, nt = decisions_match(host(b.adv)[:Bc], res)
        mism += nb; ties += nt
        same = host(b.adv)[:Bc] == res.adv
        worst = max(worst, rel_err(host(b.y_out)[:Bc][same], res.y_out[same]))
        y, n, ids = S.advance(T, as_f32_f64(res.y_out), res.adv, n, ids, out_ref)
        windows += 1
    print(f"[c1 replay] {windows} windows, decision mismatches {mism} (near ties {ties}), worst rel err {worst:.2e}")
    assert mism == ties and worst < 5 * TOL

    out, counters = smp.run(torch.arange(B, dtype=torch.int64, device="cuda"))
    ref, st = S.sample(cfg.schedule, den, B, d, K, seed=cfg.seed)
    got = host(out)
    err = np.max(np.abs(got - ref) / np.maximum(1.0, np.abs(ref).max(axis=1, keepdims=True)), axis=1)
    diverged = int((err > 1e-3).sum())
    print(f"[c1 free run] GPU counters {counters}, oracle steps {st.steps} windows {st.chain_windows} "
          f"rejections {st.rejections}; chains off the oracle path: {diverged}")
    assert counters[0] == B * T
    # a flipped near-tie moves a whole chain: every chain that ends off the oracle's path must part from it at one
    gstart, gstep = gpu_chain_stepper(cfg)

    def ostep(state, n, cid):
        r, *_ = S.window(cfg.schedule, den, state[0][None], np.array([n]), np.array([cid], dtype=np.int64), K, seed=cfg.seed)
        return (r.y_out[0],), int(r.adv[0]), r.logratio[0], r.logu[0]
    ostart = lambda cid: (philox.initial_state(cfg.seed, np.array([cid], dtype=np.int64), d)[0],)
    assert explain_divergent_chains(err, np.arange(B), gstart, gstep, ostart, ostep, T, "c1 free run") == diverged
    if diverged == 0:
        assert counters[1] == st.chain_windows and counters[2] == st.rejections


def test_batch_composition_does_not_change_results():
    from paper_2501_05370_amd.binding import Denoiser
    from paper_2501_05370_amd.sampler import DiffusionSampler
    cfg = W.make_config("c2", B=256, T=40)
    ctx = make_context(cfg.schedule, cfg.d, cfg.K, seed=3)
    g = Denoiser.sdden_gmm_create(cfg.params.means, cfg.params.stds, cfg.params.logw, cfg.schedule.alpha_bar_state)
    smp = DiffusionSampler(ctx, g, 256)
    full = host(smp.run(torch.arange(256, dtype=torch.int64, device="cuda"))[0]).copy()
    sub_ids = torch.tensor([200, 3, 77, 255, 128], dtype=torch.int64, device="cuda")
    smp2 = DiffusionSampler(ctx, g, 5, out_rows=256)
    sub = host(smp2.run(sub_ids)[0])
    assert np.array_equal(sub[[200, 3, 77, 255, 128]], full[[200, 3, 77, 255, 128]])


_LANGEVIN_SHAPES = [(64, 1000, 16, 16, 40), (40, 10, 3, 5, 12), (32, 1003, 16, 16, 30),
                    (16, 2100, 7, 8, 20), (8, 4096, 16, 4, 9),
                    # two and three coordinate groups per lane; more chains than the resident
                    # wavefronts (each wavefront then takes several chains from the counter)
                    (48, 512, 5, 6, 15), (24, 700, 16, 8, 20), (3000, 40, 4, 6, 14)]
# every shape at the exact sampler's temperature; one shape per kernel variant at a hotter and a colder one
_LANGEVIN_CASES = [s + (1.0,) for s in _LANGEVIN_SHAPES] + \
                  [s + (t,) for s in _LANGEVIN_SHAPES if s[1] in (1000, 2100, 700, 40) for t in (2.0, 0.6)]


@pytest.mark.parametrize("B,d,M,K,T,tau", _LANGEVIN_CASES)
def test_langevin_window_matches_oracle(B, d, M, K, T, tau):
    rng = np.random.default_rng(8)
    cfg = W.make_config("c5", B=B, d=d, M=M, K=K, T=T)
    p = cfg.params
    sc = GMMScore(p)
    gamma = cfg.gamma
    ctx = make_context(cfg.schedule, d, K, seed=21, tau=tau)
    # start near / between components so that gradients differ along the window
    comp = rng.integers(0, M, size=B)
    x = as_f32_f64(p.means[comp] * rng.uniform(0.3, 1.0, size=(B, 1)) + rng.standard_normal((B, d)))
    n = rng.integers(0, T, size=B)
    n[:3] = [T - 1, T - 2, 0]
    ids = rng.permutation(max(1000, 2 * B))[:B].astype(np.int64)
    xo, adv, rej, lr, lu = L.ula_window(sc, x, n, ids, K, T, gamma, seed=21, tau=tau)
    gx = torch.full((B, d), 9.0, dtype=torch.float32, device="cuda")
    gadv = torch.zeros(B, dtype=torch.int32, device="cuda")
    grej = torch.zeros(B, dtype=torch.uint8, device="cuda")
    glr = torch.full((B, K), 5.0, dtype=torch.float32, device="cuda")
    glu = torch.full((B, K), 5.0, dtype=torch.float32, device="cuda")
    ctx.sd_langevin_window(B, f32(x), dev(n, torch.int32), dev(ids, torch.int64), f32(p.means), f32(p.logw),
                           float(p.stds[0, 0]), M, gamma, gx, gadv, grej, glr, glu)

    class R:  # the fields decisions_match reads
        pass
    R.adv, R.logu, R.logratio = adv, lu, lr
    nbad, near = decisions_match(host(gadv), R)
    print(f"[langevin d={d}] rejected {rej.mean():.2f}, mean adv {adv.mean():.2f}, mismatches {nbad} (near ties {near})")
    assert nbad == near
    same = host(gadv) == adv
    assert np.array_equal(host(grej)[same].astype(bool), rej[same])
    assert rel_err(host(gx)[same], xo[same]) < TOL
    # diagnostics are reported up to the position that stopped the window, 0 after it
    for b in np.nonzero(same)[0]:
        a = adv[b]
        assert np.max(np.abs(host(glu)[b, :a] - lu[b, :a])) < 1e-5
        assert np.max(np.abs(host(glr)[b, :a] - lr[b, :a]) / np.maximum(1, np.abs(lr[b, :a]))) < 1e-5
        assert np.all(host(glr)[b, a:] == 0) and np.all(host(glu)[b, a:] == 0)


def test_langevin_free_run_small():
    from paper_2501_05370_amd.sampler import LangevinSampler
    cfg = W.make_config("c5", B=48, d=200, M=4, K=8, T=60)
    p = cfg.params
    ctx = make_context(cfg.schedule, cfg.d, cfg.K, seed=5)
    smp = LangevinSampler(ctx, f32(p.means), f32(p.logw), float(p.stds[0, 0]), cfg.gamma, cfg.B)
    out, counters = smp.run(torch.arange(cfg.B, dtype=torch.int64, device="cuda"))
    ref, cw, rejections = L.ula_sample(GMMScore(p), cfg.B, cfg.d, cfg.K, cfg.T, cfg.gamma, seed=5)
    err = np.max(np.abs(host(out) - ref), axis=1) / np.maximum(1.0, np.abs(ref).max(axis=1))
    diverged = int((err > 1e-3).sum())
    print(f"[langevin free run] counters {counters}, oracle chain-windows {cw} rejections {rejections}, off-path {diverged}")
    assert counters[0] == cfg.B * cfg.T
    assert explain_divergent_chains(err, np.arange(cfg.B), *gpu_chain_stepper(cfg, seed=5),
                                    *ula_oracle_stepper(GMMScore(p), cfg, 5), cfg.T, "langevin free run") == diverged
    if diverged == 0:
        assert counters[1] == cw and counters[2] == rejections


@pytest.mark.parametrize("L_,B,K,T", [(8, 300, 20, 50), (4, 70, 6, 30), (16, 40, 12, 40), (5, 33, 7, 25)])
@pytest.mark.parametrize("tau", [1.0, 3000.0])       # at tau = 3000 the walk goes past its second position (|Delta|^2 is 200 to 3000 here)
def test_phi4_langevin_window_matches_oracle(L_, B, K, T, tau):
    """The fused Langevin window on the phi^4 lattice energy against the oracle's ula_window with the
    oracle's Phi4Energy: grids whose sites fill the lanes exactly, leave lanes idle (5 x 5) or take a
    whole wavefront (16 x 16); chains at ragged positions, near the end of the run."""
    from oracle.langevin import Phi4Energy
    rng = np.random.default_rng(12)
    d = L_ * L_
    cfg = W.make_config("phi4", B=B, d=d, K=K, T=T)
    beta, gamma = cfg.params.beta, cfg.gamma
    E = Phi4Energy(L_, beta)
    ctx = make_context(cfg.schedule, d, K, seed=31, tau=tau)
    # ordered states with noise, the regime the chain lives in
    x = as_f32_f64(rng.choice([-1.0, 1.0], size=(B, 1)) + 0.15 * rng.standard_normal((B, d)))
    n = rng.integers(0, T, size=B)
    n[:3] = [T - 1, T - 2, 0]
    ids = rng.permutation(5000)[:B].astype(np.int64)
    xo, adv, rej, lr, lu = L.ula_window(E, x, n, ids, K, T, gamma, seed=31, tau=tau)
    gx = torch.full((B, d), 9.0, dtype=torch.float32, device="cuda")
    gadv = torch.zeros(B, dtype=torch.int32, device="cuda")
    grej = torch.zeros(B, dtype=torch.uint8, device="cuda")
    glr = torch.full((B, K), 5.0, dtype=torch.float32, device="cuda")
    glu = torch.full((B, K), 5.0, dtype=torch.float32, device="cuda")
    ctx.sd_langevin_window_phi4(B, f32(x), dev(n, torch.int32), dev(ids, torch.int64), L_, beta, gamma, gx, gadv, grej, glr, glu)

    class R:
        pass
    R.adv, R.logu, R.logratio = adv, lu, lr
    nbad, near = decisions_match(host(gadv), R)
    print(f"[phi4 L={L_} tau={tau}] rejected {rej.mean():.2f}, mean adv {adv.mean():.2f}, mismatches {nbad} (near ties {near})")
    assert nbad == near
    if tau > 1.0:
        assert adv.max() > 3                         # the temperature case does reach later positions
    same = host(gadv) == adv
    assert same.mean() > 0.9
    assert np.array_equal(host(grej)[same].astype(bool), rej[same])
    assert rel_err(host(gx)[same], xo[same]) < TOL
    for b in np.nonzero(same)[0]:
        a = adv[b]
        assert np.max(np.abs(host(glu)[b, :a] - lu[b, :a])) < 1e-5
        assert np.max(np.abs(host(glr)[b, :a] - lr[b, :a]) / np.maximum(1, np.abs(lr[b, :a]))) < 1e-5
        assert np.all(host(glr)[b, a:] == 0) and np.all(host(glu)[b, a:] == 0)


def test_phi4_langevin_free_run_and_argument_checks():
    from paper_2501_05370_amd.binding import SDError
    from paper_2501_05370_amd.runner import make_sampler
    from oracle.langevin import Phi4Energy
    cfg = W.make_config("phi4", B=64, T=120)
    smp = make_sampler(cfg)
    out, counters = smp.run(torch.arange(cfg.B, dtype=torch.int64, device="cuda"))
    ref, cw, rejections = L.ula_sample(Phi4Energy(cfg.params.L, cfg.params.beta), cfg.B, cfg.d, cfg.K, cfg.T, cfg.gamma,
                                       seed=cfg.seed)
    err = np.max(np.abs(host(out) - ref), axis=1) / np.maximum(1.0, np.abs(ref).max(axis=1))
    diverged = int((err > 1e-3).sum())
    print(f"[phi4 free run] counters {counters}, oracle chain-windows {cw} rejections {rejections}, off-path {diverged}")
    assert counters[0] == cfg.B * cfg.T
    assert explain_divergent_chains(err, np.arange(cfg.B), *gpu_chain_stepper(cfg),
                                    *ula_oracle_stepper(Phi4Energy(cfg.params.L, cfg.params.beta), cfg, cfg.seed), cfg.T,
                                    "phi4 free run") == diverged
    if diverged == 0:
        assert counters[1] == cw and counters[2] == rejections
    b = smp.buf
    with pytest.raises(SDError):                              # grid side that does not match the context's d
        smp.ctx.sd_langevin_window_phi4(4, b.y, b.n, b.chain_id, 7, 100.0, 1e-3, b.y_out, b.adv, b.rejected)
    with pytest.raises(SDError):
        smp.ctx.sd_langevin_window_phi4(4, b.y, b.n, b.chain_id, 8, 100.0, -1.0, b.y_out, b.adv, b.rejected)


@pytest.mark.parametrize("B,d,M,K,T", [(300, 200, 4, 8, 60), (64, 1000, 16, 16, 45), (37, 10, 3, 5, 23), (50, 701, 16, 8, 20)])
def test_langevin_run_equals_the_window_loop_and_the_oracle(B, d, M, K, T):
    """sd_langevin_run (every chain's windows back to back in one launch) against the launch-per-window
    loop of the same library, bit for bit, and against the oracle's sampler."""
    from paper_2501_05370_amd.binding import SDError
    from paper_2501_05370_amd.sampler import LangevinSampler
    cfg = W.make_config("c5", B=B, d=d, M=M, K=K, T=T)
    p = cfg.params
    ids = torch.arange(B, dtype=torch.int64, device="cuda")
    outs = []
    for fused in (False, True):
        ctx = make_context(cfg.schedule, d, K, seed=5)
        smp = LangevinSampler(ctx, f32(p.means), f32(p.logw), float(p.stds[0, 0]), cfg.gamma, B)
        out, counters = smp.run_fused(ids) if fused else smp.run(ids)
        outs.append((host(out)[:B].copy(), counters, host(smp.buf.n)[:B].copy() if fused else None))
    (xw, cw, _), (xf, cf, nf) = outs
    assert np.array_equal(xw, xf)
    assert [cf[i] for i in (0, 1, 2, 4)] == [cw[i] for i in (0, 1, 2, 4)] and cf[3] == 1
    assert np.all(nf == T)
    ref, ocw, orej = L.ula_sample(GMMScore(p), B, d, K, T, cfg.gamma, seed=5)
    err = np.max(np.abs(xf - ref), axis=1) / np.maximum(1.0, np.abs(ref).max(axis=1))
    diverged = int((err > 1e-3).sum())
    print(f"[langevin run d={d}] counters {cf}, oracle chain-windows {ocw} rejections {orej}, off-path {diverged}")
    assert cf[0] == B * T
    assert explain_divergent_chains(err, np.arange(B), *gpu_chain_stepper(cfg, seed=5),
                                    *ula_oracle_stepper(GMMScore(p), cfg, 5), T, f"langevin run d={d}") == diverged
    if diverged == 0:
        assert cf[1] == ocw and cf[2] == orej
    # a bound on the windows per chain: two windows advance a chain by 2..2K steps, and a second call finishes
    ctx = make_context(cfg.schedule, d, K, seed=5)
    smp = LangevinSampler(ctx, f32(p.means), f32(p.logw), float(p.stds[0, 0]), cfg.gamma, B)
    b = smp.buf
    smp.start(ids)
    ctx.sd_langevin_run(B, b.y, b.n, b.chain_id, smp.means, smp.logw, smp.comp_std, M, cfg.gamma, 2, b.y, b.n, b.counters)
    n2 = host(b.n)[:B]
    assert np.all(n2 >= min(2, T)) and np.all(n2 <= min(T, 2 * K))
    ctx.sd_langevin_run(B, b.y, b.n, b.chain_id, smp.means, smp.logw, smp.comp_std, M, cfg.gamma, T, b.y, b.n, b.counters)
    assert np.array_equal(host(b.y)[:B], xw) and np.all(host(b.n)[:B] == T)
    with pytest.raises(SDError):
        ctx.sd_langevin_run(B, b.y, b.n, b.chain_id, smp.means, smp.logw, smp.comp_std, M, cfg.gamma, 1, b.y, b.n, None)
    # chains handed over at step T are left as they are and count no window
    before = b.counters.tolist()
    xo = torch.zeros_like(b.y)
    ctx.sd_langevin_run(B, b.y, b.n, b.chain_id, smp.means, smp.logw, smp.comp_std, M, cfg.gamma, 5, xo, b.n, b.counters)
    after = b.counters.tolist()
    assert torch.equal(xo[:B], b.y[:B]) and np.all(host(b.n)[:B] == T)
    assert [after[i] for i in (0, 1, 2, 4)] == [before[i] for i in (0, 1, 2, 4)]


@pytest.mark.parametrize("kind,kw,tau", [("c5", dict(B=120, d=200, M=4, K=8, T=40), 2.0),
                                         ("phi4", dict(B=200, T=60), 400.0)])
def test_langevin_runs_with_temperature_equal_the_window_loop(kind, kw, tau):
    """The temperature of the accept test (App. "Influence of the temperature") in the one-launch forms: same
    results as window + advance repeated, bit for bit, and the acceptance moves the way the temperature says."""
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config(kind, **kw)
    ids = torch.arange(cfg.B, dtype=torch.int64, device="cuda")
    res = {}
    for t in (1.0, tau):
        outs = []
        for fused in (False, True):
            smp = make_sampler(cfg)
            smp.ctx.sd_set_temperature(t)
            out, counters = smp.run_fused(ids) if fused else smp.run(ids)
            outs.append((host(out)[:cfg.B].copy(), counters))
        (xw, cw), (xf, cf) = outs
        assert np.array_equal(xw, xf)
        assert [cf[i] for i in (0, 1, 2, 4)] == [cw[i] for i in (0, 1, 2, 4)]
        res[t] = cf
    print(f"[{kind} tau={tau}] chain-windows {res[1.0][1]} -> {res[tau][1]}, rejections {res[1.0][2]} -> {res[tau][2]}")
    assert res[tau][1] < res[1.0][1] and res[tau][2] < res[1.0][2]      # hotter: fewer rejections, fewer windows


@pytest.mark.parametrize("L_,B,K,T", [(8, 300, 20, 50), (4, 70, 6, 30), (16, 40, 12, 40), (5, 33, 7, 25)])
def test_phi4_langevin_run_equals_the_window_loop(L_, B, K, T):
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config("phi4", B=B, T=T, K=K, d=L_ * L_)
    ids = torch.arange(B, dtype=torch.int64, device="cuda")
    smp = make_sampler(cfg)
    out, cw = smp.run(ids)
    xw = host(out)[:B].copy()
    smp2 = make_sampler(cfg)
    out2, cf = smp2.run_fused(ids)
    xf = host(out2)[:B].copy()
    print(f"[phi4 run L={L_}] counters window loop {cw}, one launch {cf}")
    assert np.array_equal(xw, xf)
    assert [cf[i] for i in (0, 1, 2, 4)] == [cw[i] for i in (0, 1, 2, 4)] and cf[3] == 1
    assert np.all(host(smp2.buf.n)[:B] == T)
