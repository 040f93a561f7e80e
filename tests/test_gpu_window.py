"""GPU parity: every window stage of the HIP library against the fp64 oracle, element by element,
on the same seeded inputs (through the C ABI via the ctypes binding).

Tolerances (fp32 path): states and predictions within 1e-5 relative (row scale, floor 1);
accepted-prefix lengths bit-exact except where the oracle's own margin |log u - log ratio| is
below 1e-6 (counted and printed); integer outputs (krow, n, chain ids, counters) bit-exact.
"""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import philox
from oracle import speculative as S
from oracle.denoisers import GMMDenoiser

from _gpu import as_f32_f64, check_advance_on_matching_chains, decisions_match, dev, f32, host, make_context, rel_err

pytestmark = pytest.mark.gpu

TOL = 1e-5


def _gmm_case(name, **kw):
    cfg = W.make_config(name, **kw)
    den = GMMDenoiser(cfg.params, cfg.schedule.alpha_bar_state)
    return cfg, den


def _random_window_inputs(cfg, den, B, rng, n_hi=None):
    """Oracle-made inputs of one window at ragged positions n (some chains close to the end)."""
    T = cfg.T
    n = rng.integers(0, T if n_hi is None else n_hi, size=B)
    n[: max(1, B // 8)] = T - 1 - rng.integers(0, min(cfg.K, T), size=max(1, B // 8)) % T
    n = np.clip(n, 0, T - 1)
    ab = cfg.schedule.alpha_bar_state[n][:, None]
    comp = rng.integers(0, cfg.params.means.shape[0], size=B)
    x0 = cfg.params.means[comp] + cfg.params.stds[comp] * rng.standard_normal((B, cfg.d))
    y = as_f32_f64(np.sqrt(ab) * x0 + np.sqrt(1 - ab) * rng.standard_normal((B, cfg.d)))
    ids = rng.permutation(10 * B)[:B].astype(np.int64) + (1 << 33)      # exercises the high id word
    return y, n, ids


# ------------------------------------------------------------------------------------------
def test_init_state_matches_oracle_stream():
    sched = W.linear_beta_schedule(10)
    for d in (2, 7, 64, 1000):
        ctx = make_context(sched, d, 4, seed=0xDEADBEEF12345)
        ids = np.array([0, 1, 5, (1 << 40) + 3, 77], dtype=np.int64)
        y = torch.empty(5, d, dtype=torch.float32, device="cuda")
        n = torch.full((5,), -1, dtype=torch.int32, device="cuda")
        ctx.sd_init_state(5, dev(ids, torch.int64), y, n)
        want = philox.initial_state(0xDEADBEEF12345, ids, d)
        assert np.max(np.abs(host(y) - want)) < 2e-6
        assert host(n).tolist() == [0] * 5


@pytest.mark.parametrize("name,kw", [("c1", dict(B=64)), ("c2", dict(B=300)), ("c2", dict(B=70, d=50, K=5)),
                                     ("c2", dict(B=33, d=1000, K=16, M=3)), ("c2", dict(B=9, d=4100, K=3, M=2)),
                                     ("c2", dict(B=7, d=260, K=64, M=2)), ("c2", dict(B=20, d=64, K=1))])
def test_draft_matches_oracle(name, kw):
    cfg, den = _gmm_case(name, **kw)
    rng = np.random.default_rng(1)
    y, n, ids = _random_window_inputs(cfg, den, cfg.B, rng)
    D0 = as_f32_f64(den(y, n))
    Ytil, krow = S.draft_frozen(cfg.schedule, y, n, ids, D0, cfg.K, seed=7)
    ctx = make_context(cfg.schedule, cfg.d, cfg.K, seed=7)
    gY = torch.full((cfg.B, cfg.K, cfg.d), 123.0, dtype=torch.float32, device="cuda")
    gk = torch.full((cfg.B, cfg.K), 99, dtype=torch.int32, device="cuda")
    ctx.sd_draft(cfg.B, f32(y), dev(n, torch.int32), dev(ids, torch.int64), f32(D0), gY, gk)
    assert np.array_equal(host(gk), krow)
    assert rel_err(host(gY), Ytil) < TOL
    Kt = np.minimum(cfg.K, cfg.T - n)
    for b in range(cfg.B):
        assert np.all(host(gY)[b, Kt[b]:] == 0)


def _verify_case(cfg, den, B, seed, rng, mode="frozen", tau=1.0, shrink=1.0):
    y, n, ids = _random_window_inputs(cfg, den, B, rng)
    D0 = as_f32_f64(den(y, n))
    if mode == "frozen":
        Ytil, krow = S.draft_frozen(cfg.schedule, y, n, ids, D0, cfg.K, seed)
        mp = None
    else:
        draft = lambda x, k: den(x, k) * shrink + 0.01          # some other, cheaper network
        Ytil, mp, krow = S.draft_independent(cfg.schedule, draft, y, n, ids, cfg.K, seed)
        mp = as_f32_f64(mp)
    Ytil = as_f32_f64(Ytil)
    Dq = as_f32_f64(S.target_predictions(cfg.schedule, den, Ytil, krow, D0))
    res = S.verify(cfg.schedule, y, n, ids, Ytil, Dq, cfg.K, seed, D0=D0 if mp is None else None, mp=mp, tau=tau)
    return y, n, ids, D0, mp, Ytil, Dq, res


@pytest.mark.parametrize("name,kw,mode,tau", [
    ("c1", dict(B=64), "frozen", 1.0),
    ("c2", dict(B=400), "frozen", 1.0),
    ("c2", dict(B=100, d=52, K=7), "frozen", 1.0),           # sub-wavefront path, ragged columns
    ("c2", dict(B=64, d=600, K=16, M=4), "frozen", 1.0),     # one wavefront per chain
    ("c2", dict(B=24, d=4100, K=20, M=2), "frozen", 1.0),    # workgroup per chain, 2 position chunks
    ("c2", dict(B=16, d=3000, K=33, M=2), "frozen", 2.0),    # 3 chunks, temperature
    ("c2", dict(B=16, d=1203, K=5, M=2), "frozen", 1.0),     # d % 4 != 0: scalar loads
    ("c2", dict(B=200, d=64, K=8), "explicit", 1.0),
    ("c2", dict(B=20, d=2052, K=18, M=3), "explicit", 0.7),
    ("c2", dict(B=12, d=300, K=64, M=2), "frozen", 1.0),     # the largest window the library takes
    ("c2", dict(B=6, d=8192, K=64, M=2), "frozen", 1.0),     # the same with a workgroup of 512 threads per chain
    ("c2", dict(B=40, d=64, K=1), "frozen", 1.0),            # a window of one position: the sequential chain
    ("c2", dict(B=10, d=64, K=64, M=2), "explicit", 1.0),
])
def test_verify_matches_oracle(name, kw, mode, tau):
    cfg, den = _gmm_case(name, **kw)
    rng = np.random.default_rng(2)
    y, n, ids, D0, mp, Ytil, Dq, res = _verify_case(cfg, den, cfg.B, 11, rng, mode, tau, shrink=0.97)
    from paper_2501_05370_amd.binding import SD_DRAFT_EXPLICIT, SD_DRAFT_FROZEN
    ctx = make_context(cfg.schedule, cfg.d, cfg.K, seed=11,
                       mode=SD_DRAFT_FROZEN if mode == "frozen" else SD_DRAFT_EXPLICIT, tau=tau)
    B, K, d = cfg.B, cfg.K, cfg.d
    y_out = torch.full((B, d), 55.0, dtype=torch.float32, device="cuda")
    adv = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    rej = torch.full((B,), 9, dtype=torch.uint8, device="cuda")
    lr = torch.full((B, K), 3.0, dtype=torch.float32, device="cuda")
    lu = torch.full((B, K), 3.0, dtype=torch.float32, device="cuda")
    ctx.sd_verify(B, f32(y), dev(n, torch.int32), dev(ids, torch.int64), f32(D0 if mp is None else mp),
                  f32(Dq), f32(Ytil), y_out, adv, rej, lr, lu)
    g_adv, g_rej = host(adv), host(rej)
    nbad, near = decisions_match(g_adv, res)
    print(f"[verify {name} {kw} {mode}] rejected {res.rejected.mean():.2f} of chains, "
          f"decision mismatches {nbad} (near ties {near})")
    assert nbad == near
    same = g_adv == res.adv
    assert np.array_equal(g_rej[same].astype(bool), res.rejected[same])
    # the reflection branch is exercised (the only position of a frozen window of one is exact: nothing to reject)
    assert res.rejected.mean() > 0.05 or name == "c1" or (cfg.K == 1 and mode == "frozen")
    assert rel_err(host(y_out)[same], res.y_out[same]) < TOL
    assert np.max(np.abs(host(lu) - res.logu)) < 1e-5
    assert np.max(np.abs(host(lr) - res.logratio) / np.maximum(1.0, np.abs(res.logratio))) < 1e-5
    # without the diagnostic outputs (groups of positions past the first rejection are then not read)
    # the decisions and the states are the same, bit for bit
    adv2 = torch.zeros_like(adv)
    y_out2 = torch.full_like(y_out, -3.0)
    ctx.sd_verify(B, f32(y), dev(n, torch.int32), dev(ids, torch.int64), f32(D0 if mp is None else mp),
                  f32(Dq), f32(Ytil), y_out2, adv2, None, None, None)
    assert np.array_equal(host(adv2), g_adv)
    assert np.array_equal(host(y_out2), host(y_out))


def test_verify_degenerate_cases():
    """Draft == target accepts everything; identical predictions give Delta = 0 exactly."""
    cfg, den = _gmm_case("c2", B=50, d=64, K=8)
    rng = np.random.default_rng(3)
    y, n, ids = _random_window_inputs(cfg, den, cfg.B, rng)
    D0 = as_f32_f64(den(y, n))
    Ytil, krow = S.draft_frozen(cfg.schedule, y, n, ids, D0, cfg.K, 5)
    Ytil = as_f32_f64(Ytil)
    Dq = np.repeat(D0[:, None, :], cfg.K, axis=1)              # target prediction == frozen one
    ctx = make_context(cfg.schedule, cfg.d, cfg.K, seed=5)
    y_out = torch.empty(cfg.B, cfg.d, dtype=torch.float32, device="cuda")
    adv = torch.empty(cfg.B, dtype=torch.int32, device="cuda")
    rej = torch.empty(cfg.B, dtype=torch.uint8, device="cuda")
    lr = torch.empty(cfg.B, cfg.K, dtype=torch.float32, device="cuda")
    ctx.sd_verify(cfg.B, f32(y), dev(n, torch.int32), dev(ids, torch.int64), f32(D0), f32(Dq), f32(Ytil),
                  y_out, adv, rej, lr, None)
    Kt = np.minimum(cfg.K, cfg.T - n)
    assert np.array_equal(host(adv), Kt) and not host(rej).any() and np.all(host(lr) == 0)
    assert np.array_equal(host(y_out), Ytil[np.arange(cfg.B), Kt - 1].astype(np.float32))
    # B = 0 is a no-op
    ctx.sd_verify(0, f32(y), dev(n, torch.int32), dev(ids, torch.int64), f32(D0), f32(Dq), f32(Ytil),
                  y_out, adv, rej, None, None)


# 16385 and 40000 chains: more than one pass of the scan (16 chunks of 1024 chains per pass)
@pytest.mark.parametrize("B,d", [(1, 2), (64, 2), (1500, 64), (3000, 5), (40, 1000), (16385, 2), (40000, 4)])
def test_advance_matches_oracle(B, d):
    rng = np.random.default_rng(4)
    T, K = 50, 6
    sched = W.linear_beta_schedule(T)
    ctx = make_context(sched, d, K, seed=0)
    ws = torch.empty(ctx.sd_workspace_bytes(B), dtype=torch.uint8, device="cuda")
    ctx.sd_set_workspace(ws)
    n = rng.integers(T - 8, T, size=B)
    adv = np.minimum(rng.integers(1, K + 1, size=B), T - n).astype(np.int32)
    rej = rng.integers(0, 2, size=B).astype(np.uint8)
    ids = rng.permutation(B).astype(np.int64)
    y_out = rng.standard_normal((B, d)).astype(np.float32)
    out_ref = np.zeros((B, d))
    y_ref, n_ref, id_ref = S.advance(T, y_out.astype(np.float64), adv, n, ids, out_ref)
    gy = torch.full((B, d), -1.0, dtype=torch.float32, device="cuda")
    gn, gid = dev(n, torch.int32), dev(ids, torch.int64)
    gout = torch.zeros(B, d, dtype=torch.float32, device="cuda")
    gB = torch.zeros(1, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(5, dtype=torch.int64, device="cuda")
    ctx.sd_advance(B, f32(y_out), dev(adv, torch.int32), dev(rej, torch.uint8), gy, gn, gid, gout, gB, cnt)
    Ba = int(host(gB)[0])
    assert Ba == n_ref.size
    assert np.array_equal(host(gn)[:Ba], n_ref) and np.array_equal(host(gid)[:Ba], id_ref)
    assert np.array_equal(host(gy)[:Ba], y_ref.astype(np.float32))
    assert np.array_equal(host(gout), out_ref.astype(np.float32))
    assert host(cnt).tolist() == [int(adv.sum()), B, int(rej.sum()), 1, int(np.minimum(K, T - n).sum())]


def test_gmm_denoiser_matches_oracle():
    # c1, c2 and the small mixtures take the register-resident kernel at every lane split (1, 2, 4, 8, 16, 32
    # component lanes; ragged d, M not a power of two); M = 70 and d = 1100 take the general kernel
    for name, kw in (("c1", dict(B=64)), ("c2", dict(B=64)), ("c2", dict(B=8, d=300, M=70)),
                     ("c2", dict(B=8, d=40, M=1)), ("c2", dict(B=8, d=100, M=2)), ("c2", dict(B=8, d=200, M=3)),
                     ("c2", dict(B=8, d=17, M=5)), ("c2", dict(B=8, d=128, M=12)), ("c2", dict(B=8, d=30, M=32)),
                     ("c2", dict(B=8, d=1024, M=2)), ("c2", dict(B=8, d=1100, M=2))):
        cfg, den = _gmm_case(name, **kw)
        from paper_2501_05370_amd.binding import Denoiser
        g = Denoiser.sdden_gmm_create(cfg.params.means, cfg.params.stds, cfg.params.logw,
                                      cfg.schedule.alpha_bar_state)
        rng = np.random.default_rng(5)
        R = 257
        k = rng.integers(-1, cfg.T, size=R).astype(np.int32)
        k[:3] = [0, cfg.T - 1, -1]
        ab = cfg.schedule.alpha_bar_state[np.maximum(k, 0)][:, None]
        comp = rng.integers(0, cfg.params.means.shape[0], size=R)
        x = as_f32_f64(np.sqrt(ab) * cfg.params.means[comp] + np.sqrt(1 - ab + 0.01) * rng.standard_normal((R, cfg.d)))
        out = torch.full((R, cfg.d), 777.0, dtype=torch.float32, device="cuda")
        g.sdden_eval(R, f32(x), dev(k, torch.int32), out)
        want = den(x[k >= 0], k[k >= 0])
        got = host(out)
        assert rel_err(got[k >= 0], want) < TOL
        assert np.all(got[k < 0] == 777.0)                      # masked rows untouched


@pytest.mark.parametrize("name,kw", [("c1", dict()), ("c2", dict(B=512))])
def test_whole_window_pipeline_matches_oracle(name, kw):
    """Window-level protocol: the oracle supplies (y, n, ids); both sides run S0..S6."""
    from paper_2501_05370_amd.binding import Denoiser
    from paper_2501_05370_amd.sampler import DiffusionSampler
    cfg, den = _gmm_case(name, **kw)
    rng = np.random.default_rng(6)
    B, K, d = cfg.B, cfg.K, cfg.d
    y, n, ids = _random_window_inputs(cfg, den, B, rng)
    ids = rng.permutation(B).astype(np.int64)
    res, Ytil, Dq, D0, krow, _ = S.window(cfg.schedule, den, y, n, ids, K, seed=cfg.seed)

    ctx = make_context(cfg.schedule, d, K, seed=cfg.seed)
    g = Denoiser.sdden_gmm_create(cfg.params.means, cfg.params.stds, cfg.params.logw, cfg.schedule.alpha_bar_state)
    smp = DiffusionSampler(ctx, g, B)
    b = smp.buf
    b.y.copy_(f32(y)); b.n.copy_(dev(n, torch.int32)); b.chain_id.copy_(dev(ids, torch.int64))
    smp.window(B)
    assert rel_err(host(b.D0), D0) < TOL
    assert rel_err(host(b.Ytilde), Ytil) < TOL
    assert np.array_equal(host(b.krow), krow)
    mask = np.zeros((B, K), dtype=bool)
    mask[:, 1:] = krow[:, :K - 1] >= 0
    assert rel_err(host(b.Dq)[mask], Dq[mask]) < 2 * TOL
    nbad, near = decisions_match(host(b.adv), res)
    print(f"[window {name}] mean advance {res.adv.mean():.2f}, mismatches {nbad} (near ties {near})")
    assert nbad == near
    same = host(b.adv) == res.adv
    assert rel_err(host(b.y_out)[same], res.y_out[same]) < 5 * TOL
    # the bookkeeping, on every chain whose decisions are the oracle's (all of them unless a near tie was hit)
    assert check_advance_on_matching_chains(smp, cfg.T, n, ids, res, host(b.adv).copy(), 5 * TOL) == int(same.sum())


def test_draft_writes_the_bf16_image_of_the_drafts():
    """sd_set_draft_mirror: every drafted value also lands as bf16 (round to nearest even) in the image;
    both the vectorised and the scalar (d % 4 != 0) kernels, frozen and K+1-row layouts."""
    from paper_2501_05370_amd.binding import SD_DRAFT_FROZEN_REUSED
    for d, mode in ((64, None), (37, None), (64, SD_DRAFT_FROZEN_REUSED)):
        cfg = W.make_config("c2", B=50, d=d, T=40)
        ctx = make_context(cfg.schedule, d, cfg.K, seed=4, mode=mode)
        rng = np.random.default_rng(2)
        rows = cfg.K + (1 if mode else 0)
        y = f32(rng.standard_normal((cfg.B, d)) * 2); D0 = f32(rng.standard_normal((cfg.B, d)))
        n = dev(rng.integers(0, cfg.T, size=cfg.B), torch.int32); ids = dev(np.arange(cfg.B), torch.int64)
        Yt = torch.zeros(cfg.B, rows, d, device="cuda"); kr = torch.zeros(cfg.B, rows, dtype=torch.int32, device="cuda")
        img = torch.full((cfg.B, rows, d), 0x1234, dtype=torch.int16, device="cuda")
        ctx.sd_set_draft_mirror(img)
        ctx.sd_draft(cfg.B, y, n, ids, D0, Yt, kr)
        ctx.sd_set_draft_mirror(None)
        assert torch.equal(img, Yt.to(torch.bfloat16).view(torch.int16))
        Yt2 = torch.zeros_like(Yt); img.fill_(0x1234)
        ctx.sd_draft(cfg.B, y, n, ids, D0, Yt2, kr)         # switched off again: image untouched, drafts equal
        assert torch.equal(Yt2, Yt) and bool((img == 0x1234).all())
