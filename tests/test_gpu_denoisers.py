"""GPU parity of the MFMA denoisers (low-rank Gaussian in fp32, MLP in bf16) against the oracle,
and of the whole window with them plugged in.

Tolerances: fp32 path 1e-5 relative (row scale, floor 1); bf16 MLP 2e-2.
"""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import speculative as S
from oracle.denoisers import LowRankDenoiser, MLPDenoiser

from _gpu import as_f32_f64, decisions_match, dev, f32, host, make_context, rel_err

pytestmark = pytest.mark.gpu


def _rows(rng, R, T, d, scale=1.0):
    k = rng.integers(-1, T, size=R).astype(np.int32)
    k[:4] = [0, T - 1, -1, T // 2]
    x = as_f32_f64(rng.standard_normal((R, d)) * scale)
    return x, k


@pytest.mark.parametrize("d,r,T,R", [(64, 16, 20, 300), (48, 5, 12, 129), (512, 40, 30, 1000),
                                     (3072, 256, 250, 700)])
def test_lowrank_denoiser_matches_oracle(d, r, T, R):
    from paper_2501_05370_amd.binding import Denoiser
    rng = np.random.default_rng(0)
    p = W.lowrank_gaussian(rng, d, r)
    sched = W.cosine_schedule(T)
    den = LowRankDenoiser(p, sched.alpha_bar_state)
    g = Denoiser.sdden_lowrank_create(p.mu, p.U, p.s2, sched.alpha_bar_state)
    g.sdden_reserve(R)
    x, k = _rows(rng, R, T, d, 1.3)
    out = torch.full((R, d), 777.0, dtype=torch.float32, device="cuda")
    g.sdden_eval(R, f32(x), dev(k, torch.int32), out)
    got = host(out)
    want = den(x[k >= 0], k[k >= 0])
    err = rel_err(got[k >= 0], want)
    print(f"[lowrank d={d} r={r}] rows {int((k >= 0).sum())}/{R}, rel err {err:.2e}")
    assert err < 1e-5
    assert np.all(got[k < 0] == 777.0)
    # a smaller call after a larger one, and all rows masked
    g.sdden_eval(5, f32(x[:5]), dev(np.full(5, -1, np.int32), torch.int32), out[:5])
    assert np.all(host(out)[:5] == got[:5])


@pytest.mark.parametrize("d,H,E,T,R", [(256, 256, 8, 20, 300), (256, 512, 16, 40, 2000), (768, 256, 256, 30, 1100)])
def test_mlp_denoiser_matches_oracle(d, H, E, T, R):
    from paper_2501_05370_amd.binding import Denoiser
    rng = np.random.default_rng(1)
    p = W.random_mlp(rng, d, H, E)
    den = MLPDenoiser(p)
    g = Denoiser.sdden_mlp_create(p, T, R)
    x, k = _rows(rng, R, T, d)
    out = torch.full((R, d), 777.0, dtype=torch.float32, device="cuda")
    g.sdden_eval(R, f32(x), dev(k, torch.int32), out)
    got = host(out)
    want = den(x[k >= 0], k[k >= 0])
    err = rel_err(got[k >= 0], want)
    print(f"[mlp d={d} H={H}] rows {int((k >= 0).sum())}/{R}, rel err {err:.2e}, out rms {want.std():.3f}")
    assert err < 2e-2
    assert np.all(got[k < 0] == 777.0)
    # the time conditioning matters: the same rows at another step give another answer
    k2 = np.where(k >= 0, (k + 7) % T, -1).astype(np.int32)
    out2 = torch.zeros_like(out)
    g.sdden_eval(R, f32(x), dev(k2, torch.int32), out2)
    assert rel_err(host(out2)[k >= 0], den(x[k >= 0], k2[k >= 0])) < 2e-2
    assert np.abs(host(out2)[k >= 0] - got[k >= 0]).max() > 1e-3
    # with a bf16 image of the rows (what sd_draft can write) the first GEMM gathers from it and the
    # conversion pass is skipped: the result must be the same bits; masked rows carry garbage in the image
    xg = f32(x)
    img = xg.to(torch.bfloat16).view(torch.int16).contiguous()
    img[dev(k, torch.int32) < 0] = 0x7fc0
    out3 = torch.full((R, d), 777.0, dtype=torch.float32, device="cuda")
    g.sdden_eval_mirror(R, xg, img, dev(k, torch.int32), out3)
    assert np.array_equal(host(out3), got)


def test_mlp_denoiser_full_width_sampled_rows():
    """Config-4 widths (d = 12288, H = 4096, E = 256, bf16 weights): a few rows against the oracle."""
    from paper_2501_05370_amd.binding import Denoiser
    cfg = W.make_config("c4", B=4)
    den = MLPDenoiser(cfg.params)
    R = 40
    g = Denoiser.sdden_mlp_create(cfg.params, cfg.T, R)
    rng = np.random.default_rng(2)
    x, k = _rows(rng, R, cfg.T, cfg.d)
    out = torch.zeros(R, cfg.d, dtype=torch.float32, device="cuda")
    g.sdden_eval(R, f32(x), dev(k, torch.int32), out)
    want = den(x[k >= 0], k[k >= 0])
    err = rel_err(host(out)[k >= 0], want)
    print(f"[mlp c4 widths] rel err {err:.2e}, out rms {want.std():.3f}")
    assert err < 2e-2


def test_c3_shaped_window_pipeline():
    """Low-rank Gaussian chain (config-3 shape, reduced d): whole window S0..S6 against the oracle."""
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config("c3", B=96, d=512, r=32, T=50)
    den = LowRankDenoiser(cfg.params, cfg.schedule.alpha_bar_state)
    rng = np.random.default_rng(3)
    B, K, d, T = cfg.B, cfg.K, cfg.d, cfg.T
    n = rng.integers(0, T, size=B); n[:6] = [T - 1, T - 2, T - 5, 0, 1, T - K]
    ab = cfg.schedule.alpha_bar_state[n][:, None]
    x0 = cfg.params.mu + rng.standard_normal((B, cfg.params.U.shape[1])) @ cfg.params.U.T
    y = as_f32_f64(np.sqrt(ab) * x0 + np.sqrt(1 - ab) * rng.standard_normal((B, d)))
    ids = rng.permutation(B).astype(np.int64)
    res, Ytil, Dq, D0, krow, _ = S.window(cfg.schedule, den, y, n, ids, K, seed=cfg.seed)
    smp = make_sampler(cfg)
    b = smp.buf
    b.y.copy_(f32(y)); b.n.copy_(dev(n, torch.int32)); b.chain_id.copy_(dev(ids, torch.int64))
    smp.window(B)
    assert rel_err(host(b.D0), D0) < 1e-5
    assert rel_err(host(b.Ytilde), Ytil) < 1e-5
    mask = np.zeros((B, K), dtype=bool); mask[:, 1:] = krow[:, :K - 1] >= 0
    assert rel_err(host(b.Dq)[mask], Dq[mask]) < 2e-5
    # decisions: the predictions differ by fp32 rounding of the GEMMs, so the band is wider than
    # for verify on identical inputs: |delta log-ratio| <= |Z| * |delta Delta|, here below 1e-3
    nbad, near = decisions_match(host(b.adv), res, band=1e-3)
    print(f"[c3 window] mean adv {res.adv.mean():.2f} rejected {res.rejected.mean():.2f}, mismatches {nbad} (near ties {near})")
    assert nbad == near
    same = host(b.adv) == res.adv
    assert rel_err(host(b.y_out)[same], res.y_out[same]) < 5e-5


def test_c4_shaped_window_pipeline():
    """MLP chain (config-4 shape, reduced widths).  bf16 predictions move the log-ratios by far
    more than the near-tie band, so accept decisions are compared stage-wise (verify on oracle
    inputs, in test_gpu_window); here the states are checked at the bf16 tolerance."""
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config("c4", B=48, d=256, H=256, T=60)
    den = MLPDenoiser(cfg.params)
    rng = np.random.default_rng(4)
    B, K, d, T = cfg.B, cfg.K, cfg.d, cfg.T
    n = rng.integers(0, T, size=B); n[:4] = [T - 1, T - 2, 0, T - K]
    y = as_f32_f64(rng.standard_normal((B, d)))
    ids = np.arange(B, dtype=np.int64)
    res, Ytil, Dq, D0, krow, _ = S.window(cfg.schedule, den, y, n, ids, K, seed=cfg.seed)
    smp = make_sampler(cfg)
    b = smp.buf
    b.y.copy_(f32(y)); b.n.copy_(dev(n, torch.int32)); b.chain_id.copy_(dev(ids, torch.int64))
    smp.window(B)
    assert rel_err(host(b.D0), D0) < 2e-2
    assert rel_err(host(b.Ytilde), Ytil) < 2e-2
    assert np.array_equal(host(b.krow), krow)
    mask = np.zeros((B, K), dtype=bool); mask[:, 1:] = krow[:, :K - 1] >= 0
    assert rel_err(host(b.Dq)[mask], Dq[mask]) < 2e-2
    adv = host(b.adv)
    Kt = np.minimum(K, T - n)
    assert np.all(adv >= np.minimum(2, Kt)) and np.all(adv <= Kt)
    print(f"[c4 window] oracle mean adv {res.adv.mean():.2f}, gpu mean adv {adv.mean():.2f}, "
          f"same decisions on {np.mean(adv == res.adv):.2f} of chains")
    same = adv == res.adv
    assert same.mean() > 0.5
    assert rel_err(host(b.y_out)[same], res.y_out[same]) < 2e-2


def test_c4_shaped_efficient_frozen_window_uses_the_bf16_image():
    """Efficient frozen drafter on the MLP chain: the draft kernel writes the K+1 window rows (start state
    + drafts) both as fp32 and as a bf16 image, and the one batched target call gathers its rows from the
    image.  Drafts at the fp32 tolerance, image = round-to-nearest-even of the fp32 rows, predictions at the
    bf16 tolerance."""
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config("c4", B=40, d=256, H=256, K=6, T=50)
    den = MLPDenoiser(cfg.params)
    rng = np.random.default_rng(7)
    B, K, d, T = cfg.B, cfg.K, cfg.d, cfg.T
    n = rng.integers(0, T, size=B); n[:4] = [T - 1, T - 2, 0, T - K]
    y = as_f32_f64(rng.standard_normal((B, d)))
    ids = np.arange(B, dtype=np.int64)
    Dfz = as_f32_f64(den(y, n) + 0.1 * rng.standard_normal((B, d)))
    res, Ytil, Dq_ext, krow_ext, Dnext = S.window_efficient(cfg.schedule, den, y, n, ids, Dfz, K, cfg.seed)
    smp = make_sampler(cfg, drafter="efficient_frozen")
    assert smp.mirror is not None
    b = smp.buf
    b.y.copy_(f32(y)); b.n.copy_(dev(n, torch.int32)); b.chain_id.copy_(dev(ids, torch.int64)); b.Dfz.copy_(f32(Dfz))
    smp.window(B)
    X = host(b.X_ext)
    assert np.array_equal(X[:, 0], y.astype(np.float32))
    assert rel_err(X[:, 1:], Ytil) < 1e-5
    assert np.array_equal(host(b.krow_ext), krow_ext)
    img = smp.mirror.view(torch.bfloat16).float().cpu().numpy()
    want = torch.from_numpy(X).to(torch.bfloat16).float().numpy()
    assert np.array_equal(img, want)
    ev = krow_ext >= 0
    assert rel_err(host(b.Dq_ext)[ev], Dq_ext[ev]) < 2e-2
    adv = host(b.adv)
    Kt = np.minimum(K, T - n)
    assert np.all(adv >= 1) and np.all(adv <= Kt)


def test_step_indices_the_chain_does_not_have_are_masked_rows():
    """A step index >= T is treated like a negative one by every denoiser (their per-step tables end at T): the row
    is skipped and its output left untouched; and the draft kernel of the efficient frozen drafter asks for no
    prediction for a chain that is handed over at step T."""
    from paper_2501_05370_amd.binding import Denoiser, SD_DRAFT_FROZEN_REUSED
    rng = np.random.default_rng(3)
    T, R = 12, 70
    cases = []
    p = W.lowrank_gaussian(rng, 64, 8)
    sched = W.cosine_schedule(T)
    g = Denoiser.sdden_lowrank_create(p.mu, p.U, p.s2, sched.alpha_bar_state)
    g.sdden_reserve(R)
    cases.append((g, 64))
    pm = W.random_mlp(rng, 256, 256, 8)
    cases.append((Denoiser.sdden_mlp_create(pm, T, R), 256))
    cfg = W.make_config("c2", B=8, d=40, M=3, T=T)
    cases.append((Denoiser.sdden_gmm_create(cfg.params.means, cfg.params.stds, cfg.params.logw, cfg.schedule.alpha_bar_state), 40))
    for g, d in cases:
        x = as_f32_f64(rng.standard_normal((R, d)))
        k = rng.integers(0, T, size=R).astype(np.int32)
        bad = np.array([3, 17, 40, 69])
        k_bad = k.copy()
        k_bad[bad] = [T, T + 3, 2 ** 30, -5]
        out = torch.full((R, d), 777.0, dtype=torch.float32, device="cuda")
        g.sdden_eval(R, f32(x), dev(k_bad, torch.int32), out)
        ref = torch.full((R, d), 777.0, dtype=torch.float32, device="cuda")
        g.sdden_eval(R, f32(x), dev(k, torch.int32), ref)
        got, want = host(out), host(ref)
        ok = np.ones(R, dtype=bool); ok[bad] = False
        assert np.all(got[bad] == 777.0)
        assert np.array_equal(got[ok], want[ok])
    # sd_draft with one extra row per chain: row 0 carries the chain's own step, or -1 when the chain is at T
    K, d, B = 4, 8, 3
    ctx = make_context(W.linear_beta_schedule(T), d, K, seed=1, mode=SD_DRAFT_FROZEN_REUSED)
    n = np.array([0, T - 1, T], dtype=np.int32)
    X = torch.zeros(B, K + 1, d, dtype=torch.float32, device="cuda")
    kr = torch.full((B, K + 1), 99, dtype=torch.int32, device="cuda")
    ctx.sd_draft(B, f32(rng.standard_normal((B, d))), dev(n, torch.int32), dev(np.arange(B), torch.int64),
                 f32(rng.standard_normal((B, d))), X, kr)
    assert host(kr).tolist() == [[0, 1, 2, 3, 4], [T - 1, -1, -1, -1, -1], [-1, -1, -1, -1, -1]]


@pytest.mark.parametrize("R,pattern", [(8192 * 2, "random"), (8192 * 3 + 517, "random"), (8192 * 2 + 1, "last_share_masked"),
                                       (8193, "first_share_masked")])
def test_row_compaction_over_several_workgroups(R, pattern):
    """More rows than one workgroup of the row-compaction kernel ranks (8192): every workgroup has to place its
    kept rows behind those of the shares before it.  Checked through the low-rank denoiser, whose output rows
    must be the oracle's for every kept row and untouched for every masked one."""
    from paper_2501_05370_amd.binding import Denoiser
    d, r, T = 64, 8, 20
    rng = np.random.default_rng(7)
    p = W.lowrank_gaussian(rng, d, r)
    sched = W.cosine_schedule(T)
    den = LowRankDenoiser(p, sched.alpha_bar_state)
    g = Denoiser.sdden_lowrank_create(p.mu, p.U, p.s2, sched.alpha_bar_state)
    g.sdden_reserve(R)
    x, k = _rows(rng, R, T, d, 1.3)
    if pattern == "last_share_masked":
        k[8192 * 2:] = -1
    if pattern == "first_share_masked":
        k[:8192] = -1
    out = torch.full((R, d), 777.0, dtype=torch.float32, device="cuda")
    g.sdden_eval(R, f32(x), dev(k, torch.int32), out)
    got = host(out)
    want = den(x[k >= 0], k[k >= 0])
    err = rel_err(got[k >= 0], want)
    print(f"[row compaction R={R} {pattern}] rows {int((k >= 0).sum())}/{R}, rel err {err:.2e}")
    assert err < 1e-5
    assert np.all(got[k < 0] == 777.0)
