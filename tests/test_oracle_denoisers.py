"""Pins for the oracle's analytic / MLP predictions and for the schedule coefficients. No GPU."""
import numpy as np
from scipy import stats
from scipy.special import logsumexp

import workloads as W
from oracle.denoisers import (GMMDenoiser, GMMScore, LowRankDenoiser, MLPDenoiser,
                              sinusoidal_embedding)


# ------------------------------------------------------------------ schedules
def test_ddpm_coefficients_are_the_gaussian_posterior_mean():
    """a_k, c_k must be E[x_{t-1} | x_t, x0] for the forward chain, obtained here by plain
    bivariate-Gaussian conditioning instead of the textbook closed form."""
    f = lambda t, T: np.cos((t / T + 0.008) / 1.008 * np.pi / 2) ** 2
    lin_ab = np.concatenate([[1.0], np.cumprod(1 - np.linspace(1e-4, 0.02, 50))])
    cos_ab = f(np.arange(41), 40) / f(0, 40)
    cos_ab[40] = cos_ab[39] * (1 - 0.999)                      # the last beta is clipped to 0.999
    for sched, ab in ((W.linear_beta_schedule(50), lin_ab), (W.cosine_schedule(40), cos_ab)):
        T = sched.T
        assert np.allclose(sched.alpha_bar_state[::-1], ab, rtol=1e-6, atol=1e-9)
        assert ab[0] == 1.0 and np.all(np.diff(ab) < 0)
        for k in (0, 1, T // 2, T - 2, T - 1):
            t = T - k
            alpha_t = ab[t] / ab[t - 1]
            # x_{t-1} | x0 ~ N(sqrt(ab_{t-1}) x0, 1-ab_{t-1});  x_t = sqrt(alpha_t) x_{t-1} + sqrt(beta_t) e
            var_prev = 1 - ab[t - 1]
            cov = np.sqrt(alpha_t) * var_prev
            var_t = alpha_t * var_prev + (1 - alpha_t)
            coef_xt = cov / var_t
            coef_x0 = np.sqrt(ab[t - 1]) - coef_xt * np.sqrt(alpha_t) * np.sqrt(ab[t - 1])
            assert abs(sched.a[k] - coef_xt) < 2e-7 * max(1, abs(coef_xt))
            assert abs(sched.c[k] - coef_x0) < 2e-7 * max(1, abs(coef_x0))
            assert abs(sched.sigma[k] ** 2 - (1 - alpha_t)) < 1e-7
    lin = W.linear_beta_schedule(100)
    assert abs(lin.sigma[0] ** 2 - 0.02) < 1e-7 and abs(lin.sigma[-1] ** 2 - 1e-4) < 1e-9
    assert lin.a[-1] == 0.0 and abs(lin.c[-1] - 1.0) < 1e-6     # last step returns the prediction
    cos = W.cosine_schedule(200)
    assert np.all(cos.sigma > 0) and np.all(cos.sigma ** 2 <= 0.999 + 1e-6)
    assert abs(cos.alpha_bar_state[100] - f(100, 200) / f(0, 200)) < 1e-7


def test_langevin_schedule():
    s = W.langevin_schedule(10, 1e-2)
    g = float(np.float32(1e-2))
    assert np.all(s.a == 1) and np.allclose(s.c, -g, rtol=1e-7) and np.allclose(s.sigma, np.sqrt(2 * g), rtol=1e-7)


# ------------------------------------------------------------------ GMM posterior mean
def _gmm_logpt(p, ab, x):
    comps = [p.logw[m] + stats.multivariate_normal(np.sqrt(ab) * p.means[m],
                                                   np.diag(ab * p.stds[m] ** 2 + 1 - ab)).logpdf(x)
             for m in range(p.means.shape[0])]
    return logsumexp(np.stack(comps, 0), axis=0)


def test_gmm_denoiser_tweedie_identity():
    """E[x0|x_t] = (x_t + (1-ab) grad log p_t(x_t)) / sqrt(ab), the gradient taken by central
    differences of a log-density assembled from scipy's multivariate normal."""
    rng = np.random.default_rng(0)
    p = W.random_gmm(rng, 5, 3, 2.0, 0.2, 1.0, uniform_weights=False)
    sched = W.cosine_schedule(20)
    den = GMMDenoiser(p, sched.alpha_bar_state)
    x = rng.standard_normal((6, 3)) * 1.5
    for k in (0, 7, 15, 19):
        ab = sched.alpha_bar_state[k]
        D = den(x, np.full(6, k))
        h = 1e-5
        grad = np.zeros_like(x)
        for i in range(3):
            e = np.zeros(3); e[i] = h
            grad[:, i] = (_gmm_logpt(p, ab, x + e) - _gmm_logpt(p, ab, x - e)) / (2 * h)
        tweedie = (x + (1 - ab) * grad) / np.sqrt(ab)
        assert np.max(np.abs(D - tweedie)) < 1e-5 * max(1.0, np.abs(tweedie).max()), k
        assert np.allclose(den.log_marginal(x, np.full(6, k))[0], _gmm_logpt(p, ab, x), atol=1e-10)


def test_gmm_denoiser_brute_force_posterior_mean():
    """Self-normalised importance sampling of E[x0 | x_t] from draws of the mixture (d = 2)."""
    rng = np.random.default_rng(1)
    p = W.ring_gmm()
    sched = W.linear_beta_schedule(100)
    den = GMMDenoiser(p, sched.alpha_bar_state)
    N = 2_000_000
    comp = rng.integers(0, 8, size=N)
    x0 = p.means[comp] + p.stds[comp] * rng.standard_normal((N, 2))
    k = 30
    ab = sched.alpha_bar_state[k]
    for xt in (np.array([1.0, 0.5]), np.array([-2.0, 1.0])):
        logw = -0.5 * np.sum((xt - np.sqrt(ab) * x0) ** 2, axis=1) / (1 - ab)
        w = np.exp(logw - logw.max())
        est = (w[:, None] * x0).sum(0) / w.sum()
        D = den(xt[None], np.array([k]))[0]
        assert np.max(np.abs(D - est)) < 0.03, (D, est)


def test_gmm_single_component_rows_with_mixed_steps():
    rng = np.random.default_rng(2)
    p = W.random_gmm(rng, 1, 4, 1.0, 0.5, 0.5)
    sched = W.cosine_schedule(10)
    den = GMMDenoiser(p, sched.alpha_bar_state)
    x = rng.standard_normal((5, 4))
    k = np.array([0, 3, 3, 9, 5])
    D = den(x, k)
    for r in range(5):                                          # Gaussian conditioning, dense
        ab = sched.alpha_bar_state[k[r]]
        S = np.diag(p.stds[0] ** 2)
        G = np.sqrt(ab) * S @ np.linalg.inv(ab * S + (1 - ab) * np.eye(4))
        assert np.allclose(D[r], p.means[0] + G @ (x[r] - np.sqrt(ab) * p.means[0]), atol=1e-12)


# ------------------------------------------------------------------ low-rank Gaussian
def test_lowrank_denoiser_against_dense_solve_and_tweedie():
    rng = np.random.default_rng(3)
    p = W.lowrank_gaussian(rng, 12, 3)
    sched = W.cosine_schedule(25)
    den = LowRankDenoiser(p, sched.alpha_bar_state)
    x = rng.standard_normal((7, 12))
    k = np.array([0, 24, 10, 10, 3, 17, 24])
    D = den(x, k)
    S = p.U @ p.U.T + p.s2 * np.eye(12)
    for r in range(7):
        ab = sched.alpha_bar_state[k[r]]
        C = ab * S + (1 - ab) * np.eye(12)
        dense = p.mu + np.sqrt(ab) * S @ np.linalg.solve(C, x[r] - np.sqrt(ab) * p.mu)
        assert np.allclose(D[r], dense, atol=1e-10)
        score = -np.linalg.solve(C, x[r] - np.sqrt(ab) * p.mu)   # grad log N(sqrt(ab) mu, C)
        assert np.allclose(D[r], (x[r] + (1 - ab) * score) / np.sqrt(ab), atol=1e-9)
        G, h = den.affine_map(int(k[r]))
        assert np.allclose(D[r], G @ x[r] + h, atol=1e-10)


# ------------------------------------------------------------------ MLP
def test_mlp_denoiser_against_scalar_loops():
    rng = np.random.default_rng(4)
    p = W.random_mlp(rng, 5, 7, E=4)
    den = MLPDenoiser(p)
    W1, W2, W3 = (W.bf16_bits_to_f64(w) for w in (p.W1, p.W2, p.W3))
    x = rng.standard_normal((3, 5))
    k = np.array([0, 2, 11])
    out = den(x, k)
    for r in range(3):
        emb = [np.sin(k[r] * 1.0), np.sin(k[r] * 10000.0 ** -0.5),
               np.cos(k[r] * 1.0), np.cos(k[r] * 10000.0 ** -0.5)]
        inp = list(x[r]) + emb
        h1 = []
        for o in range(7):
            s = p.b1[o] + sum(inp[i] * W1[i, o] for i in range(9))
            h1.append(s / (1 + np.exp(-s)))
        h2 = []
        for o in range(7):
            s = p.b2[o] + sum(h1[i] * W2[i, o] for i in range(7))
            h2.append(s / (1 + np.exp(-s)))
        for o in range(5):
            s = p.b3[o] + sum(h2[i] * W3[i, o] for i in range(7))
            assert abs(out[r, o] - s) < 1e-12


def test_bf16_rounding_of_weights():
    x = np.array([1.0, 1.00390625, 1.005859375, -3.14159, 1e-3, 65504.0], dtype=np.float32)
    bits = W.bf16_round_bits(x)
    back = W.bf16_bits_to_f64(bits)
    assert back[0] == 1.0
    assert back[1] == 1.0                    # 1 + 2^-8 is a tie: rounds to even (1.0)
    assert back[2] == 1.0078125              # 1 + 1.5*2^-8 rounds up to 1 + 2^-7
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)
    assert sinusoidal_embedding(np.array([0]), 8).tolist() == [[0, 0, 0, 0, 1, 1, 1, 1]]


# ------------------------------------------------------------------ Langevin score
def test_gmm_score_is_gradient_of_energy():
    rng = np.random.default_rng(5)
    p = W.random_gmm(rng, 4, 6, 1.0, 1.0, 1.0, uniform_weights=False)
    sc = GMMScore(p)
    x = rng.standard_normal((5, 6))
    # energy against scipy's mixture log-density
    comps = np.stack([p.logw[m] + stats.multivariate_normal(p.means[m], np.eye(6)).logpdf(x)
                      for m in range(4)], 0)
    assert np.allclose(sc.energy(x), -logsumexp(comps, axis=0), atol=1e-12)
    g = sc(x)
    h = 1e-6
    for i in range(6):
        e = np.zeros(6); e[i] = h
        fd = (sc.energy(x + e) - sc.energy(x - e)) / (2 * h)
        assert np.allclose(g[:, i], fd, atol=1e-6)
