"""Pins for the oracle's speculative unadjusted-Langevin sampler (no GPU)."""
import numpy as np
from scipy import stats

import workloads as W
from oracle import langevin as L
from oracle import speculative as S
from oracle.denoisers import GMMScore


def test_ula_window_is_the_general_window_with_langevin_coefficients():
    """ULA is the Gaussian chain a = 1, c = -gamma, sigma = sqrt(2 gamma), D = grad E; the
    separately written Langevin listing and the general detailed algorithm must agree."""
    rng = np.random.default_rng(0)
    d, M, K, T, B = 12, 3, 5, 9, 300
    gamma = float(np.float32(0.05))
    p = W.random_gmm(rng, M, d, 1.0, 1.0, 1.0, uniform_weights=False)
    sc = GMMScore(p)
    sched = W.langevin_schedule(T, 0.05)
    x = rng.standard_normal((B, d)) * 1.5
    n = rng.integers(0, T, size=B)
    ids = np.arange(B, dtype=np.int64) * 7
    xo, adv, rej, lr, lu = L.ula_window(sc, x, n, ids, K, T, gamma, seed=11)
    res, *_ = S.window(sched, lambda v, k: sc(v), x, n, ids, K, seed=11)
    assert rej.any() and (~rej).any()
    assert np.array_equal(adv, res.adv) and np.array_equal(rej, res.rejected)
    assert np.allclose(xo, res.y_out, atol=1e-6)          # sched holds fp32-rounded sqrt(2 gamma)
    assert np.allclose(lr, res.logratio, atol=1e-5) and np.allclose(lu, res.logu, atol=0)
    # with a proxy gradient (independent drafter)
    proxy = lambda v: sc(v) + 0.3
    xo2, adv2, rej2, _, _ = L.ula_window(sc, x, n, ids, K, T, gamma, seed=11, grad_proxy=proxy)
    res2, *_ = S.window(sched, lambda v, k: sc(v), x, n, ids, K, seed=11, drafter="independent",
                        D_draft=lambda v, k: proxy(v))
    assert np.array_equal(adv2, res2.adv) and np.allclose(xo2, res2.y_out, atol=1e-6)


def test_ula_exact_proxy_reproduces_sequential_ula():
    rng = np.random.default_rng(1)
    p = W.random_gmm(rng, 2, 4, 1.0, 1.0, 1.0)
    sc = GMMScore(p)
    seq = L.ula_sequential(sc, 20, 4, 17, 0.02, seed=2)
    out, cw, rejections = L.ula_sample(sc, 20, 4, 5, 17, 0.02, seed=2, grad_proxy=sc)
    assert np.array_equal(out, seq) and rejections == 0 and cw == 20 * 4


def test_speculative_ula_stationary_variance_on_quadratic_energy():
    """E = x^2/(2 s^2): ULA is AR(1) with coefficient 1 - gamma/s^2 and innovation variance
    2 gamma, so its stationary variance is s^2 / (1 - gamma/(2 s^2)).  Frozen-gradient
    speculative ULA must have the same law as plain ULA."""
    s2, gamma, T, K, B = 0.5, 0.1, 120, 8, 40_000
    grad = lambda x: x / s2
    var_inf = s2 / (1 - gamma / (2 * s2))
    rho = 1 - gamma / s2
    var_T = rho ** (2 * T) * 1.0 + var_inf * (1 - rho ** (2 * T))     # X_0 ~ N(0,1)
    out, cw, rejections = L.ula_sample(grad, B, 1, K, T, gamma, seed=3)
    assert rejections > 0.2 * cw
    assert abs(out.var() - var_T) < 5 * var_T * np.sqrt(2 / B)
    assert stats.kstest(out[:, 0] / np.sqrt(var_T), "norm").pvalue > 1e-4
    seq = L.ula_sequential(grad, B, 1, T, gamma, seed=4)
    assert stats.ks_2samp(out[:, 0], seq[:, 0]).pvalue > 1e-4
