"""Pins for the oracle's rejection mechanism (reflection maximal coupling). No GPU.

Sources: Prop. "Reflection Coupling" (acceptance probability = 1 - TV), its proof (output law
N(m^q, sigma^2 I); the reflection preserves norms and is an involution), the identity
q(Y~)/p(Y~) = N(Z+Delta)/N(Z) of Sec. 3.3, and the worked Gaussian pairs of two figures.
"""
import os

import numpy as np
from scipy import stats

from oracle.speculative import incorrect_rejection, reflection_rejection

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_gaussian_pairs.txt")


def _draws(rng, mp, sigma, N):
    d = mp.shape[0]
    z = rng.standard_normal((N, d))
    u = rng.uniform(size=N)
    return mp[None] + sigma * z, z, u


def test_worked_pairs_acceptance_probability():
    rng = np.random.default_rng(1)
    rows = [list(map(float, l.split())) for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for mp, mq, sigma, p_acc in rows:
        # the stored value is what the closed form gives for the printed parameters
        assert abs(2 * stats.norm.cdf(-abs(mp - mq) / (2 * sigma)) - p_acc) < 1e-12
        N = 400_000
        ytil, _, u = _draws(rng, np.array([mp]), sigma, N)
        _, acc, _ = reflection_rejection(np.full((N, 1), mp), np.full((N, 1), mq),
                                         np.full(N, sigma), ytil, u)
        se = np.sqrt(p_acc * (1 - p_acc) / N)
        assert abs(acc.mean() - p_acc) < 4 * se


def test_acceptance_probability_is_one_minus_tv_any_dimension():
    rng = np.random.default_rng(2)
    for d, sigma, dist in [(1, 0.7, 0.5), (3, 0.2, 0.3), (16, 1.3, 2.0), (64, 0.05, 0.1)]:
        mp = rng.standard_normal(d)
        direction = rng.standard_normal(d)
        mq = mp + dist * direction / np.linalg.norm(direction)
        N = 200_000
        ytil, _, u = _draws(rng, mp, sigma, N)
        _, acc, _ = reflection_rejection(np.broadcast_to(mp, (N, d)), np.broadcast_to(mq, (N, d)),
                                         np.full(N, sigma), ytil, u)
        p = 2 * stats.norm.cdf(-dist / (2 * sigma))
        assert abs(acc.mean() - p) < 4 * np.sqrt(p * (1 - p) / N), (d, acc.mean(), p)


def test_log_ratio_equals_naive_log_densities():
    rng = np.random.default_rng(3)
    d, sigma = 5, 0.37
    mp, mq = rng.standard_normal(d), rng.standard_normal(d)
    ytil, _, u = _draws(rng, mp, sigma, 2000)
    _, _, lr = reflection_rejection(np.broadcast_to(mp, ytil.shape), np.broadcast_to(mq, ytil.shape),
                                    np.full(2000, sigma), ytil, u)
    naive = (stats.multivariate_normal(mq, sigma ** 2 * np.eye(d)).logpdf(ytil)
             - stats.multivariate_normal(mp, sigma ** 2 * np.eye(d)).logpdf(ytil))
    assert np.max(np.abs(lr - naive)) < 1e-9
    # E[log ratio] = -|Delta|^2 / 2  (App. "Lower bound on acceptance ratio", first display)
    N = 400_000
    ytil, _, u = _draws(rng, mp, sigma, N)
    _, _, lr = reflection_rejection(np.broadcast_to(mp, ytil.shape), np.broadcast_to(mq, ytil.shape),
                                    np.full(N, sigma), ytil, u)
    D2 = np.sum((mp - mq) ** 2) / sigma ** 2
    assert abs(lr.mean() + 0.5 * D2) < 5 * np.sqrt(D2 / N)


def test_output_law_is_target_and_reflection_invariants():
    rng = np.random.default_rng(4)
    for d in (1, 2, 8):
        sigma = 0.6
        mp = rng.standard_normal(d)
        mq = mp + rng.standard_normal(d) * 0.8 / np.sqrt(d)
        N = 300_000
        ytil, z, u = _draws(rng, mp, sigma, N)
        MP, MQ = np.broadcast_to(mp, (N, d)), np.broadcast_to(mq, (N, d))
        Y, acc, _ = reflection_rejection(MP, MQ, np.full(N, sigma), ytil, u)
        assert 0.05 < acc.mean() < 0.95                       # both branches exercised
        # accepted drafts are returned untouched
        assert np.array_equal(Y[acc], ytil[acc])
        zt = (Y - mq) / sigma
        # pooled output ~ N(mq, sigma^2 I)
        assert np.all(np.abs(zt.mean(0)) < 4.5 / np.sqrt(N))
        cov = np.cov(zt.T).reshape(d, d)
        assert np.max(np.abs(cov - np.eye(d))) < 6 / np.sqrt(N) * 2
        for i in range(d):
            assert stats.kstest(zt[:, i], "norm").pvalue > 1e-4
        # along the direction e the law must be N(0,1) as well (this is where a wrong sign shows)
        e = (mp - mq) / np.linalg.norm(mp - mq)
        assert stats.kstest(zt @ e, "norm").pvalue > 1e-4
        # on rejection: norm preserved, only the component along Delta changes, involution
        rej = ~acc
        Delta = (mp - mq) / sigma
        zr, ztr = z[rej], zt[rej]
        assert np.allclose(np.linalg.norm(ztr, axis=1), np.linalg.norm(zr, axis=1), rtol=1e-12)
        diff = ztr - zr
        cosang = np.abs(diff @ Delta) / (np.linalg.norm(diff, axis=1) * np.linalg.norm(Delta))
        assert np.allclose(cosang, 1.0, atol=1e-9)
        H = np.eye(d) - 2 * np.outer(e, e)
        assert np.allclose(ztr, zr @ H.T, atol=1e-12)
        assert np.allclose(ztr @ H.T, zr, atol=1e-12)
        # a rejected draft has log ratio < 0, i.e. Z.Delta > -|Delta|^2/2, and |Delta| > 0:
        # the reflection is well defined whenever it is needed
        assert np.all(zr @ Delta > -0.5 * Delta @ Delta)


def test_equal_means_always_accept_and_never_nan():
    rng = np.random.default_rng(5)
    m = rng.standard_normal((100, 4))
    ytil = m + 0.3 * rng.standard_normal((100, 4))
    Y, acc, lr = reflection_rejection(m, m, np.full(100, 0.3), ytil, rng.uniform(size=100))
    assert acc.all() and np.array_equal(Y, ytil) and np.all(lr == 0) and np.isfinite(Y).all()


def test_temperature_limits():
    rng = np.random.default_rng(6)
    d, sigma, N = 3, 0.5, 50_000
    mp, mq = np.zeros(d), np.array([0.6, 0.0, 0.0])
    ytil, _, u = _draws(rng, mp, sigma, N)
    MP, MQ, S = np.broadcast_to(mp, (N, d)), np.broadcast_to(mq, (N, d)), np.full(N, sigma)
    Y1, a1, l1 = reflection_rejection(MP, MQ, S, ytil, u, tau=1.0)
    Yd, ad, ld = reflection_rejection(MP, MQ, S, ytil, u)
    assert np.array_equal(Y1, Yd) and np.array_equal(a1, ad)
    _, ainf, _ = reflection_rejection(MP, MQ, S, ytil, u, tau=1e12)
    assert ainf.mean() > 0.999                                  # tau -> infinity always accepts
    _, a2, l2 = reflection_rejection(MP, MQ, S, ytil, u, tau=2.0)
    assert np.allclose(l2, l1 / 2) and a2.mean() > a1.mean()


def test_discrete_example_of_the_incorrect_mechanism():
    """p = Unif{0,1}, q = Unif{0,1,2,3}: accept w.p. 1/2; resampling from q on rejection gives
    3/4 mass on {0,1}; the residual max(0, q-p) is Unif{2,3} and restores q (paper's example)."""
    p = np.array([.5, .5, 0, 0])
    q = np.full(4, .25)
    acc_prob = np.sum(p * np.minimum(1, q / np.where(p > 0, p, 1)))
    assert acc_prob == 0.5
    wrong = p * np.minimum(1, q / np.where(p > 0, p, 1)) + (1 - acc_prob) * q
    assert np.allclose(wrong, [.375, .375, .125, .125])
    resid = np.maximum(0, q - p)
    resid /= resid.sum()
    assert np.allclose(resid, [0, 0, .5, .5])
    right = p * np.minimum(1, q / np.where(p > 0, p, 1)) + (1 - acc_prob) * resid
    assert np.allclose(right, q)


def test_incorrect_mechanism_has_wrong_output_law():
    rng = np.random.default_rng(7)
    d, sigma, N = 1, 0.5, 200_000
    mp, mq = np.array([1.0]), np.array([3.0])                   # the temperature figure's pair
    ytil, _, u = _draws(rng, mp, sigma, N)
    MP, MQ, S = np.broadcast_to(mp, (N, d)), np.broadcast_to(mq, (N, d)), np.full(N, sigma)
    Yr, _, _ = reflection_rejection(MP, MQ, S, ytil, u)
    Yw, _, _ = incorrect_rejection(MP, MQ, S, ytil, u, rng.standard_normal((N, d)))
    assert stats.kstest((Yr[:, 0] - 3.0) / sigma, "norm").pvalue > 1e-4
    assert stats.kstest((Yw[:, 0] - 3.0) / sigma, "norm").pvalue < 1e-12


def test_temperature_mean_shift_closed_form():
    """App. "Influence of the temperature", Prop. "Link with guidance": E[Y] = m^q + C_tau (m^p - m^q)
    with C_tau = 0 at tau = 1, < 0 below and > 0 above.  The expression printed for C_tau does not
    reproduce the mechanism's mean (checked by Monte Carlo), so the pin is the closed form obtained
    by integrating the algorithm directly along e = Delta/|Delta| (D = |Delta|, w0 = D(1/tau - 1/2),
    c = exp(D^2 (1 - tau) / (2 tau^2))):
        D C_tau = -2 phi(D/2) + D Phi(-D/2) + c [ 2 phi(w0) + D (1 - 2/tau) Phi(-w0) ]."""
    rng = np.random.default_rng(8)
    Phi, phi = stats.norm.cdf, stats.norm.pdf

    def C(D, tau):
        w0 = D * (1 / tau - 0.5)
        c = np.exp(D * D * (1 - tau) / (2 * tau * tau))
        return (-2 * phi(D / 2) + D * Phi(-D / 2) + c * (2 * phi(w0) + D * (1 - 2 / tau) * Phi(-w0))) / D

    assert abs(C(1.3, 1.0)) < 1e-15
    assert abs(C(0.7, 1e9) - 1.0) < 1e-6                       # tau -> infinity: Y ~ p, mean m^p
    for tau in (0.5, 2.0, 4.0):
        for d, sigma, dist in ((1, 0.5, 2.0), (3, 1.0, 1.0), (6, 2.0, 1.2)):
            N = 1_000_000
            mp = rng.standard_normal(d)
            direction = rng.standard_normal(d)
            mq = mp + dist * direction / np.linalg.norm(direction)
            ytil, _, u = _draws(rng, mp, sigma, N)
            Y, _, _ = reflection_rejection(np.broadcast_to(mp, (N, d)), np.broadcast_to(mq, (N, d)),
                                           np.full(N, sigma), ytil, u, tau)
            D = dist / sigma
            shift = (Y.mean(0) - mq) @ (mp - mq) / dist ** 2     # component of E[Y] - m^q along m^p - m^q
            se = sigma / dist / np.sqrt(N) * 2
            assert abs(shift - C(D, tau)) < 5 * se, (tau, d, shift, C(D, tau))
            assert (C(D, tau) < 0) == (tau < 1)
            # nothing moves orthogonally to e
            orth = (Y.mean(0) - mq) - shift * (mp - mq)
            assert np.linalg.norm(orth) < 6 * sigma * np.sqrt(d / N)
