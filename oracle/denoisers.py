"""ORACLE (test infrastructure only) -- the target network's prediction D(y, k), in fp64.

The paper treats the drift b^q as a black box that a neural network stands in for (Sec. 3.1).  The
synthetic workloads replace it by functions with a plain definition, each written out here as that
definition:

* ``GMMDenoiser``        E[x0 | x_t] for x0 ~ sum_m w_m N(mu_m, diag(s_m^2)), x_t = sqrt(ab) x0 +
                          sqrt(1-ab) eps -- Bayes' rule over the components.
* ``LowRankDenoiser``    E[x0 | x_t] for x0 ~ N(mu, U U^T + s2 I) -- Gaussian conditioning, with the
                          (d x d) inverse taken through the Woodbury identity (an r x r solve).
* ``MLPDenoiser``        a 3-layer SiLU MLP on [x ; sinusoidal(k)], evaluated in fp64 on the
                          bf16-rounded weights.
* ``GMMScore``           grad E for E = -log sum_m w_m N(x; mu_m, s^2 I)  (Langevin target).

Every callable maps rows ``x [R, d]`` and integer chain steps ``k [R]`` to ``[R, d]``.
Pinned by tests/test_oracle_denoisers.py (single-component closed form, Tweedie's identity via
finite differences of log p_t, dense-solve comparison, hand-written loops on tiny sizes).
"""
from __future__ import annotations

import numpy as np

from workloads import GMMParams, LowRankGaussianParams, MLPParams, bf16_bits_to_f64


def _logsumexp(a: np.ndarray, axis: int) -> np.ndarray:
    m = np.max(a, axis=axis, keepdims=True)
    return np.squeeze(m, axis) + np.log(np.sum(np.exp(a - m), axis=axis))


class GMMDenoiser:
    """Posterior mean of a diagonal-covariance Gaussian mixture under the forward noising.

    Component m of the noised marginal: N(sqrt(ab) mu_m, diag(ab s_m^2 + 1 - ab)).
    Responsibilities r_m(x) are the softmax of log w_m + log N(x; ...), and
    E[x0 | x, m] = mu_m + sqrt(ab) s_m^2 / v_m * (x - sqrt(ab) mu_m)   (coordinate-wise).
    """

    def __init__(self, p: GMMParams, alpha_bar_state: np.ndarray):
        self.mu, self.s2, self.logw = p.means, p.stds ** 2, p.logw
        self.ab = np.asarray(alpha_bar_state, dtype=np.float64)

    def log_marginal(self, x: np.ndarray, k: np.ndarray):
        ab = self.ab[k][:, None, None]                              # [R,1,1]
        v = ab * self.s2[None] + (1.0 - ab)                         # [R,M,d]
        diff = x[:, None, :] - np.sqrt(ab) * self.mu[None]          # [R,M,d]
        logit = self.logw[None] - 0.5 * np.sum(diff ** 2 / v + np.log(2.0 * np.pi * v), axis=2)
        return _logsumexp(logit, 1), logit, diff, v, ab

    def __call__(self, x: np.ndarray, k: np.ndarray) -> np.ndarray:
        x = np.asarray(x, dtype=np.float64)
        k = np.asarray(k)
        out = np.empty_like(x)
        step = max(1, 2_000_000 // (self.mu.size))                  # bound the [R,M,d] temporaries
        for s in range(0, x.shape[0], step):
            xs, ks = x[s:s + step], k[s:s + step]
            lse, logit, diff, v, ab = self.log_marginal(xs, ks)
            r = np.exp(logit - lse[:, None])                        # [R,M]
            cond = self.mu[None] + np.sqrt(ab) * self.s2[None] / v * diff
            out[s:s + step] = np.sum(r[:, :, None] * cond, axis=1)
        return out


class LowRankDenoiser:
    """E[x0 | x_t] = mu + sqrt(ab) S (ab S + (1-ab) I)^-1 (x_t - sqrt(ab) mu),  S = U U^T + s2 I.

    With rho = ab s2 + 1 - ab:  (ab U U^T + rho I)^-1 v = (v - U (rho/ab I_r + U^T U)^-1 U^T v) / rho.
    """

    def __init__(self, p: LowRankGaussianParams, alpha_bar_state: np.ndarray):
        self.mu, self.U, self.s2 = p.mu, p.U, p.s2
        self.ab = np.asarray(alpha_bar_state, dtype=np.float64)
        self.UtU = self.U.T @ self.U

    def __call__(self, x: np.ndarray, k: np.ndarray) -> np.ndarray:
        x = np.asarray(x, dtype=np.float64)
        k = np.asarray(k)
        out = np.empty_like(x)
        r = self.U.shape[1]
        for kk in np.unique(k):
            rows = np.nonzero(k == kk)[0]
            ab = self.ab[kk]
            rho = ab * self.s2 + (1.0 - ab)
            v = (x[rows] - np.sqrt(ab) * self.mu).T                           # [d, n]
            if ab > 0.0:
                inner = np.linalg.solve((rho / ab) * np.eye(r) + self.UtU, self.U.T @ v)
                w = (v - self.U @ inner) / rho
            else:
                w = v / rho
            Sw = self.U @ (self.U.T @ w) + self.s2 * w
            out[rows] = (self.mu[:, None] + np.sqrt(ab) * Sw).T
        return out

    def affine_map(self, kk: int):
        """Dense (G, h) with D(x, k) = G x + h -- only for small d (tests of the chain marginal)."""
        d = self.mu.shape[0]
        ab = self.ab[kk]
        S = self.U @ self.U.T + self.s2 * np.eye(d)
        G = np.sqrt(ab) * S @ np.linalg.inv(ab * S + (1.0 - ab) * np.eye(d))
        return G, self.mu - np.sqrt(ab) * (G @ self.mu)


def sinusoidal_embedding(k: np.ndarray, E: int) -> np.ndarray:
    """emb[i] = sin(k w_i), emb[E/2+i] = cos(k w_i), w_i = 10000^(-i/(E/2)), i < E/2."""
    half = E // 2
    w = 10000.0 ** (-np.arange(half, dtype=np.float64) / half)
    ang = np.asarray(k, dtype=np.float64)[:, None] * w[None]
    return np.concatenate([np.sin(ang), np.cos(ang)], axis=1)


def silu(x):
    return x / (1.0 + np.exp(-x))


class MLPDenoiser:
    """D = W3^T silu(W2^T silu(W1^T [x ; emb(k)] + b1) + b2) + b3, weights are bf16 values."""

    def __init__(self, p: MLPParams):
        self.p = p
        self.W1 = bf16_bits_to_f64(p.W1)
        self.W2 = bf16_bits_to_f64(p.W2)
        self.W3 = bf16_bits_to_f64(p.W3)

    def __call__(self, x: np.ndarray, k: np.ndarray) -> np.ndarray:
        x = np.asarray(x, dtype=np.float64)
        inp = np.concatenate([x, sinusoidal_embedding(k, self.p.E)], axis=1)
        h1 = silu(inp @ self.W1 + self.p.b1)
        h2 = silu(h1 @ self.W2 + self.p.b2)
        return h2 @ self.W3 + self.p.b3


class GMMScore:
    """grad E(x) for the unnormalised Langevin target exp(-E), E = -log sum_m w_m N(x; mu_m, s^2 I):
    grad E = sum_m r_m(x) (x - mu_m) / s^2.  ``k`` is accepted and ignored (time-homogeneous)."""

    def __init__(self, p: GMMParams):
        self.mu, self.logw = p.means, p.logw
        s = np.unique(p.stds)
        assert s.size == 1, "Langevin target uses one shared isotropic std"
        self.s2 = float(s[0]) ** 2

    def energy(self, x: np.ndarray) -> np.ndarray:
        x = np.asarray(x, dtype=np.float64)
        d = x.shape[1]
        sq = np.sum((x[:, None, :] - self.mu[None]) ** 2, axis=2)
        return -_logsumexp(self.logw[None] - 0.5 * sq / self.s2
                           - 0.5 * d * np.log(2.0 * np.pi * self.s2), 1)

    def __call__(self, x: np.ndarray, k=None) -> np.ndarray:
        x = np.asarray(x, dtype=np.float64)
        out = np.empty_like(x)
        step = max(1, 4_000_000 // self.mu.size)
        for s in range(0, x.shape[0], step):
            xs = x[s:s + step]
            diff = xs[:, None, :] - self.mu[None]                    # [R,M,d]
            logit = self.logw[None] - 0.5 * np.sum(diff ** 2, axis=2) / self.s2
            r = np.exp(logit - _logsumexp(logit, 1)[:, None])
            out[s:s + step] = np.sum(r[:, :, None] * diff, axis=1) / self.s2
        return out
