"""ORACLE (test infrastructure only) -- speculative sampling for unadjusted Langevin, in fp64.

What it computes (Sec. 5 and the Langevin appendix, Alg. "Speculative Sampling for Unadjusted
Langevin Diffusion"), vectorised over independent chains only.  The target chain is unadjusted
Langevin on an energy E: a gradient step of size gamma plus Gaussian noise of variance 2 gamma.
The draft chain is the same step with a cheaper gradient in place of grad E -- a proxy energy's, or
the gradient at the window's first state kept for the whole window (the frozen drafter).  A window
drafts up to K states one after the other, evaluates grad E at all of them at once, and then walks
them in order: each drafted state is tested with the reflection-coupling rule for two Gaussians of
equal covariance whose means differ by sqrt(2 gamma) * Delta, Delta being sqrt(gamma/2) times the
gap between the true and the proxy gradient at the previous state, with Z the noise that drew the
draft; the first rejected draft is replaced by the target step from the previous state driven by
Z reflected across Delta, and the window ends there.  The optional temperature divides the log
acceptance ratio (App. "Influence of the temperature"); 1 is the exact sampler.

Readings: the reject branch of the appendix's algorithm prints the energy where the target step
needs its gradient (taken as the gradient, as in the target update); the start state is drawn
N(0, Id) from the keyed initial stream (the paper leaves it arbitrary).

This is written independently of oracle/speculative.py on purpose: the two formulations are
pinned to each other in tests/test_oracle_langevin.py (the ULA chain is the general Gaussian
chain with a = 1, c = -gamma, sigma = sqrt(2 gamma), D = grad E), and to the stationary
variance of ULA on a quadratic energy.
"""
from __future__ import annotations

from typing import Callable, Optional

import numpy as np

from . import philox

Grad = Callable[[np.ndarray], np.ndarray]


class Phi4Energy:
    """The phi^4 lattice energy of the Langevin appendix on an L x L grid,
        E(x) = (beta/2) sum_{|i-j|=1} (x_i - x_j)^2 + sum_i (x_i^2 - 1)^2.
    Reading (the text fixes neither): the neighbour sum runs over ORDERED pairs, so every bond of the
    grid counts twice, and the grid is periodic.  Of the four combinations (ordered / unordered
    pairs, periodic / free boundary) this is the one whose plain ULA run (step 1e-3, 1e5 iterations,
    beta = 100, 8 x 8) reproduces the mean energy printed in the table of that appendix (62.27);
    the others give about 41, 40 and 56.
        grad E_i = 2 beta (4 x_i - sum of the four neighbours) + 4 x_i (x_i^2 - 1).
    Sites are numbered row by row, i = row * L + col."""

    def __init__(self, L: int, beta: float):
        assert L >= 3, "with L < 3 the four neighbours of a site are not distinct"
        self.L, self.beta = int(L), float(beta)

    def _grid(self, x):
        x = np.asarray(x, dtype=np.float64)
        return x.reshape(x.shape[0], self.L, self.L)

    def energy(self, x) -> np.ndarray:
        X = self._grid(x)
        bonds = np.sum((X - np.roll(X, 1, axis=1)) ** 2, axis=(1, 2)) + np.sum((X - np.roll(X, 1, axis=2)) ** 2, axis=(1, 2))
        return self.beta * bonds + np.sum((X * X - 1.0) ** 2, axis=(1, 2))

    def __call__(self, x, k=None) -> np.ndarray:
        X = self._grid(x)
        nb = np.roll(X, 1, axis=1) + np.roll(X, -1, axis=1) + np.roll(X, 1, axis=2) + np.roll(X, -1, axis=2)
        g = 2.0 * self.beta * (4.0 * X - nb) + 4.0 * X * (X * X - 1.0)
        return g.reshape(np.asarray(x).shape)


def ula_window(gradE: Grad, x, n, chain_id, K: int, T: int, gamma: float, seed: int,
               grad_proxy: Optional[Grad] = None, tau: float = 1.0):
    """One window for every chain.  Returns (x_out [B,d], adv [B], rejected [B],
    logratio [B,K], logu [B,K]).  ``grad_proxy`` None = frozen gradient; ``tau`` = temperature of
    the accept test (the reported log-ratios are already divided by it)."""
    x = np.asarray(x, dtype=np.float64)
    n = np.asarray(n)
    B, d = x.shape
    Kt = np.minimum(K, T - n)
    sq2g = np.sqrt(2.0 * gamma)
    g_start = gradE(x)
    # -- draft states, sequentially, remembering the noise that drew them
    Ytil = np.zeros((B, K + 1, d))
    Ytil[:, 0] = x
    Z = np.zeros((B, K, d))
    Ghat = np.zeros((B, K, d))
    for j in range(1, K + 1):
        act = np.nonzero(j <= Kt)[0]
        if act.size == 0:
            break
        gh = g_start[act] if grad_proxy is None else grad_proxy(Ytil[act, j - 1])
        z = philox.normals(seed, chain_id[act], n[act] + j, d)
        Ytil[act, j] = Ytil[act, j - 1] - gamma * gh + sq2g * z
        Z[act, j - 1] = z
        Ghat[act, j - 1] = gh
    # -- in parallel: grad E at Y~_n .. Y~_{n_L - 1}
    G = np.zeros((B, K, d))
    G[:, 0] = g_start
    for j in range(2, K + 1):
        act = np.nonzero(j <= Kt)[0]
        if act.size:
            G[act, j - 1] = gradE(Ytil[act, j - 1])
    # -- sequential accept / reject
    x_out = np.zeros((B, d))
    adv = np.zeros(B, dtype=np.int32)
    rejected = np.zeros(B, dtype=bool)
    logratio = np.zeros((B, K))
    logu = np.zeros((B, K))
    running = np.ones(B, dtype=bool)
    for j in range(1, K + 1):
        act = np.nonzero(j <= Kt)[0]
        if act.size == 0:
            break
        Delta = np.sqrt(gamma / 2.0) * (G[act, j - 1] - Ghat[act, j - 1])
        z = Z[act, j - 1]
        zd = np.sum(z * Delta, axis=1)
        dd = np.sum(Delta * Delta, axis=1)
        lr = (-zd - 0.5 * dd) / tau                           # (log N(Z+Delta) - log N(Z)) / tau
        lu = np.log(philox.uniforms(seed, chain_id[act], n[act] + j))
        acc = (dd == 0.0) | (lu <= np.minimum(0.0, lr))
        with np.errstate(divide="ignore", invalid="ignore"):
            coef = np.where(dd > 0.0, zd / dd, 0.0)
        refl = (Ytil[act, j - 1] - gamma * G[act, j - 1]
                + sq2g * (z - 2.0 * coef[:, None] * Delta))
        Y = np.where(acc[:, None], Ytil[act, j], refl)
        logratio[act, j - 1] = lr
        logu[act, j - 1] = lu
        live = running[act]
        upd = act[live]
        x_out[upd] = Y[live]
        adv[upd] = j
        rej_now = act[live & ~acc]
        rejected[rej_now] = True
        running[rej_now] = False
    return x_out, adv, rejected, logratio, logu


def ula_sample(gradE: Grad, B: int, d: int, K: int, T: int, gamma: float, seed: int,
               grad_proxy: Optional[Grad] = None, chain_ids: Optional[np.ndarray] = None, tau: float = 1.0):
    """Whole algorithm; X_0 ~ N(0, Id) from the keyed initial stream (the paper leaves the start arbitrary).
    Returns (X_T in the order of chain_ids, total windows over chains, total rejections)."""
    ids0 = np.arange(B, dtype=np.int64) if chain_ids is None else np.asarray(chain_ids, dtype=np.int64)
    ids = ids0.copy()
    pos = np.arange(ids.shape[0])
    x = philox.initial_state(seed, ids, d)
    n = np.zeros(ids.shape[0], dtype=np.int64)
    out = np.zeros((ids.shape[0], d))
    chain_windows = 0
    rejections = 0
    while n.size:
        x_out, adv, rej, _, _ = ula_window(gradE, x, n, ids, K, T, gamma, seed, grad_proxy, tau)
        chain_windows += n.size
        rejections += int(rej.sum())
        n = n + adv
        done = n >= T
        out[pos[done]] = x_out[done]
        keep = ~done
        x, n, ids, pos = x_out[keep], n[keep], ids[keep], pos[keep]
    return out, chain_windows, rejections


def ula_sequential(gradE: Grad, B: int, d: int, T: int, gamma: float, seed: int,
                   chain_ids: Optional[np.ndarray] = None):
    """Plain ULA with the same keyed noise."""
    ids = np.arange(B, dtype=np.int64) if chain_ids is None else np.asarray(chain_ids, dtype=np.int64)
    x = philox.initial_state(seed, ids, d)
    sq2g = np.sqrt(2.0 * gamma)
    for k in range(T):
        z = philox.normals(seed, ids, np.full(ids.shape[0], k + 1), d)
        x = x - gamma * gradE(x) + sq2g * z
    return x
