"""Seeded synthetic workloads: the inputs that both the CPU oracle and the HIP library consume.

This module only *describes problems*: noise schedules as the per-step coefficient arrays of
a Gaussian transition, the parameters of the synthetic data distributions, random-init network
weights, and the five benchmark configurations.  It contains none of the sampler's arithmetic
(no drafting, no accept test, no reflection, no denoiser evaluation, no random-stream
generator for the chains): those are written twice, independently, in ``oracle/`` and in the
HIP library.

Every array that crosses into the fp32 C-ABI is rounded to fp32 here and handed to the oracle
as the fp64 image of those same fp32 numbers, so both sides start from identical inputs.

Transition convention (the Gaussian autoregressive form of the target chain, paper Sec. 3.1):
state ``y_k`` (k = 0..T) moves to ``y_{k+1} ~ N(a[k]*y_k + c[k]*D(y_k, k), sigma[k]^2 I)`` where
``D`` is the target network's prediction.  The paper's Euler-Maruyama chain is ``a=1, c=gamma,
D=b^q``; unadjusted Langevin is ``a=1, c=-gamma, D=grad E, sigma=sqrt(2 gamma)``; the DDPM
ancestral sampler with an x0-predicting denoiser has the textbook posterior-mean coefficients.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np


def _f32(x) -> np.ndarray:
    """Round to fp32 and return the fp64 image (exactly representable on both sides)."""
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


# --------------------------------------------------------------------------------------
# Schedules
# --------------------------------------------------------------------------------------
@dataclass
class Schedule:
    """Coefficient arrays of the chain, indexed by the chain step k = 0..T-1.

    ``alpha_bar_state[k]`` (k = 0..T) is the signal level of state ``y_k`` for diffusion
    schedules (``x_t = sqrt(ab) x0 + sqrt(1-ab) eps``); it is what a denoiser conditions on.
    For Langevin it is None.
    """
    name: str
    T: int
    a: np.ndarray
    c: np.ndarray
    sigma: np.ndarray
    alpha_bar_state: Optional[np.ndarray] = None


def _ddpm_from_betas(name: str, betas: np.ndarray) -> Schedule:
    """DDPM ancestral sampler, x0-prediction.  Chain step k <-> diffusion index t = T - k.

    q(x_{t-1} | x_t, x0) has mean
        sqrt(ab_{t-1}) beta_t / (1 - ab_t) * x0 + sqrt(alpha_t) (1 - ab_{t-1}) / (1 - ab_t) * x_t
    (Ho et al. 2020, eq. 7); the sampler plugs the prediction D in for x0.  The step variance is
    beta_t at every step including the last, so sigma > 0 everywhere as the accept test needs.
    """
    T = betas.shape[0]
    alphas = 1.0 - betas
    ab = np.concatenate([[1.0], np.cumprod(alphas)])          # ab[t], t = 0..T
    t = T - np.arange(T)                                       # t for chain step k
    beta_t, alpha_t = betas[t - 1], alphas[t - 1]
    a = np.sqrt(alpha_t) * (1.0 - ab[t - 1]) / (1.0 - ab[t])
    c = np.sqrt(ab[t - 1]) * beta_t / (1.0 - ab[t])
    sigma = np.sqrt(beta_t)
    ab_state = ab[T - np.arange(T + 1)]                        # state k has level ab_{T-k}
    return Schedule(name, T, _f32(a), _f32(c), _f32(sigma), _f32(ab_state))


def linear_beta_schedule(T: int, beta_lo: float = 1e-4, beta_hi: float = 0.02) -> Schedule:
    betas = np.linspace(beta_lo, beta_hi, T, dtype=np.float64) if T > 1 else np.array([beta_hi])
    return _ddpm_from_betas(f"linear{T}", betas)


def cosine_schedule(T: int, s: float = 0.008, beta_max: float = 0.999) -> Schedule:
    """Discrete cosine schedule (Nichol & Dhariwal 2021): ab_t = f(t)/f(0), betas clipped."""
    tt = np.arange(T + 1, dtype=np.float64) / T
    f = np.cos((tt + s) / (1.0 + s) * np.pi / 2.0) ** 2
    ab = f / f[0]
    betas = np.minimum(1.0 - ab[1:] / ab[:-1], beta_max)
    return _ddpm_from_betas(f"cosine{T}", betas)


def em_schedule(T: int, gamma: float, sigma: float, name: str = "em") -> Schedule:
    """Constant-coefficient Euler-Maruyama chain y + gamma*b(y) + sigma*z (paper eq. for m^q)."""
    one = np.ones(T)
    return Schedule(name, T, _f32(one), _f32(gamma * one), _f32(sigma * one), None)


def langevin_schedule(T: int, gamma: float) -> Schedule:
    """ULA: x - gamma grad E(x) + sqrt(2 gamma) w  (paper Sec. 5)."""
    one = np.ones(T)
    g32 = float(np.float32(gamma))
    return Schedule(f"ula{T}", T, _f32(one), _f32(-g32 * one),
                    _f32(np.sqrt(2.0 * g32) * one), None)


# --------------------------------------------------------------------------------------
# Data-distribution / network parameters
# --------------------------------------------------------------------------------------
@dataclass
class GMMParams:
    means: np.ndarray      # [M, d]
    stds: np.ndarray       # [M, d]  per-component diagonal std
    logw: np.ndarray       # [M]     log mixture weights (normalised)


@dataclass
class LowRankGaussianParams:
    mu: np.ndarray         # [d]
    U: np.ndarray          # [d, r]   covariance = U U^T + s2 I
    s2: float


@dataclass
class Phi4Params:
    L: int                 # grid side, d = L*L sites numbered row by row, periodic
    beta: float            # coupling


@dataclass
class MLPParams:
    """x0-predicting MLP: [x ; temb(k)] -> H -> H -> d, SiLU, weights stored as bf16 bit patterns."""
    d: int
    H: int
    E: int                              # time-embedding width
    W1: np.ndarray                      # uint16 [d+E, H]  bf16 bits (row = input feature)
    b1: np.ndarray                      # fp32-valued [H]
    W2: np.ndarray                      # uint16 [H, H]
    b2: np.ndarray
    W3: np.ndarray                      # uint16 [H, d]
    b3: np.ndarray


def bf16_round_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern (uint16), round-to-nearest-even. Data preparation only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def ring_gmm(M: int = 8, radius: float = 4.0, std: float = 0.3) -> GMMParams:
    ang = 2.0 * np.pi * np.arange(M) / M
    means = np.stack([radius * np.cos(ang), radius * np.sin(ang)], axis=1)
    return GMMParams(_f32(means), _f32(np.full((M, 2), std)), _f32(np.full(M, -np.log(M))))


def random_gmm(rng: np.random.Generator, M: int, d: int, mean_std: float,
               std_lo: float, std_hi: float, uniform_weights: bool = True) -> GMMParams:
    means = rng.normal(0.0, mean_std, size=(M, d))
    if std_lo == std_hi:
        stds = np.full((M, d), std_lo)
    else:
        stds = rng.uniform(std_lo, std_hi, size=(M, d))   # i.i.d. per coordinate: "diagonal"
    if uniform_weights:
        w = np.full(M, 1.0 / M)
    else:
        w = rng.dirichlet(np.full(M, 2.0))
    return GMMParams(_f32(means), _f32(stds), _f32(np.log(w)))


def lowrank_gaussian(rng: np.random.Generator, d: int, r: int, s2: float = 0.01,
                     mu_std: float = 0.5) -> LowRankGaussianParams:
    U = rng.normal(0.0, 1.0 / np.sqrt(r), size=(d, r))      # entries ~ N(0, 1/r)
    mu = rng.normal(0.0, mu_std, size=d)                   # mu ~ N(0, mu_std^2 I)
    return LowRankGaussianParams(_f32(mu), _f32(U), float(np.float32(s2)))


def random_mlp(rng: np.random.Generator, d: int, H: int, E: int = 256) -> MLPParams:
    """Kaiming-normal weights (std sqrt(2/fan_in)), uniform(+-1/sqrt(fan_in)) biases."""
    def layer(fan_in, fan_out):
        W = rng.standard_normal((fan_in, fan_out), dtype=np.float32) * np.float32(np.sqrt(2.0 / fan_in))
        b = rng.uniform(-1.0, 1.0, size=fan_out) / np.sqrt(fan_in)
        return bf16_round_bits(W), _f32(b)
    W1, b1 = layer(d + E, H)
    W2, b2 = layer(H, H)
    W3, b3 = layer(H, d)
    return MLPParams(d, H, E, W1, b1, W2, b2, W3, b3)


# --------------------------------------------------------------------------------------
# The five configurations
# --------------------------------------------------------------------------------------
@dataclass
class Config:
    name: str
    kind: str                 # "gmm" | "lowrank" | "mlp" | "langevin"
    B: int                    # chains
    d: int                    # state dimension
    K: int                    # draft window length (the paper's L)
    T: int                    # chain length (the paper's K)
    seed: int
    schedule: Schedule
    params: object
    gamma: float = 0.0        # Langevin step size
    stands_in_for: str = ""
    extra: Dict[str, object] = field(default_factory=dict)


def draft_params(cfg: "Config"):
    """Parameters of a cheaper draft model of the same family as the target (input preparation
    for the independent drafter of Sec. 3.1; no claim of a trained fit):
    gmm      every second component of the mixture, weights renormalised;
    lowrank  the first quarter of the columns of U, the dropped variance spread over s2;
    mlp      a separately drawn MLP of a quarter of the hidden width."""
    p = cfg.params
    if cfg.kind == "gmm":
        idx = np.arange(0, p.means.shape[0], 2)
        logw = p.logw[idx] - np.log(np.sum(np.exp(p.logw[idx])))
        return GMMParams(p.means[idx].copy(), p.stds[idx].copy(), _f32(logw))
    if cfg.kind == "lowrank":
        r = max(1, p.U.shape[1] // 4)
        dropped = float(np.sum(p.U[:, r:] ** 2)) / p.U.shape[0]
        return LowRankGaussianParams(p.mu.copy(), p.U[:, :r].copy(), float(_f32(p.s2 + dropped)))
    if cfg.kind == "mlp":
        rng = np.random.default_rng([cfg.seed, 977, p.H])
        return random_mlp(rng, p.d, max(256, p.H // 4), p.E)
    raise ValueError(f"no draft model for workload kind {cfg.kind!r}")


def make_config(name: str, *, B: Optional[int] = None, d: Optional[int] = None,
                K: Optional[int] = None, T: Optional[int] = None, seed: int = 0,
                H: Optional[int] = None, r: Optional[int] = None,
                M: Optional[int] = None) -> Config:
    """Build configuration ``c1`` .. ``c5``; keyword overrides give the scaled-down test cases.

    The parameter stream is numpy's PCG64 seeded with (seed, config number); the chains' own
    noise comes from the counter-based generator each side implements for itself.
    """
    name = name.lower()
    idx = {"c1": 1, "c2": 2, "c3": 3, "c4": 4, "c5": 5, "phi4": 6}[name]
    rng = np.random.default_rng([seed, idx])
    if name == "c1":
        T = T or 100
        return Config(name, "gmm", B or 64, 2, K or 4, T, seed, linear_beta_schedule(T),
                      ring_gmm(M or 8), stands_in_for="low-dimensional mixture study (d=2)")
    if name == "c2":
        T = T or 200
        d = d or 64
        return Config(name, "gmm", B or 4096, d, K or 8, T, seed, cosine_schedule(T),
                      random_gmm(rng, M or 32, d, 3.0, 0.2, 1.0),
                      stands_in_for="low-dimensional mixture study (d<=64)")
    if name == "c3":
        T = T or 250
        d = d or 3072
        return Config(name, "lowrank", B or 2048, d, K or 10, T, seed, cosine_schedule(T),
                      lowrank_gaussian(rng, d, r or 256),
                      stands_in_for="32x32x3 image chain (shape only)")
    if name == "c4":
        T = T or 500
        d = d or 12288
        return Config(name, "mlp", B or 512, d, K or 16, T, seed, linear_beta_schedule(T),
                      random_mlp(rng, d, H or 4096),
                      stands_in_for="64x64x3 image chain, 500 steps (shape only)")
    if name == "c5":
        T = T or 2000
        d = d or 1000
        gamma = 1e-2
        return Config(name, "langevin", B or 16384, d, K or 16, T, seed,
                      langevin_schedule(T, gamma),
                      random_gmm(rng, M or 16, d, 2.0, 1.0, 1.0), gamma=float(np.float32(gamma)),
                      stands_in_for="speculative unadjusted Langevin appendix")
    if name == "phi4":
        # the phi^4 lattice of the Langevin appendix: 8 x 8 grid, beta = 100, step 1e-3, window 20
        # (d = L*L; "M" is unused).  The appendix runs 1e5 iterations; the benchmark runs T of them.
        T = T or 2000
        L = int(round(np.sqrt(d))) if d else 8
        gamma = 1e-3
        return Config(name, "phi4", B or 16384, L * L, K or 20, T, seed, langevin_schedule(T, gamma),
                      Phi4Params(L, float(np.float32(100.0))), gamma=float(np.float32(gamma)),
                      stands_in_for="phi^4 lattice Langevin experiment (energy is analytic; no data)")
    raise ValueError(name)
