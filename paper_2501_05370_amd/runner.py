"""Glue from a ``workloads.Config`` to the library objects that run it (no arithmetic)."""
from __future__ import annotations

import torch

from .binding import Context, Denoiser
from .sampler import DiffusionSampler, EfficientFrozenSampler, IndependentDrafterSampler, LangevinSampler, Phi4LangevinSampler


def make_context(cfg, seed=None) -> Context:
    s = cfg.schedule
    ctx = Context(s.a, s.c, s.sigma, cfg.d, cfg.K)
    ctx.sd_set_seed(cfg.seed if seed is None else seed)
    return ctx


def make_denoiser(cfg, max_rows: int, params=None) -> Denoiser:
    p, s = (cfg.params if params is None else params), cfg.schedule
    if cfg.kind == "gmm":
        return Denoiser.sdden_gmm_create(p.means, p.stds, p.logw, s.alpha_bar_state)
    if cfg.kind == "lowrank":
        den = Denoiser.sdden_lowrank_create(p.mu, p.U, p.s2, s.alpha_bar_state)
        den.sdden_reserve(max_rows)
        return den
    if cfg.kind == "mlp":
        return Denoiser.sdden_mlp_create(p, cfg.T, max_rows)
    raise ValueError(f"no denoiser for workload kind {cfg.kind!r}")


def make_sampler(cfg, B=None, out_rows=None, seed=None, drafter: str = "frozen", draft_params=None):
    """A sampler for up to B chains of configuration ``cfg`` on the current device.  ``drafter`` is
    "frozen" (default) or "independent" with the draft model's parameters in ``draft_params``."""
    B = cfg.B if B is None else B
    ctx = make_context(cfg, seed)
    if cfg.kind == "phi4":
        return Phi4LangevinSampler(ctx, cfg.params.L, cfg.params.beta, cfg.gamma, B, out_rows)
    if drafter == "independent":
        if cfg.kind == "langevin" or draft_params is None:
            raise ValueError("the independent drafter needs a diffusion workload and draft_params")
        den = make_denoiser(cfg, B * cfg.K)
        draft = make_denoiser(cfg, B, draft_params)
        return IndependentDrafterSampler(ctx, den, draft, B, out_rows)
    if drafter in ("efficient_frozen", "efficient_frozen_last_accepted"):
        if cfg.kind == "langevin":
            raise ValueError("the efficient frozen drafter needs a diffusion workload")
        carry = "last_accepted" if drafter.endswith("last_accepted") else "draft"
        return EfficientFrozenSampler(ctx, make_denoiser(cfg, B * (cfg.K + 1)), B, out_rows, carry=carry)
    if drafter != "frozen":
        raise ValueError(drafter)
    if cfg.kind == "langevin":
        p = cfg.params
        dev = lambda a: torch.as_tensor(a, dtype=torch.float32).cuda().contiguous()
        return LangevinSampler(ctx, dev(p.means), dev(p.logw), float(p.stds[0, 0]), cfg.gamma, B, out_rows)
    den = make_denoiser(cfg, B * cfg.K)
    return DiffusionSampler(ctx, den, B, out_rows)
