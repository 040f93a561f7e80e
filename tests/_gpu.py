"""Helpers shared by the GPU parity tests (marshalling between numpy oracle data and tensors)."""
import numpy as np
import torch


def dev(a, dtype):
    return torch.as_tensor(np.ascontiguousarray(a), dtype=dtype).cuda().contiguous()


def f32(a):
    return dev(np.asarray(a, dtype=np.float32), torch.float32)


def host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


def as_f32_f64(a):
    """fp64 image of the fp32 rounding of `a` (what both sides are given)."""
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def rel_err(got, want):
    """max |got-want| / max(1, row scale) -- row-wise relative error with an absolute floor of 1."""
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    scale = np.maximum(1.0, np.max(np.abs(want), axis=-1, keepdims=True)) if want.ndim > 1 else np.maximum(1.0, np.abs(want))
    return float(np.max(np.abs(got - want) / scale))


def make_context(sched, d, K, seed, mode=None, tau=None):
    from paper_2501_05370_amd.binding import Context
    ctx = Context(sched.a, sched.c, sched.sigma, d, K)
    ctx.sd_set_seed(seed)
    if mode is not None:
        ctx.sd_set_draft_mode(mode)
    if tau is not None:
        ctx.sd_set_temperature(tau)
    return ctx


def decisions_match(adv_gpu, res, band=1e-6):
    """Accepted-prefix lengths must be bit-exact except where the oracle's own margin
    |log u - min(0, log ratio)| at the deciding position is inside `band`.
    Returns (number of mismatches, number of those that are near ties)."""
    adv_gpu = np.asarray(adv_gpu)
    bad = np.nonzero(adv_gpu != res.adv)[0]
    near = 0
    for b in bad:
        j = min(adv_gpu[b], res.adv[b]) - 1          # first position where the two disagree
        margin = abs(res.logu[b, j] - min(0.0, res.logratio[b, j]))
        near += margin < band
    return bad.size, near
