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


# --------------------------------------------------------------------------------------------------
# Free-running samplers: a flipped accept decision moves the whole rest of a chain, so a chain that ends
# away from the oracle's is only acceptable if its FIRST differing window is a near tie.  The oracle carries
# its states in fp64, the GPU rounds them to fp32 at every window, so after some windows the two sides test
# slightly different inputs: the replay below follows one chain window by window on both sides, each from
# its own state, and shows that
#   * on the GPU's own input the oracle takes the GPU's decision (identical-input parity, 1e-6 tie band), and
#   * where the two paths first part, the oracle's decision margin on its own path is no larger than the
#     shift of the log-ratio that the difference of the two inputs explains (+ 1e-6).
# --------------------------------------------------------------------------------------------------
def gpu_chain_stepper(cfg, drafter="frozen", draft_params=None, tau=None, seed=None):
    """One chain on the GPU, window by window: returns (start(cid) -> state, step(state, n, cid) -> (state', adv)).
    A state is a tuple of fp64 images of the fp32 arrays the library holds for the chain: (y,) or, for the
    efficient frozen drafter, (y, carried prediction)."""
    from paper_2501_05370_amd.runner import make_sampler
    smp = make_sampler(cfg, B=1, out_rows=1, seed=seed, drafter=drafter, draft_params=draft_params)
    if tau is not None:
        smp.ctx.sd_set_temperature(tau)
    b = smp.buf
    eff = drafter.startswith("efficient_frozen")

    def start(cid):
        smp.start(torch.tensor([cid], dtype=torch.int64, device="cuda"))
        st = (host(b.y)[0].astype(np.float64),)
        return st + ((host(b.Dfz)[0].astype(np.float64),) if eff else ())

    def step(state, n, cid):
        b.y[:1].copy_(f32(state[0][None])); b.n[:1].fill_(int(n)); b.chain_id[:1].fill_(int(cid))
        if eff:
            b.Dfz[:1].copy_(f32(state[1][None]))
        smp.window(1)
        adv = int(host(b.adv)[0])
        out = (host(b.y_out)[0].astype(np.float64),)
        if eff:
            out = out + (host(b.Dq_ext)[0, adv].astype(np.float64),)
        return out, adv

    return start, step


def first_divergence_is_a_near_tie(gpu_step, oracle_step, state_g, state_o, cid, T, slack=1e-6):
    """Replay of one chain (see above).  oracle_step(state, n, cid) -> (state', adv, logratio [K], logu [K]).
    Returns (window, margin, shift) of the first window whose outcomes differ, None if there is none."""
    n, w = 0, 0
    while n < T:
        out_o, adv_o, lr_o, lu_o = oracle_step(state_o, n, cid)
        out_g, adv_g = gpu_step(state_g, n, cid)
        _, adv_og, lr_og, lu_og = oracle_step(state_g, n, cid)
        if adv_g != adv_og:
            j = min(adv_g, adv_og) - 1
            assert abs(lu_og[j] - min(0.0, lr_og[j])) < slack, \
                f"chain {cid}, window {w}: on identical inputs the GPU advances {adv_g}, the oracle {adv_og}"
        if adv_g != adv_o:
            j = min(adv_g, adv_o) - 1
            margin = abs(lu_o[j] - min(0.0, lr_o[j]))
            shift = abs(lr_o[j] - lr_og[j])
            assert margin <= shift + slack, \
                f"chain {cid}, window {w}: paths part at a margin of {margin:.3e}, the inputs explain {shift:.3e}"
            return w, margin, shift
        state_o, state_g, n, w = out_o, out_g, n + adv_o, w + 1
    return None


def explain_divergent_chains(err, chain_ids, gpu_start, gpu_step, oracle_start, oracle_step, T, label, limit=1e-3):
    """For every chain whose final state is off the oracle's (err > limit): its first differing window must be a
    near tie in the sense above.  Returns the number of such chains."""
    off = np.nonzero(np.asarray(err) > limit)[0]
    for i in off:
        cid = int(chain_ids[i])
        found = first_divergence_is_a_near_tie(gpu_step, oracle_step, gpu_start(cid), oracle_start(cid), cid, T)
        assert found is not None, f"{label}: chain {cid} ends off the oracle's path although every window agrees"
        print(f"[{label}] chain {cid} leaves the oracle's path in window {found[0]}: margin {found[1]:.2e}, "
              f"log-ratio shift from the fp32 states {found[2]:.2e}")
    return off.size


def ula_oracle_stepper(grad, cfg, seed, tau=1.0):
    """(start, step) of the oracle's Langevin chain in the form first_divergence_is_a_near_tie takes."""
    from oracle import langevin as L
    from oracle import philox

    def step(state, n, cid):
        xo, adv, _, lr, lu = L.ula_window(grad, state[0][None], np.array([n]), np.array([cid], dtype=np.int64), cfg.K, cfg.T,
                                          cfg.gamma, seed=seed, tau=tau)
        return (xo[0],), int(adv[0]), lr[0], lu[0]

    start = lambda cid: (philox.initial_state(seed, np.array([cid], dtype=np.int64), cfg.d)[0],)
    return start, step


def check_advance_on_matching_chains(smp, T, n, ids, res, gpu_adv, tol, carry_ref=None):
    """sd_advance on the whole batch the sampler just verified, checked on the chains whose window decisions equal
    the oracle's (`res`): those that go on sit among the survivors in their old order with the oracle's new step
    and state (and carried prediction, `carry_ref` [B,d]), those that finish have their state in out[chain id].
    With every decision equal this is the whole bookkeeping, survivor count included."""
    from oracle import speculative as S
    B = len(n)
    b = smp.buf
    same = np.asarray(gpu_adv) == res.adv
    d = res.y_out.shape[1]
    out_ref = np.zeros((int(max(ids)) + 1, d))
    y_ref, n_ref, id_ref = S.advance(T, res.y_out[same], res.adv[same], n[same], ids[same], out_ref)
    smp.advance(B)
    Ba = int(host(b.B_active)[0])
    gid, gn, gy = host(b.chain_id)[:Ba], host(b.n)[:Ba], host(b.y)[:Ba]
    pick = np.isin(gid, ids[same])
    assert np.array_equal(gid[pick], id_ref) and np.array_equal(gn[pick], n_ref)
    assert rel_err(gy[pick], y_ref) < tol
    if carry_ref is not None:
        keep = same & (n + res.adv < T)
        assert rel_err(host(b.Dfz)[:Ba][pick], carry_ref[keep]) < tol
    done = same & (n + res.adv >= T)
    if done.any():
        assert rel_err(host(b.out)[ids[done]], res.y_out[done]) < tol
    if same.all():
        assert Ba == n_ref.size
    return int(same.sum())
