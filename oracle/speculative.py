"""ORACLE (test infrastructure only) -- speculative sampling for diffusion chains, in fp64.

A plain, slow CPU statement of what the library's hot path computes, written from the paper:

* ``reflection_rejection``  the rejection mechanism for two Gaussians with the same covariance
                            (Alg. "REJECTION via reflection maximal coupling", Sec. 3.3), with
                            the optional temperature of App. "Influence of the temperature".
* ``draft_frozen`` / ``draft_independent``  the draft rollouts of Sec. 3.1 (frozen target draft,
                            independent draft).
* ``verify``                the accept / first-reject / reflect loop of the detailed algorithm
                            (App. "Detailed implementation of speculative sampling").
* ``advance``               the step index moves to where the window stopped (last line of the while-loop
                            body), plus the batch bookkeeping the paper leaves implicit.
* ``window`` / ``sample``   one pass of the while-loop body of Alg. "Speculative Sampling for
                            DDM", and the whole loop.
* ``sequential_chain``      the plain (non-speculative) target chain, eq. for q(y_k | y_{k-1}).

The method does not reproduce the sequential chain's path; it produces another path with
exactly the same law.  There is therefore no "plain definition of the result" to write out:
this file follows the algorithm's steps in the paper's order, vectorised over independent
chains only.  Notation: T = chain length (the paper's K), K = window (the paper's L),
Kt = min(K, T - n) (the paper's L-tilde), j = 1..Kt the position in the window, k = n + j - 1
the chain step whose transition is drafted/tested at position j.

Conventions fixed where the paper is silent (each also listed in the design document):
accept iff ``log u <= min(0, log-ratio / tau)`` with u in (0,1); ``||Delta|| = 0`` accepts and
never reflects; under the frozen drafter the position j = 1 has draft mean == target mean by
definition; on full acceptance n advances by Kt, on a rejection at position j by j (the
reflected state is kept); noise and uniforms are keyed by (seed, chain id, absolute state
index), never by window.

Pinned by tests/test_oracle_*.py: total-variation acceptance probability and the paper's two
worked Gaussian pairs, output law N(m^q, sigma^2 I), reflection invariants, log-ratio against
naive log-densities, draft == target reproducing the sequential chain bit for bit,
truncated-geometric advance law, closed-form Gaussian chain marginals, two-sample tests against
the sequential chain, and the paper's INCORRECT mechanism failing those same tests.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Optional

import numpy as np

from . import philox

Denoiser = Callable[[np.ndarray, np.ndarray], np.ndarray]


# --------------------------------------------------------------------------------------
# Rejection mechanism
# --------------------------------------------------------------------------------------
def reflection_rejection(mp, mq, sigma, ytil, u, tau: float = 1.0):
    """(Y, accept, log-ratio) for p = N(mp, sigma^2 I), q = N(mq, sigma^2 I), draft ytil ~ p.

    Delta = (mp - mq)/sigma, Z = (ytil - mp)/sigma,
    ratio = N(Z + Delta; 0, tau I) / N(Z; 0, tau I)  =>  log ratio = (-Z.Delta - |Delta|^2/2)/tau,
    accept iff u <= min(1, ratio); on reject Y = mq + sigma (I - 2 e e^T) Z, e = Delta/|Delta|.
    Shapes: mp, mq, ytil [..., d]; sigma, u [...].
    """
    mp, mq, ytil = (np.asarray(v, dtype=np.float64) for v in (mp, mq, ytil))
    sig = np.asarray(sigma, dtype=np.float64)[..., None]
    Delta = (mp - mq) / sig
    Z = (ytil - mp) / sig
    zd = np.sum(Z * Delta, axis=-1)
    dd = np.sum(Delta * Delta, axis=-1)
    logratio = (-zd - 0.5 * dd) / tau
    accept = (dd == 0.0) | (np.log(u) <= np.minimum(0.0, logratio))
    with np.errstate(divide="ignore", invalid="ignore"):
        coef = np.where(dd > 0.0, zd / dd, 0.0)               # (e.Z)/|Delta|
    reflected = mq + sig * (Z - 2.0 * coef[..., None] * Delta)
    Y = np.where(accept[..., None], ytil, reflected)
    return Y, accept, logratio


def incorrect_rejection(mp, mq, sigma, ytil, u, fresh_noise):
    """The paper's INCORRECT mechanism (App. "The need for adjusted rejection sampling"):
    same accept test, but a rejected draft is replaced by an independent draw from q.
    Exists only so that the statistical tests can be shown to detect a wrong sampler."""
    _, accept, logratio = reflection_rejection(mp, mq, sigma, ytil, u)
    fresh = np.asarray(mq) + np.asarray(sigma)[..., None] * fresh_noise
    return np.where(accept[..., None], ytil, fresh), accept, logratio


# --------------------------------------------------------------------------------------
# Draft rollouts
# --------------------------------------------------------------------------------------
def _krow(n: np.ndarray, Kt: np.ndarray, K: int) -> np.ndarray:
    """Chain step at which the target must be evaluated on drafted row j (= state n+j+1), or -1.
    The algorithm evaluates the target at states n .. n+Kt-1 only; state n is the window start
    (its prediction is D0), and the last drafted state n+Kt is not evaluated."""
    j = np.arange(K)[None, :]
    return np.where(j + 1 <= Kt[:, None] - 1, n[:, None] + j + 1, -1).astype(np.int32)


def draft_frozen(sched, y, n, chain_id, D0, K: int, seed: int):
    """Frozen target draft: m^p_k = a_k y~_k + c_k D0 with D0 = D(y_n, n) for the whole window
    (eq. "frozen draft model"; for a = 1 this is y~_k + gamma b^q_{t_n}(y_n) verbatim).

    Returns Ytil [B,K,d] with Ytil[:, j-1] = y~_{n+j} (zeros past the end of the chain) and
    krow [B,K]."""
    y = np.asarray(y, dtype=np.float64)
    D0 = np.asarray(D0, dtype=np.float64)
    n = np.asarray(n)
    B, d = y.shape
    Kt = np.minimum(K, sched.T - n)
    Ytil = np.zeros((B, K, d))
    prev = y.copy()
    for j in range(1, K + 1):
        act = np.nonzero(j <= Kt)[0]
        if act.size == 0:
            break
        k = n[act] + j - 1
        z = philox.normals(seed, chain_id[act], k + 1, d)
        nxt = sched.a[k, None] * prev[act] + sched.c[k, None] * D0[act] + sched.sigma[k, None] * z
        Ytil[act, j - 1] = nxt
        prev[act] = nxt
    return Ytil, _krow(n, Kt, K)


def draft_independent(sched, D_draft: Denoiser, y, n, chain_id, K: int, seed: int):
    """Independent draft model: m^p_k = a_k y~_k + c_k D^p(y~_k, k), a cheaper network called once
    per position (eq. "Euler-Maruyama backward draft").  Returns Ytil, mp [B,K,d], krow."""
    y = np.asarray(y, dtype=np.float64)
    n = np.asarray(n)
    B, d = y.shape
    Kt = np.minimum(K, sched.T - n)
    Ytil = np.zeros((B, K, d))
    mp = np.zeros((B, K, d))
    prev = y.copy()
    for j in range(1, K + 1):
        act = np.nonzero(j <= Kt)[0]
        if act.size == 0:
            break
        k = n[act] + j - 1
        m = sched.a[k, None] * prev[act] + sched.c[k, None] * D_draft(prev[act], k)
        z = philox.normals(seed, chain_id[act], k + 1, d)
        nxt = m + sched.sigma[k, None] * z
        mp[act, j - 1] = m
        Ytil[act, j - 1] = nxt
        prev[act] = nxt
    return Ytil, mp, _krow(n, Kt, K)


# --------------------------------------------------------------------------------------
# Verification: accept test, first rejection, reflection
# --------------------------------------------------------------------------------------
@dataclass
class VerifyResult:
    y_out: np.ndarray        # [B,d]  state the chain holds after the window
    adv: np.ndarray          # [B]    how many steps the chain advanced (1..Kt)
    rejected: np.ndarray     # [B]    whether a draft was rejected (then y_out is the reflection)
    logratio: np.ndarray     # [B,K]  log acceptance ratio at every position j <= Kt (0 elsewhere)
    logu: np.ndarray         # [B,K]  log of the uniform of every position j <= Kt (0 elsewhere)


def verify(sched, y, n, chain_id, Ytil, Dq, K: int, seed: int, *, D0=None, mp=None,
           tau: float = 1.0, mechanism: str = "reflection") -> VerifyResult:
    """For k = n+1 .. n+Kt in order: test y~_k, keep it on accept, else reflect and stop.

    ``Dq[:, j-1]`` is the target prediction D(y~_{n+j-1}, n+j-1) (row 0 belongs to the window
    start).  Exactly one of ``D0`` (frozen drafter: draft means are a y~ + c D0, and row 0 of Dq
    *is* D0) and ``mp`` (explicit draft means [B,K,d]) must be given.
    Log-ratios and log-uniforms are reported for all positions j <= Kt -- they are functions of
    the inputs -- although the algorithm only looks at them up to the first rejection.
    """
    assert (D0 is None) != (mp is None)
    y = np.asarray(y, dtype=np.float64)
    Ytil = np.asarray(Ytil, dtype=np.float64)
    Dq = np.asarray(Dq, dtype=np.float64)
    n = np.asarray(n)
    B, d = y.shape
    Kt = np.minimum(K, sched.T - n)
    logratio = np.zeros((B, K))
    logu = np.zeros((B, K))
    y_out = np.zeros((B, d))
    adv = np.zeros(B, dtype=np.int32)
    rejected = np.zeros(B, dtype=bool)
    running = np.ones(B, dtype=bool)               # chains still inside their for-loop
    for j in range(1, K + 1):
        act = np.nonzero(j <= Kt)[0]
        if act.size == 0:
            break
        k = n[act] + j - 1
        prev = y[act] if j == 1 else Ytil[act, j - 2]
        ytil = Ytil[act, j - 1]
        a, c, sig = sched.a[k, None], sched.c[k, None], sched.sigma[k]
        if D0 is not None:
            m_p = a * prev + c * np.asarray(D0, dtype=np.float64)[act]
            Dq_j = np.asarray(D0, dtype=np.float64)[act] if j == 1 else Dq[act, j - 1]
        else:
            m_p = np.asarray(mp, dtype=np.float64)[act, j - 1]
            Dq_j = Dq[act, j - 1]
        m_q = a * prev + c * Dq_j
        u = philox.uniforms(seed, chain_id[act], k + 1)
        if mechanism == "reflection":
            Y, acc, lr = reflection_rejection(m_p, m_q, sig, ytil, u, tau)
        elif mechanism == "incorrect":
            fresh = philox.normals(seed, chain_id[act], k + 1, d, stream=3)
            Y, acc, lr = incorrect_rejection(m_p, m_q, sig, ytil, u, fresh)
        else:
            raise ValueError(mechanism)
        logratio[act, j - 1] = lr
        logu[act, j - 1] = np.log(u)
        live = running[act]                         # not rejected earlier in this window
        upd = act[live]
        y_out[upd] = Y[live]
        adv[upd] = j
        rej_now = act[live & ~acc]
        rejected[rej_now] = True
        running[rej_now] = False                    # "Exit For Loop"
    return VerifyResult(y_out, adv, rejected, logratio, logu)


# --------------------------------------------------------------------------------------
# Bookkeeping: the step index moves to where the window stopped; finished chains leave the batch
# --------------------------------------------------------------------------------------
def advance(T: int, y_out, adv, n, chain_id, out):
    """n += adv; chains that reached T write their state to out[chain_id] and leave; the others
    keep their relative order.  Returns (y, n, chain_id) of the remaining chains."""
    n_new = np.asarray(n) + np.asarray(adv)
    done = n_new >= T
    out[np.asarray(chain_id)[done]] = np.asarray(y_out)[done]
    keep = ~done
    return np.asarray(y_out)[keep], n_new[keep], np.asarray(chain_id)[keep]


# --------------------------------------------------------------------------------------
# One window and the whole sampler
# --------------------------------------------------------------------------------------
def target_predictions(sched, D: Denoiser, Ytil, krow, D0) -> np.ndarray:
    """The target's predictions at the window start and at every drafted state but the last, all of which
    the algorithm obtains in one parallel evaluation (Alg. "Speculative Sampling for DDM", the parallel
    step): Dq [B,K,d], row 0 = D0, row j = D(Ytil[:, j-1], krow[:, j-1]) where krow >= 0."""
    B, K, d = Ytil.shape
    Dq = np.zeros((B, K, d))
    Dq[:, 0] = D0
    b_idx, j_idx = np.nonzero(krow[:, :K - 1] >= 0)             # drafted rows to evaluate
    if b_idx.size:
        Dq[b_idx, j_idx + 1] = D(Ytil[b_idx, j_idx], krow[b_idx, j_idx])
    return Dq


def window(sched, D: Denoiser, y, n, chain_id, K: int, seed: int, *, drafter: str = "frozen",
           D_draft: Optional[Denoiser] = None, tau: float = 1.0,
           mechanism: str = "reflection"):
    """One pass of the while-loop body.  Returns (VerifyResult, Ytil, Dq, D0, krow, target_calls)."""
    n = np.asarray(n)
    D0 = D(y, n)                                     # one target query at the window start
    if drafter == "frozen":
        Ytil, krow = draft_frozen(sched, y, n, chain_id, D0, K, seed)
        mp = None
    elif drafter == "independent":
        Ytil, mp, krow = draft_independent(sched, D_draft, y, n, chain_id, K, seed)
    else:
        raise ValueError(drafter)
    Dq = target_predictions(sched, D, Ytil, krow, D0)
    calls = 1 + int(np.any(krow >= 0))
    res = verify(sched, y, n, chain_id, Ytil, Dq, K, seed, D0=D0 if mp is None else None,
                 mp=mp, tau=tau, mechanism=mechanism)
    return res, Ytil, Dq, D0, krow, calls


@dataclass
class SampleStats:
    windows: int = 0                # passes of the while-loop over the (shrinking) batch
    chain_windows: int = 0          # sum over passes of the number of chains in the batch
    steps: int = 0                  # sum of advances = B * T at the end
    rejections: int = 0
    target_calls: int = 0           # batched target calls (the paper's NFE definition)
    target_rows: int = 0            # rows evaluated by the target

    @property
    def mean_advance(self) -> float:
        return self.steps / max(1, self.chain_windows)


def sample(sched, D: Denoiser, B: int, d: int, K: int, seed: int, *, drafter: str = "frozen",
           D_draft: Optional[Denoiser] = None, tau: float = 1.0, mechanism: str = "reflection",
           chain_ids: Optional[np.ndarray] = None):
    """Alg. "Speculative Sampling for DDM" for independent chains; returns (Y_T, stats), Y_T in
    the order of ``chain_ids`` (default 0..B-1).

    Chains advance by different amounts, so each carries its own n; finished chains leave the
    batch (``advance``)."""
    ids0 = np.arange(B, dtype=np.int64) if chain_ids is None else np.asarray(chain_ids, dtype=np.int64)
    ids = ids0.copy()
    y = philox.initial_state(seed, ids, d)
    n = np.zeros(ids.shape[0], dtype=np.int64)
    out = np.zeros((int(ids0.max()) + 1, d))
    st = SampleStats()
    while n.size:
        res, _, _, _, krow, calls = window(sched, D, y, n, ids, K, seed, drafter=drafter,
                                           D_draft=D_draft, tau=tau, mechanism=mechanism)
        st.windows += 1
        st.chain_windows += n.size
        st.steps += int(res.adv.sum())
        st.rejections += int(res.rejected.sum())
        st.target_calls += calls
        st.target_rows += n.size + int((krow >= 0).sum())
        y, n, ids = advance(sched.T, res.y_out, res.adv, n, ids, out)
    return out[ids0], st


# --------------------------------------------------------------------------------------
# Efficient frozen drafter (App. "Extending the draft models", paragraph on the efficient frozen
# draft strategy): the draft mean freezes the target's prediction at the DRAFT state of the
# window's first position, D(y~_n, n), which the previous window's verification computed, instead
# of a fresh D(y_n, n).  A window then needs one batched target call, on y_n and all Kt drafts.
# The paragraph's last sentence names an alternative for the case y~_n != y_n (the previous window
# ended with a rejection): freeze the prediction at the last ACCEPTED state, D(y_{n-1}, n-1), which
# that call computed as well.  carry = "draft" is the first rule, "last_accepted" the second.
# --------------------------------------------------------------------------------------
CARRY_RULES = ("draft", "last_accepted")


def window_efficient(sched, D: Denoiser, y, n, chain_id, Dfz, K: int, seed: int, *, tau: float = 1.0,
                     carry: str = "draft"):
    """One window with the carried-over frozen prediction ``Dfz`` [B,d].

    Returns (VerifyResult, Ytil, Dq_ext [B,K+1,d], krow_ext [B,K+1], Dfz_next [B,d]):
    Dq_ext[:, j] = D(state j of the window, n+j) for j = 0 (y_n itself) .. Kt (rows whose step
    index would be T are not evaluated and stay zero).  Dfz_next, the vector the next window
    freezes: carry "draft": Dq_ext[b, adv[b]], the prediction at the draft state of the position
    the next window starts from (the rejected draft, or the last accepted one when nothing was
    rejected); carry "last_accepted": after a rejection Dq_ext[b, adv[b]-1] instead, the
    prediction at the last state the chain kept unchanged (the window's own start state when the
    first draft was rejected), at that state's step index."""
    if carry not in CARRY_RULES:
        raise ValueError(f"carry must be one of {CARRY_RULES}")
    y = np.asarray(y, dtype=np.float64)
    n = np.asarray(n)
    B, d = y.shape
    Kt = np.minimum(K, sched.T - n)
    Ytil, _ = draft_frozen(sched, y, n, chain_id, Dfz, K, seed)
    # draft means, explicitly: m^p_j = a_k prev + c_k Dfz
    mp = np.zeros((B, K, d))
    for j in range(1, K + 1):
        act = np.nonzero(j <= Kt)[0]
        if act.size == 0:
            break
        k = n[act] + j - 1
        prev = y[act] if j == 1 else Ytil[act, j - 2]
        mp[act, j - 1] = sched.a[k, None] * prev + sched.c[k, None] * np.asarray(Dfz, dtype=np.float64)[act]
    # the one batched target call: the true start state and every draft (also the last one)
    krow_ext = np.full((B, K + 1), -1, dtype=np.int64)
    krow_ext[:, 0] = n
    for j in range(1, K + 1):
        ok = (j <= Kt) & (n + j < sched.T)
        krow_ext[ok, j] = n[ok] + j
    X_ext = np.concatenate([y[:, None, :], Ytil], axis=1)
    Dq_ext = np.zeros((B, K + 1, d))
    b_idx, j_idx = np.nonzero(krow_ext >= 0)
    Dq_ext[b_idx, j_idx] = D(X_ext[b_idx, j_idx], krow_ext[b_idx, j_idx])
    res = verify(sched, y, n, chain_id, Ytil, Dq_ext[:, :K], K, seed, mp=mp, tau=tau)
    row = res.adv.copy()
    if carry == "last_accepted":
        row = row - res.rejected.astype(row.dtype)
    Dfz_next = Dq_ext[np.arange(B), row]
    return res, Ytil, Dq_ext, krow_ext, Dfz_next


def sample_efficient(sched, D: Denoiser, B: int, d: int, K: int, seed: int, *, tau: float = 1.0,
                     chain_ids: Optional[np.ndarray] = None, carry: str = "draft"):
    """The whole sampler with the efficient frozen drafter; initialised with D(y_0, 0).
    Returns (Y_T, stats): stats.target_calls = 1 + number of windows."""
    ids0 = np.arange(B, dtype=np.int64) if chain_ids is None else np.asarray(chain_ids, dtype=np.int64)
    ids = ids0.copy()
    y = philox.initial_state(seed, ids, d)
    n = np.zeros(ids.shape[0], dtype=np.int64)
    out = np.zeros((int(ids0.max()) + 1, d))
    st = SampleStats()
    Dfz = D(y, n)
    st.target_calls, st.target_rows = 1, n.size
    while n.size:
        res, _, _, krow_ext, Dfz_next = window_efficient(sched, D, y, n, ids, Dfz, K, seed, tau=tau, carry=carry)
        st.windows += 1
        st.chain_windows += n.size
        st.steps += int(res.adv.sum())
        st.rejections += int(res.rejected.sum())
        st.target_calls += 1
        st.target_rows += int((krow_ext >= 0).sum())
        keep = n + res.adv < sched.T
        y, n, ids = advance(sched.T, res.y_out, res.adv, n, ids, out)
        Dfz = Dfz_next[keep]
    return out[ids0], st


def sequential_chain(sched, D: Denoiser, B: int, d: int, seed: int,
                     chain_ids: Optional[np.ndarray] = None, upto: Optional[int] = None):
    """The target chain itself: y_{k+1} = a_k y_k + c_k D(y_k, k) + sigma_k z_{k+1}, with the
    same keyed noise the speculative sampler's drafts use."""
    ids = np.arange(B, dtype=np.int64) if chain_ids is None else np.asarray(chain_ids, dtype=np.int64)
    y = philox.initial_state(seed, ids, d)
    for k in range(sched.T if upto is None else upto):
        kk = np.full(ids.shape[0], k, dtype=np.int64)
        z = philox.normals(seed, ids, kk + 1, d)
        y = sched.a[k] * y + sched.c[k] * D(y, kk) + sched.sigma[k] * z
    return y
