"""Pins for the oracle's window loop and whole sampler (no GPU).

The sampler has no printed trajectory to compare with ("parity unpinned" for exact values of a
path); what the paper and the mathematics fix is pinned instead: exactness in law, the
degenerate draft == target case, the advance law under i.i.d. acceptance, and the closed-form
marginals of an affine-Gaussian chain.
"""
import numpy as np
import pytest
from scipy import stats

import workloads as W
from oracle import philox
from oracle import speculative as S
from oracle.denoisers import GMMDenoiser, LowRankDenoiser


def _ring(T=25, beta_hi=0.35):
    sched = W._ddpm_from_betas("test", np.linspace(1e-3, beta_hi, T))
    return sched, GMMDenoiser(W.ring_gmm(), sched.alpha_bar_state)


def test_draft_equal_to_target_reproduces_sequential_chain_bit_for_bit():
    sched, den = _ring(T=23)
    B, K = 50, 5
    seq = S.sequential_chain(sched, den, B, 2, seed=9)
    out, st = S.sample(sched, den, B, 2, K, seed=9, drafter="independent", D_draft=den)
    assert np.array_equal(out, seq)
    assert st.rejections == 0
    assert st.windows == -(-23 // K) and st.chain_windows == B * st.windows
    assert st.steps == B * 23


def test_frozen_window_structure():
    sched, den = _ring(T=10)
    rng = np.random.default_rng(0)
    B, K, d = 200, 4, 2
    y = rng.standard_normal((B, d)) * 2
    n = rng.integers(0, 10, size=B)
    ids = np.arange(B, dtype=np.int64) + 1000
    res, Ytil, Dq, D0, krow, calls = S.window(sched, den, y, n, ids, K, seed=3)
    Kt = np.minimum(K, 10 - n)
    assert calls == 2
    # first position: draft mean == target mean, always accepted -> advance >= min(2, Kt)
    assert np.all(res.logratio[:, 0] == 0)
    assert np.all(res.adv >= np.minimum(2, Kt)) and np.all(res.adv <= Kt) and np.all(res.adv >= 1)
    assert np.all(res.rejected <= (res.adv >= 2))
    # the target is evaluated at states n .. n+Kt-1: krow names rows 0..Kt-2 of the drafts
    for b in range(B):
        expect = [n[b] + j + 1 if j + 1 <= Kt[b] - 1 else -1 for j in range(K)]
        assert krow[b].tolist() == expect
        assert np.all(Ytil[b, Kt[b]:] == 0) and np.all(res.logratio[b, Kt[b]:] == 0)
    # drafts follow the frozen recursion with the keyed noise of the state they produce
    b = int(np.argmax(Kt))
    z2 = philox.normals(3, ids[b:b + 1], n[b:b + 1] + 2, d)[0]
    k = n[b] + 1
    assert np.allclose(Ytil[b, 1], sched.a[k] * Ytil[b, 0] + sched.c[k] * D0[b] + sched.sigma[k] * z2,
                       atol=1e-14)
    # accepted prefix is the draft itself; a full acceptance returns the last draft
    full = ~res.rejected
    assert np.array_equal(res.y_out[full], Ytil[full, res.adv[full] - 1])
    # rejected: the kept state differs from the draft, and first failing position is adv
    rej = res.rejected
    assert rej.any() and full.any()
    for b in np.nonzero(rej)[0]:
        j = res.adv[b]
        assert res.logu[b, j - 1] > min(0.0, res.logratio[b, j - 1])
        assert np.all(res.logu[b, :j - 1] <= np.minimum(0.0, res.logratio[b, :j - 1]))
        assert not np.array_equal(res.y_out[b], Ytil[b, j - 1])
    # verify() on the stored arrays reproduces the window
    again = S.verify(sched, y, n, ids, Ytil, Dq, K, 3, D0=D0)
    assert np.array_equal(again.y_out, res.y_out) and np.array_equal(again.adv, res.adv)
    # explicit-mean mode with the frozen means gives the same decisions and states
    mp = np.zeros_like(Ytil)
    for j in range(1, K + 1):
        act = j <= Kt
        k = np.minimum(n + j - 1, 9)
        prev = y if j == 1 else Ytil[:, j - 2]
        mp[act, j - 1] = (sched.a[k, None] * prev + sched.c[k, None] * D0)[act]
    expl = S.verify(sched, y, n, ids, Ytil, Dq, K, 3, mp=mp)
    assert np.array_equal(expl.adv, res.adv) and np.allclose(expl.y_out, res.y_out, atol=1e-12)


def test_results_do_not_depend_on_batch_composition():
    sched, den = _ring(T=12)
    full, _ = S.sample(sched, den, 64, 2, 4, seed=5)
    sub_ids = np.array([3, 40, 17, 63])
    sub, _ = S.sample(sched, den, 0, 2, 4, seed=5, chain_ids=sub_ids)
    assert np.array_equal(sub, full[sub_ids])


def test_advance_bookkeeping():
    out = np.zeros((6, 2))
    y_out = np.arange(8.0).reshape(4, 2)
    y, n, ids = S.advance(10, y_out, np.array([2, 1, 3, 4]), np.array([8, 3, 6, 6]),
                          np.array([5, 0, 2, 4]), out)
    assert n.tolist() == [4, 9] and ids.tolist() == [0, 2]
    assert np.array_equal(y, y_out[[1, 2]])
    assert np.array_equal(out[5], y_out[0]) and np.array_equal(out[4], y_out[3])
    assert np.all(out[[0, 1, 2, 3]] == 0)


def test_advance_law_under_iid_acceptance():
    """Draft mean = target mean + delta*sigma*e  =>  every position is accepted independently
    with alpha = 2 Phi(-delta/2) (time-to-first-rejection product form), so the advance is a
    truncated geometric with mean sum_{i<K} alpha^i  (the sum in the complexity analysis; the
    closed form printed after it does not equal that sum -- at K = 1 it gives 1-a+a^2, not 1)."""
    d, K, T = 3, 6, 6
    gamma, sigma, delta = 0.05, 0.3, 0.9
    sched = W.em_schedule(T, gamma, sigma)
    e = np.array([1.0, 2.0, -2.0]) / 3.0
    target = lambda x, k: -x
    draft = lambda x, k: -x + (delta * sched.sigma[k] / sched.c[k])[:, None] * e
    B = 200_000
    rng = np.random.default_rng(0)
    y = rng.standard_normal((B, d))
    res, *_ = S.window(sched, target, y, np.zeros(B, dtype=np.int64), np.arange(B), K, seed=1,
                       drafter="independent", D_draft=draft)
    alpha = 2 * stats.norm.cdf(-delta / 2)
    pmf = np.array([alpha ** (j - 1) * (1 - alpha) for j in range(1, K)] + [alpha ** (K - 1)])
    counts = np.bincount(res.adv, minlength=K + 1)[1:]
    assert stats.chisquare(counts, pmf * B).pvalue > 1e-3
    mean = (1 - alpha ** K) / (1 - alpha)
    assert abs(res.adv.mean() - mean) < 4 * res.adv.std() / np.sqrt(B)
    assert abs(pmf @ np.arange(1, K + 1) - mean) < 1e-12
    # all K drafts accepted <=> no rejection flag; a rejection at the last position also advances K
    assert np.array_equal(res.rejected, ~np.all(res.logu <= np.minimum(0, res.logratio), axis=1))


def test_gaussian_data_closed_form_chain_marginal():
    """With the linear (Gaussian-data) denoiser the target chain is affine-Gaussian:
    mean_{k+1} = A_k mean_k + c_k h_k,  P_{k+1} = A_k P_k A_k^T + sigma_k^2 I,  A_k = a_k I + c_k G_k.
    An exact sampler must reproduce that marginal at k = T."""
    rng = np.random.default_rng(3)
    d, r, T, K = 5, 2, 16, 4
    p = W.lowrank_gaussian(rng, d, r, s2=0.05)
    sched = W.cosine_schedule(T)
    den = LowRankDenoiser(p, sched.alpha_bar_state)
    mean, P = np.zeros(d), np.eye(d)
    for k in range(T):
        G, h = den.affine_map(k)
        A = sched.a[k] * np.eye(d) + sched.c[k] * G
        mean = A @ mean + sched.c[k] * h
        P = A @ P @ A.T + sched.sigma[k] ** 2 * np.eye(d)
    B = 60_000
    out, st = S.sample(sched, den, B, d, K, seed=4)
    assert st.rejections > 0.1 * st.chain_windows                # the reflection branch is exercised
    L = np.linalg.cholesky(P)
    white = np.linalg.solve(L, (out - mean).T).T
    assert np.all(np.abs(white.mean(0)) < 4.5 / np.sqrt(B))
    assert np.max(np.abs(np.cov(white.T) - np.eye(d))) < 6 * np.sqrt(2 / B)
    for i in range(d):
        assert stats.kstest(white[:, i], "norm").pvalue > 1e-4
    # the sequential chain passes the same check (the recursion itself is right)
    seq = S.sequential_chain(sched, den, 20_000, d, seed=5)
    ws = np.linalg.solve(L, (seq - mean).T).T
    assert np.max(np.abs(np.cov(ws.T) - np.eye(d))) < 6 * np.sqrt(2 / 20_000)


def test_speculative_sampler_is_exact_in_law_and_the_incorrect_one_is_not():
    """d = 2 ring mixture, large steps so that about half of the windows reject.  Speculative
    samples (own seed) against plain sequential samples (another seed): two-sample KS on both
    coordinates, radius and angle, at the end and at an intermediate step.  The paper's
    INCORRECT mechanism must fail the same test."""
    B, K = 40_000, 6
    radius = lambda v: np.linalg.norm(v, axis=1)
    feats = (lambda v: v[:, 0], lambda v: v[:, 1], radius, lambda v: np.arctan2(v[:, 1], v[:, 0]))
    for T_stop in (25, 14):
        sched, den = _ring()
        if T_stop < 25:                                          # the chain up to step T_stop
            sched = W.Schedule("prefix", T_stop, sched.a[:T_stop], sched.c[:T_stop],
                               sched.sigma[:T_stop], sched.alpha_bar_state[:T_stop + 1])
        seq = S.sequential_chain(sched, den, B, 2, seed=101)
        spec, st = S.sample(sched, den, B, 2, K, seed=202)
        assert 0.3 < st.rejections / st.chain_windows < 0.8
        for f in feats:
            assert stats.ks_2samp(f(spec), f(seq)).pvalue > 1e-4
    bad, _ = S.sample(sched, den, B, 2, K, seed=303, mechanism="incorrect")
    assert stats.ks_2samp(radius(bad), radius(seq)).pvalue < 1e-12


def test_efficient_frozen_reduces_to_the_sequential_chain_when_nothing_is_rejected():
    """A prediction that does not depend on the state makes draft and target means coincide for any
    frozen vector, so nothing is rejected: the efficient variant must then return the sequential
    chain bit for bit with one target call per window plus the initialisation."""
    sched = W.cosine_schedule(19)
    const = lambda v, k: np.full_like(np.asarray(v, dtype=np.float64), 0.7)
    B, K = 30, 4
    seq = S.sequential_chain(sched, const, B, 3, seed=2)
    out, st = S.sample_efficient(sched, const, B, 3, K, seed=2)
    assert np.array_equal(out, seq)
    assert st.rejections == 0 and st.windows == -(-19 // K)
    assert st.target_calls == st.windows + 1


def test_efficient_frozen_window_structure():
    sched, den = _ring(T=12)
    rng = np.random.default_rng(1)
    B, K, d = 300, 4, 2
    y = rng.standard_normal((B, d)) * 2
    n = rng.integers(0, 12, size=B)
    ids = np.arange(B, dtype=np.int64) + 50
    Kt = np.minimum(K, 12 - n)
    # (a) frozen vector = the exact prediction at y_n: identical to the plain frozen window
    D0 = den(y, n)
    res, Ytil, Dq_ext, krow_ext, Dnext = S.window_efficient(sched, den, y, n, ids, D0, K, seed=5)
    ref, Ytil_ref, Dq_ref, _, _, _ = S.window(sched, den, y, n, ids, K, seed=5)
    assert np.array_equal(Ytil, Ytil_ref) and np.array_equal(res.adv, ref.adv)
    assert np.allclose(res.y_out, ref.y_out, atol=1e-13) and np.allclose(res.logratio, ref.logratio, atol=1e-12)
    # rows evaluated: the start state and every draft whose step index is below T
    for b in range(B):
        expect = [n[b]] + [n[b] + j if (j <= Kt[b] and n[b] + j < 12) else -1 for j in range(1, K + 1)]
        assert krow_ext[b].tolist() == expect
    # the carried prediction is the target's prediction at the draft state of position adv
    b = int(np.nonzero(ref.rejected & (n + ref.adv < 12))[0][0])
    j = ref.adv[b]
    assert np.allclose(Dnext[b], den(Ytil[b:b + 1, j - 1], n[b:b + 1] + j)[0], atol=1e-14)
    full = np.nonzero(~ref.rejected & (n + ref.adv < 12))[0]
    assert np.allclose(Dnext[full], den(res.y_out[full], n[full] + res.adv[full]), atol=1e-13)
    # (b) a stale frozen vector: the first position is no longer accepted for certain
    stale = D0 + 0.8 * rng.standard_normal((B, d))
    res2, *_ = S.window_efficient(sched, den, y, n, ids, stale, K, seed=5)
    assert np.all(res2.logratio[:, 0] != 0) and (res2.adv == 1).sum() > 0 and np.all(res2.adv <= Kt)


def test_efficient_frozen_sampler_is_exact_in_law():
    """Any draft mean gives an exact sampler; with the carried-over prediction the final states must
    still pass the two-sample tests against the sequential chain."""
    B, K = 40_000, 6
    sched, den = _ring()
    seq = S.sequential_chain(sched, den, B, 2, seed=111)
    spec, st = S.sample_efficient(sched, den, B, 2, K, seed=222)
    assert st.steps == B * sched.T and st.target_calls == st.windows + 1
    assert 0.3 < st.rejections / st.chain_windows < 0.95
    radius = lambda v: np.linalg.norm(v, axis=1)
    for f in (lambda v: v[:, 0], lambda v: v[:, 1], radius, lambda v: np.arctan2(v[:, 1], v[:, 0])):
        assert stats.ks_2samp(f(spec), f(seq)).pvalue > 1e-4


def test_efficient_frozen_last_accepted_rule_structure():
    """The alternative carry rule of the same appendix paragraph: after a rejection the next window freezes the
    prediction at the last state the chain kept, with that state's step index.  Rebuilt here from the states
    themselves (a direct call of the denoiser, not an index into the window's prediction array), so a wrong row or
    a wrong step index fails; chains without a rejection carry the same vector under both rules."""
    sched, den = _ring(T=12)
    rng = np.random.default_rng(4)
    B, K, d = 400, 4, 2
    y = rng.standard_normal((B, d)) * 2
    n = rng.integers(0, 12, size=B)
    ids = np.arange(B, dtype=np.int64) + 9
    stale = den(y, n) + 0.5 * rng.standard_normal((B, d))
    res_a, Ytil_a, _, _, next_a = S.window_efficient(sched, den, y, n, ids, stale, K, seed=8, carry="draft")
    res_b, Ytil_b, _, _, next_b = S.window_efficient(sched, den, y, n, ids, stale, K, seed=8, carry="last_accepted")
    # the rule changes what is carried, nothing inside the window
    assert np.array_equal(Ytil_a, Ytil_b) and np.array_equal(res_a.adv, res_b.adv)
    assert np.array_equal(res_a.y_out, res_b.y_out)
    rej, keep = res_b.rejected, ~res_b.rejected
    assert rej.sum() > 50 and (rej & (res_b.adv == 1)).sum() > 5 and (rej & (res_b.adv > 1)).sum() > 5
    assert np.array_equal(next_a[keep], next_b[keep])
    for b in np.nonzero(rej)[0]:
        j = int(res_b.adv[b])                                        # rejected position: state j-1 is the last kept one
        state = y[b] if j == 1 else Ytil_b[b, j - 2]
        want = den(state[None], np.array([n[b] + j - 1]))[0]
        assert np.allclose(next_b[b], want, atol=1e-14)
        assert not np.allclose(next_b[b], next_a[b], atol=1e-9) or n[b] + j >= 12
    with pytest.raises(ValueError):
        S.window_efficient(sched, den, y, n, ids, stale, K, seed=8, carry="previous")


def test_efficient_frozen_last_accepted_sampler_is_exact_in_law():
    B, K = 40_000, 6
    sched, den = _ring()
    seq = S.sequential_chain(sched, den, B, 2, seed=111)
    spec, st = S.sample_efficient(sched, den, B, 2, K, seed=333, carry="last_accepted")
    assert st.steps == B * sched.T and st.target_calls == st.windows + 1
    assert 0.3 < st.rejections / st.chain_windows < 0.95
    radius = lambda v: np.linalg.norm(v, axis=1)
    for f in (lambda v: v[:, 0], lambda v: v[:, 1], radius, lambda v: np.arctan2(v[:, 1], v[:, 0])):
        assert stats.ks_2samp(f(spec), f(seq)).pvalue > 1e-4
    const = lambda v, k: np.full_like(np.asarray(v, dtype=np.float64), 0.7)
    sched19 = W.cosine_schedule(19)
    out, st2 = S.sample_efficient(sched19, const, 30, 3, 4, seed=2, carry="last_accepted")
    assert np.array_equal(out, S.sequential_chain(sched19, const, 30, 3, seed=2)) and st2.rejections == 0
