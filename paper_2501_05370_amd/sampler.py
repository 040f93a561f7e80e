"""Host-side window loop over the C entry points (buffers + call order only; no arithmetic).

``DiffusionSampler`` runs Alg. "Speculative Sampling for DDM" for a batch of chains: per window
``sdden_eval`` (window-start prediction) -> ``sd_draft`` -> ``sdden_eval`` (all drafted states in
one batched call) -> ``sd_verify`` -> ``sd_advance``.  ``LangevinSampler`` loops
``sd_langevin_window`` + ``sd_advance``.  Tensors are allocated once with PyTorch and reused.
"""
from __future__ import annotations

from collections import defaultdict
from contextlib import contextmanager
from typing import Optional

import torch

from .binding import Context, Denoiser


class StageTimer:
    """HIP-event timing of chosen stages on the stream the kernels are launched on (torch's
    current stream, whose handle the binding passes to the library)."""

    def __init__(self, stages=None):
        self.stages = None if stages is None else set(stages)
        self._open = defaultdict(list)

    @contextmanager
    def stage(self, name: str, chains: int):
        if self.stages is not None and name not in self.stages:
            yield
            return
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        yield
        e1.record()
        self._open[name].append((e0, e1, chains))

    def collect(self):
        """{stage: (total ms, launches, total chains)}; resets."""
        torch.cuda.synchronize()
        res = {}
        for name, evs in self._open.items():
            res[name] = (sum(a.elapsed_time(b) for a, b, _ in evs), len(evs), sum(c for _, _, c in evs))
        self._open.clear()
        return res


class _NoTimer:
    @contextmanager
    def stage(self, name, chains):
        yield


class WindowBuffers:
    """Device buffers of one batch of at most B chains (layouts as in include/sd.h)."""

    def __init__(self, B: int, d: int, K: int, out_rows: Optional[int] = None, window: bool = True,
                 device="cuda"):
        f32 = dict(dtype=torch.float32, device=device)
        self.B, self.d, self.K = B, d, K
        self.y = torch.zeros(B, d, **f32)
        self.n = torch.zeros(B, dtype=torch.int32, device=device)
        self.chain_id = torch.zeros(B, dtype=torch.int64, device=device)
        if window:
            self.D0 = torch.zeros(B, d, **f32)
            self.Ytilde = torch.zeros(B, K, d, **f32)
            self.krow = torch.full((B, K), -1, dtype=torch.int32, device=device)
            self.Dq = torch.zeros(B, K, d, **f32)
        self.y_out = torch.zeros(B, d, **f32)
        self.adv = torch.zeros(B, dtype=torch.int32, device=device)
        self.rejected = torch.zeros(B, dtype=torch.uint8, device=device)
        self.out = torch.zeros(out_rows if out_rows is not None else B, d, **f32)
        self.B_active = torch.full((1,), B, dtype=torch.int32, device=device)
        self.counters = torch.zeros(5, dtype=torch.int64, device=device)


class _SamplerBase:
    timer = _NoTimer()

    def _setup(self, ctx: Context, B: int, out_rows, window: bool):
        self.ctx = ctx
        self.buf = WindowBuffers(B, ctx.d, ctx.K, out_rows, window)
        self.ws = torch.empty(max(8, ctx.sd_workspace_bytes(B)), dtype=torch.uint8, device="cuda")
        ctx.sd_set_workspace(self.ws)

    def start(self, chain_ids: torch.Tensor, reset_counters: bool = True) -> int:
        b = self.buf
        B = chain_ids.numel()
        b.chain_id[:B].copy_(chain_ids)
        self.ctx.sd_init_state(B, b.chain_id, b.y, b.n)
        if reset_counters:
            b.counters.zero_()
        return B

    def advance(self, B: int):
        b = self.buf
        with self.timer.stage("advance", B):
            self.ctx.sd_advance(B, b.y_out, b.adv, b.rejected, b.y, b.n, b.chain_id, b.out, b.B_active,
                                b.counters)

    def run(self, chain_ids: torch.Tensor, reset_counters: bool = True, windows_per_sync: int = 1,
            graph: bool = False):
        """All chains to step T.  Returns (out tensor indexed by chain id, counters as a list
        [sum adv, chain-windows, rejections, windows, sum Kt]).

        ``windows_per_sync`` > 1 (or ``graph``) keeps the batch size on the device: the kernels read
        it from ``B_active`` (``sd_set_active_count``), the host launches that many windows with the
        last known bound before it reads the 4 bytes back, and windows launched after the last chain
        finished do nothing.  ``graph`` additionally captures window + advance for a bound in a HIP
        graph (through torch.cuda.CUDAGraph) and replays it: for workloads whose windows are a few
        tens of microseconds of kernels, launch cost is what is left.  Results do not depend on
        either option (noise is keyed by chain id and step, never by the launch)."""
        B = self.start(chain_ids, reset_counters)
        if windows_per_sync <= 1 and not graph:
            while B > 0:
                self.window(B)
                self.advance(B)
                B = int(self.buf.B_active.item())               # the one 4-byte readback per window
            return self.buf.out, self.buf.counters.tolist()
        if not isinstance(self.timer, _NoTimer):
            raise RuntimeError("stage timing records events per call: not available with windows_per_sync / graph")
        b = self.buf
        b.B_active.fill_(B)
        self._set_active(b.B_active)
        try:
            while B > 0:
                bound = self._bound(B)
                if graph:
                    g = self._graph(bound)
                    for _ in range(max(1, windows_per_sync)):
                        g.replay()
                else:
                    for _ in range(windows_per_sync):
                        self.window(bound)
                        self.advance(bound)
                B = int(b.B_active.item())
        finally:
            self._set_active(None)
        return b.out, b.counters.tolist()

    def _bound(self, B: int) -> int:
        """Launch bound for B remaining chains: B rounded up to 1/8 steps of the capacity, so that a
        handful of graphs serves a whole run."""
        step = max(1, self.buf.B // 8)
        return min(self.buf.B, -(-B // step) * step)

    def _set_active(self, count: Optional[torch.Tensor]):
        self._active = count
        self.ctx.sd_set_active_count(count)
        if count is None and getattr(self, "den", None) is not None:
            self.den.sdden_set_active_count(None, 1)
            if getattr(self, "draft_den", None) is not None:
                self.draft_den.sdden_set_active_count(None, 1)

    def _den_rows(self, den, rows_per_chain: int):
        """Before a denoiser call in device-count mode: rows beyond count * rows_per_chain are skipped."""
        if getattr(self, "_active", None) is not None:
            den.sdden_set_active_count(self._active, rows_per_chain)

    def _graph(self, bound: int):
        cache = self.__dict__.setdefault("_graphs", {})
        if bound not in cache:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                self.window(bound)
                self.advance(bound)
            cache[bound] = g
        return cache[bound]


class DiffusionSampler(_SamplerBase):
    def __init__(self, ctx: Context, den: Denoiser, B: int, out_rows: Optional[int] = None):
        self.den = den
        self._setup(ctx, B, out_rows, True)
        # a network with bf16 inputs gets the drafts as bf16 straight from the draft kernel
        self.mirror = (torch.zeros(B, ctx.K, ctx.d, dtype=torch.int16, device="cuda")
                       if getattr(den, "wants_bf16", False) else None)

    def window(self, B: int, diagnostics=None):
        """One pass of the while-loop body for the first B chains of the buffers."""
        b, ctx, den, d, K, t = self.buf, self.ctx, self.den, self.ctx.d, self.ctx.K, self.timer
        with t.stage("predict_start", B):
            self._den_rows(den, 1)
            den.sdden_eval(B, b.y, b.n, b.D0)                   # D0 = D(y_n, n)
        with t.stage("draft", B):
            ctx.sd_set_draft_mirror(self.mirror)
            ctx.sd_draft(B, b.y, b.n, b.chain_id, b.D0, b.Ytilde, b.krow)
            ctx.sd_set_draft_mirror(None)
        if K > 1:
            # row (b,j) of Ytilde feeds row (b,j+1) of Dq: same flat layout shifted by one row;
            # the last row of every chain is masked by krow, so the shifted write stays in bounds
            with t.stage("predict_drafts", B):
                self._den_rows(den, K)
                if self.mirror is not None:
                    den.sdden_eval_mirror(B * K, b.Ytilde.view(-1, d), self.mirror.view(-1, d), b.krow.view(-1),
                                          b.Dq.view(-1, d)[1:])
                else:
                    den.sdden_eval(B * K, b.Ytilde.view(-1, d), b.krow.view(-1), b.Dq.view(-1, d)[1:])
        lr, lu = diagnostics if diagnostics is not None else (None, None)
        with t.stage("verify", B):
            ctx.sd_verify(B, b.y, b.n, b.chain_id, b.D0, b.Dq, b.Ytilde, b.y_out, b.adv, b.rejected, lr, lu)


class IndependentDrafterSampler(_SamplerBase):
    """The same loop with the independent draft model of Sec. 3.1: a cheaper network ``draft_den`` is
    called once per window position (``sd_draft_step`` between the calls), then the target runs once
    on all drafted states and ``sd_verify`` works in EXPLICIT mode on the stored draft means."""

    def __init__(self, ctx: Context, den: Denoiser, draft_den: Denoiser, B: int, out_rows: Optional[int] = None):
        from .binding import SD_DRAFT_EXPLICIT
        self.den, self.draft_den = den, draft_den
        self._setup(ctx, B, out_rows, True)
        b, f32 = self.buf, dict(dtype=torch.float32, device="cuda")
        b.mp = torch.zeros(B, ctx.K, ctx.d, **f32)
        b.Dp = torch.zeros(B, ctx.d, **f32)
        b.cur = [torch.zeros(B, ctx.d, **f32), torch.zeros(B, ctx.d, **f32)]
        b.kcur = [torch.full((B,), -1, dtype=torch.int32, device="cuda") for _ in range(2)]
        ctx.sd_set_draft_mode(SD_DRAFT_EXPLICIT)
        ctx.sd_set_start_prediction(b.D0)

    def window(self, B: int, diagnostics=None):
        b, ctx, d, K, t = self.buf, self.ctx, self.ctx.d, self.ctx.K, self.timer
        with t.stage("predict_start", B):
            self._den_rows(self.den, 1)
            self.den.sdden_eval(B, b.y, b.n, b.D0)              # target at the window start
        prev, kprev = b.y, b.n
        with t.stage("draft", B):
            self._den_rows(self.draft_den, 1)
            for j in range(1, K + 1):
                self.draft_den.sdden_eval(B, prev, kprev, b.Dp)
                nxt, knext = b.cur[j & 1], b.kcur[j & 1]
                ctx.sd_draft_step(B, j, prev, b.n, b.chain_id, b.Dp, b.mp, b.Ytilde, b.krow, nxt, knext)
                prev, kprev = nxt, knext
        if K > 1:
            with t.stage("predict_drafts", B):
                self._den_rows(self.den, K)
                self.den.sdden_eval(B * K, b.Ytilde.view(-1, d), b.krow.view(-1), b.Dq.view(-1, d)[1:])
        lr, lu = diagnostics if diagnostics is not None else (None, None)
        with t.stage("verify", B):
            ctx.sd_verify(B, b.y, b.n, b.chain_id, b.mp, b.Dq, b.Ytilde, b.y_out, b.adv, b.rejected, lr, lu)


class EfficientFrozenSampler(_SamplerBase):
    """The efficient frozen drafter: the draft mean freezes the target's prediction at the previous
    window's draft state, carried through ``sd_advance``; one batched target call per window on the
    start state and all drafts (``sd_draft`` -> ``sdden_eval`` -> ``sd_verify`` -> ``sd_advance``).
    carry: "draft" (the prediction at the draft state of the position advanced to) or "last_accepted" (after a
    rejection, the prediction at the last state the chain kept): the two rules of ``sd_set_carry_rule``."""

    def __init__(self, ctx: Context, den: Denoiser, B: int, out_rows: Optional[int] = None, carry: str = "draft"):
        from .binding import SD_CARRY_DRAFT, SD_CARRY_LAST_ACCEPTED, SD_DRAFT_FROZEN_REUSED
        rules = {"draft": SD_CARRY_DRAFT, "last_accepted": SD_CARRY_LAST_ACCEPTED}
        if carry not in rules:
            raise ValueError(f"carry must be one of {sorted(rules)}")
        self.den = den
        self._setup(ctx, B, out_rows, False)
        b, K, d, f32 = self.buf, ctx.K, ctx.d, dict(dtype=torch.float32, device="cuda")
        b.Dfz = torch.zeros(B, d, **f32)
        b.X_ext = torch.zeros(B, K + 1, d, **f32)
        b.krow_ext = torch.full((B, K + 1), -1, dtype=torch.int32, device="cuda")
        b.Dq_ext = torch.zeros(B, K + 1, d, **f32)
        ctx.sd_set_draft_mode(SD_DRAFT_FROZEN_REUSED)
        ctx.sd_set_carry(b.Dq_ext, b.Dfz)
        ctx.sd_set_carry_rule(rules[carry])
        # bf16 image of the window rows for denoisers whose first GEMM reads bf16 (written by sd_draft)
        self.mirror = (torch.zeros(B, K + 1, d, dtype=torch.int16, device="cuda")
                       if getattr(den, "wants_bf16", False) else None)

    def start(self, chain_ids: torch.Tensor, reset_counters: bool = True) -> int:
        B = super().start(chain_ids, reset_counters)
        b = self.buf
        self.den.sdden_eval(B, b.y, b.n, b.Dfz)                 # initialisation: D(y_0, 0)
        return B

    def window(self, B: int, diagnostics=None):
        b, ctx, d, K, t = self.buf, self.ctx, self.ctx.d, self.ctx.K, self.timer
        with t.stage("draft", B):
            ctx.sd_set_draft_mirror(self.mirror)
            ctx.sd_draft(B, b.y, b.n, b.chain_id, b.Dfz, b.X_ext, b.krow_ext)
            ctx.sd_set_draft_mirror(None)
        with t.stage("predict_drafts", B):
            self._den_rows(self.den, K + 1)
            if self.mirror is not None:
                self.den.sdden_eval_mirror(B * (K + 1), b.X_ext.view(-1, d), self.mirror.view(-1, d),
                                           b.krow_ext.view(-1), b.Dq_ext.view(-1, d))
            else:
                self.den.sdden_eval(B * (K + 1), b.X_ext.view(-1, d), b.krow_ext.view(-1), b.Dq_ext.view(-1, d))
        lr, lu = diagnostics if diagnostics is not None else (None, None)
        with t.stage("verify", B):
            ctx.sd_verify(B, b.y, b.n, b.chain_id, b.Dfz, b.Dq_ext, b.X_ext, b.y_out, b.adv, b.rejected, lr, lu)


class LangevinSampler(_SamplerBase):
    def __init__(self, ctx: Context, means: torch.Tensor, logw: torch.Tensor, comp_std: float,
                 gamma: float, B: int, out_rows: Optional[int] = None):
        self.means, self.logw = means, logw
        self.comp_std, self.gamma, self.M = comp_std, gamma, means.shape[0]
        self._setup(ctx, B, out_rows, False)

    def window(self, B: int, logratio=None, logu=None):
        b = self.buf
        with self.timer.stage("langevin_window", B):
            self.ctx.sd_langevin_window(B, b.y, b.n, b.chain_id, self.means, self.logw, self.comp_std,
                                        self.M, self.gamma, b.y_out, b.adv, b.rejected, logratio, logu)


    def run_fused(self, chain_ids: torch.Tensor, reset_counters: bool = True):
        """All chains to step T in one launch (``sd_langevin_run``): same results as ``run``, bit for bit.
        Returns (final states in the order of chain_ids, counters)."""
        B = self.start(chain_ids, reset_counters)
        b = self.buf
        if B > 0:
            with self.timer.stage("langevin_run", B):
                self.ctx.sd_langevin_run(B, b.y, b.n, b.chain_id, self.means, self.logw, self.comp_std, self.M,
                                         self.gamma, max(2, self.ctx.T), b.y_out, b.n, b.counters)
        return b.y_out[:B], b.counters.tolist()


class Phi4LangevinSampler(_SamplerBase):
    """Speculative unadjusted Langevin on the phi^4 lattice energy: ``sd_langevin_window_phi4`` + ``sd_advance``."""

    def __init__(self, ctx: Context, L: int, beta: float, gamma: float, B: int, out_rows: Optional[int] = None):
        self.L, self.beta, self.gamma = L, beta, gamma
        self._setup(ctx, B, out_rows, False)

    def window(self, B: int, logratio=None, logu=None):
        b = self.buf
        with self.timer.stage("langevin_window", B):
            self.ctx.sd_langevin_window_phi4(B, b.y, b.n, b.chain_id, self.L, self.beta,
                                             self.gamma, b.y_out, b.adv, b.rejected, logratio, logu)

    def run_fused(self, chain_ids: torch.Tensor, reset_counters: bool = True):
        """All chains to step T in one launch (``sd_langevin_run_phi4``): same results as ``run``, bit for bit."""
        B = self.start(chain_ids, reset_counters)
        b = self.buf
        if B > 0:
            with self.timer.stage("langevin_run", B):
                self.ctx.sd_langevin_run_phi4(B, b.y, b.n, b.chain_id, self.L, self.beta, self.gamma,
                                              max(2, self.ctx.T), b.y_out, b.n, b.counters)
        return b.y_out[:B], b.counters.tolist()
