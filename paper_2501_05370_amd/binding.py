"""ctypes binding of libsd_mi355x.so -- argument marshalling only.

Every function here has the name of the C entry point it forwards to (``include/sd.h``,
``include/sdden.h``).  PyTorch is used for device memory and streams: tensors are checked for
device / dtype / contiguity and their raw pointers handed to the library.  There is no
fallback: if the shared library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_uint64, c_void_p
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsd_mi355x.so")

SD_DRAFT_FROZEN = 0
SD_DRAFT_EXPLICIT = 1
SD_DRAFT_FROZEN_REUSED = 2
SD_MAX_WINDOW = 64
SD_STATIC_MAX_CHAINS = 65536
SD_CARRY_DRAFT = 0
SD_CARRY_LAST_ACCEPTED = 1


class SDError(RuntimeError):
    pass


class _Schedule(ctypes.Structure):
    _fields_ = [("T", c_int32), ("a", POINTER(c_float)), ("c", POINTER(c_float)),
                ("sigma", POINTER(c_float))]


_SIGNATURES = {
    # sd.h
    "sd_create": (c_int, [POINTER(_Schedule), c_int32, c_int32, POINTER(c_void_p)]),
    "sd_destroy": (c_int, [c_void_p]),
    "sd_set_seed": (c_int, [c_void_p, c_uint64]),
    "sd_set_draft_mode": (c_int, [c_void_p, c_int]),
    "sd_set_temperature": (c_int, [c_void_p, c_float]),
    "sd_set_active_count": (c_int, [c_void_p, c_void_p]),
    "sd_set_verify_shape": (c_int, [c_void_p, c_int32]),
    "sd_workspace_bytes": (c_size_t, [c_void_p, c_int32]),
    "sd_set_workspace": (c_int, [c_void_p, c_void_p, c_size_t]),
    "sd_init_state": (c_int, [c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p]),
    "sd_draft": (c_int, [c_void_p, c_int32] + [c_void_p] * 7),
    "sd_draft_step": (c_int, [c_void_p, c_int32, c_int32] + [c_void_p] * 10),
    "sd_set_start_prediction": (c_int, [c_void_p, c_void_p]),
    "sd_set_carry": (c_int, [c_void_p, c_void_p, c_void_p]),
    "sd_set_carry_rule": (c_int, [c_void_p, c_int32]),
    "sd_set_draft_mirror": (c_int, [c_void_p, c_void_p]),
    "sdden_eval_mirror": (c_int, [c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "sd_verify": (c_int, [c_void_p, c_int32] + [c_void_p] * 12),
    "sd_advance": (c_int, [c_void_p, c_int32] + [c_void_p] * 10),
    "sd_advance_static": (c_int, [c_void_p, c_int32] + [c_void_p] * 10),
    "sd_langevin_window": (c_int, [c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                   c_float, c_int32, c_float] + [c_void_p] * 6),
    "sd_langevin_window_phi4": (c_int, [c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_int32, c_float, c_float]
                                + [c_void_p] * 6),
    "sd_langevin_run": (c_int, [c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                c_float, c_int32, c_float, c_int32] + [c_void_p] * 4),
    "sd_langevin_run_phi4": (c_int, [c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_int32, c_float, c_float,
                                     c_int32] + [c_void_p] * 4),
    "sd_last_error": (c_char_p, [c_void_p]),
    # sd_measure.h
    "sd_measure_stream": (c_int, [c_void_p, c_void_p, c_size_t, c_int32, c_int32, c_void_p]),
    "sd_measure_mfma": (c_int, [c_int32, c_int32, c_int32, c_void_p, POINTER(ctypes.c_double), c_void_p]),
    # sdden.h
    "sdden_gmm_create": (c_int, [c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_int32, c_void_p,
                                 POINTER(c_void_p)]),
    "sdden_lowrank_create": (c_int, [c_int32, c_int32, c_void_p, c_void_p, c_float, c_int32, c_void_p,
                                     POINTER(c_void_p)]),
    "sdden_mlp_create": (c_int, [c_int32, c_int32, c_int32] + [c_void_p] * 6 + [c_int32, c_int32,
                                                                               POINTER(c_void_p)]),
    "sdden_reserve": (c_int, [c_void_p, c_int32]),
    "sdden_eval": (c_int, [c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p]),
    "sdden_set_active_count": (c_int, [c_void_p, c_void_p, c_int32]),
    "sdden_profile": (c_int, [c_void_p, c_int32]),
    "sdden_profile_min_rows": (c_int, [c_void_p, c_int32]),
    "sdden_profile_collect": (c_int, [c_void_p, POINTER(ctypes.c_double), POINTER(c_int64)]),
    "sdden_mlp_select_gemm": (c_int, [c_void_p, c_int32]),
    "sdden_destroy": (c_int, [c_void_p]),
    "sdden_last_error": (c_char_p, [c_void_p]),
}

_lib = None


def exported_symbols():
    """Names the headers declare (and the binding expects)."""
    return sorted(_SIGNATURES)


def load_library(path: Optional[str] = None):
    """dlopen the HIP library; raises SDError when it has not been built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise SDError(f"{p} not found: build it first (python -m paper_2501_05370_amd.build). "
                      "There is no CPU fallback.")
    lib = ctypes.CDLL(p)
    for name, (res, args) in _SIGNATURES.items():
        fn = getattr(lib, name)            # AttributeError if a declared symbol is not exported
        fn.restype, fn.argtypes = res, args
    if path is None:
        _lib = lib
    return lib


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: Optional[torch.Tensor], dtype, name: str, allow_none: bool = False) -> Optional[int]:
    if t is None:
        if allow_none:
            return None
        raise SDError(f"{name}: tensor required")
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise SDError(f"{name}: need a contiguous {dtype} CUDA tensor, got {t.dtype} on {t.device}, "
                      f"contiguous={t.is_contiguous()}")
    return t.data_ptr()


def _host(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=dtype)


class Context:
    """Owns one ``sd_ctx``.  Methods are the C calls with tensors in place of pointers."""

    def __init__(self, a, c, sigma, d: int, K: int):
        self._lib = load_library()
        self._a, self._c, self._s = _host(a, np.float32), _host(c, np.float32), _host(sigma, np.float32)
        T = self._a.shape[0]
        if self._c.shape[0] != T or self._s.shape[0] != T:
            raise SDError("schedule arrays must have the same length")
        sch = _Schedule(T, self._a.ctypes.data_as(POINTER(c_float)), self._c.ctypes.data_as(POINTER(c_float)),
                        self._s.ctypes.data_as(POINTER(c_float)))
        h = c_void_p()
        rc = self._lib.sd_create(ctypes.byref(sch), d, K, ctypes.byref(h))
        if rc != 0:
            raise SDError(f"sd_create failed ({rc}): {self._lib.sd_last_error(None).decode()}")
        self._h = h
        self.T, self.d, self.K = T, d, K
        self._ws = None
        self._keep = []

    def close(self):
        if getattr(self, "_h", None):
            self._lib.sd_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int, what: str):
        if rc != 0:
            raise SDError(f"{what} failed ({rc}): {self._lib.sd_last_error(self._h).decode()}")

    # -- setters
    def sd_set_seed(self, seed: int):
        self._check(self._lib.sd_set_seed(self._h, seed), "sd_set_seed")

    def sd_set_draft_mode(self, mode: int):
        self._check(self._lib.sd_set_draft_mode(self._h, mode), "sd_set_draft_mode")

    def sd_set_temperature(self, tau: float):
        self._check(self._lib.sd_set_temperature(self._h, tau), "sd_set_temperature")

    def sd_set_verify_shape(self, shape: int):
        self._check(self._lib.sd_set_verify_shape(self._h, shape), "sd_set_verify_shape")

    def sd_set_active_count(self, count: Optional[torch.Tensor]):
        ptr = _dev(count, torch.int32, "count", allow_none=True)
        self._keep_count = count
        self._check(self._lib.sd_set_active_count(self._h, ptr), "sd_set_active_count")

    def sd_set_start_prediction(self, D_start: Optional[torch.Tensor]):
        ptr = _dev(D_start, torch.float32, "D_start", allow_none=True)
        self._keep_start = D_start
        self._check(self._lib.sd_set_start_prediction(self._h, ptr), "sd_set_start_prediction")

    def sd_set_draft_mirror(self, mirror: Optional[torch.Tensor]):
        """mirror: int16 tensor holding bf16 bit patterns, shape of Ytilde."""
        self._keep_mirror = mirror
        self._check(self._lib.sd_set_draft_mirror(self._h, _dev(mirror, torch.int16, "mirror", True)), "sd_set_draft_mirror")

    def sd_set_carry(self, Dq_ext: Optional[torch.Tensor], D_frozen: Optional[torch.Tensor]):
        self._keep_carry = (Dq_ext, D_frozen)
        self._check(self._lib.sd_set_carry(self._h, _dev(Dq_ext, torch.float32, "Dq_ext", True),
                                           _dev(D_frozen, torch.float32, "D_frozen", True)), "sd_set_carry")

    def sd_set_carry_rule(self, rule: int):
        self._check(self._lib.sd_set_carry_rule(self._h, int(rule)), "sd_set_carry_rule")

    def sd_workspace_bytes(self, Bmax: int) -> int:
        return int(self._lib.sd_workspace_bytes(self._h, Bmax))

    def sd_set_workspace(self, ws: Optional[torch.Tensor]):
        self._ws = ws
        if ws is None:
            self._check(self._lib.sd_set_workspace(self._h, None, 0), "sd_set_workspace")
        else:
            if not ws.is_cuda or not ws.is_contiguous():
                raise SDError("workspace: need a contiguous CUDA tensor")
            self._check(self._lib.sd_set_workspace(self._h, ws.data_ptr(), ws.numel() * ws.element_size()),
                        "sd_set_workspace")

    # -- window calls
    def sd_init_state(self, B, chain_id, y, n):
        self._check(self._lib.sd_init_state(self._h, B, _dev(chain_id, torch.int64, "chain_id"),
                                            _dev(y, torch.float32, "y"), _dev(n, torch.int32, "n"),
                                            _stream()), "sd_init_state")

    def sd_draft(self, B, y, n, chain_id, D0, Ytilde, krow):
        self._check(self._lib.sd_draft(self._h, B, _dev(y, torch.float32, "y"), _dev(n, torch.int32, "n"),
                                       _dev(chain_id, torch.int64, "chain_id"), _dev(D0, torch.float32, "D0"),
                                       _dev(Ytilde, torch.float32, "Ytilde"), _dev(krow, torch.int32, "krow"),
                                       _stream()), "sd_draft")

    def sd_draft_step(self, B, j, prev, n, chain_id, Dp, mp, Ytilde, krow, next=None, knext=None):
        self._check(self._lib.sd_draft_step(
            self._h, B, j, _dev(prev, torch.float32, "prev"), _dev(n, torch.int32, "n"),
            _dev(chain_id, torch.int64, "chain_id"), _dev(Dp, torch.float32, "Dp"),
            _dev(mp, torch.float32, "mp"), _dev(Ytilde, torch.float32, "Ytilde"),
            _dev(krow, torch.int32, "krow"), _dev(next, torch.float32, "next", True),
            _dev(knext, torch.int32, "knext", True), _stream()), "sd_draft_step")

    def sd_verify(self, B, y, n, chain_id, D0_or_mp, Dq, Ytilde, y_out, adv, rejected=None,
                  logratio=None, logu=None):
        self._check(self._lib.sd_verify(
            self._h, B, _dev(y, torch.float32, "y"), _dev(n, torch.int32, "n"),
            _dev(chain_id, torch.int64, "chain_id"), _dev(D0_or_mp, torch.float32, "D0_or_mp"),
            _dev(Dq, torch.float32, "Dq"), _dev(Ytilde, torch.float32, "Ytilde"),
            _dev(y_out, torch.float32, "y_out"), _dev(adv, torch.int32, "adv"),
            _dev(rejected, torch.uint8, "rejected", True), _dev(logratio, torch.float32, "logratio", True),
            _dev(logu, torch.float32, "logu", True), _stream()), "sd_verify")

    def sd_advance(self, B, y_out, adv, rejected, y, n, chain_id, out, B_active, counters=None):
        self._check(self._lib.sd_advance(
            self._h, B, _dev(y_out, torch.float32, "y_out"), _dev(adv, torch.int32, "adv"),
            _dev(rejected, torch.uint8, "rejected", True), _dev(y, torch.float32, "y"),
            _dev(n, torch.int32, "n"), _dev(chain_id, torch.int64, "chain_id"),
            _dev(out, torch.float32, "out"), _dev(B_active, torch.int32, "B_active"),
            _dev(counters, torch.int64, "counters", True), _stream()), "sd_advance")

    def sd_advance_static(self, B, y_out, adv, rejected, y, n, chain_id, out, B_active, counters=None):
        self._check(self._lib.sd_advance_static(
            self._h, B, _dev(y_out, torch.float32, "y_out"), _dev(adv, torch.int32, "adv"),
            _dev(rejected, torch.uint8, "rejected", True), _dev(y, torch.float32, "y"),
            _dev(n, torch.int32, "n"), _dev(chain_id, torch.int64, "chain_id"),
            _dev(out, torch.float32, "out"), _dev(B_active, torch.int32, "B_active"),
            _dev(counters, torch.int64, "counters", True), _stream()), "sd_advance_static")

    def sd_langevin_window(self, B, x, n, chain_id, means, logw, comp_std, M, gamma, x_out, adv,
                           rejected=None, logratio=None, logu=None):
        self._check(self._lib.sd_langevin_window(
            self._h, B, _dev(x, torch.float32, "x"), _dev(n, torch.int32, "n"),
            _dev(chain_id, torch.int64, "chain_id"), _dev(means, torch.float32, "means"),
            _dev(logw, torch.float32, "logw"), comp_std, M, gamma, _dev(x_out, torch.float32, "x_out"),
            _dev(adv, torch.int32, "adv"), _dev(rejected, torch.uint8, "rejected", True),
            _dev(logratio, torch.float32, "logratio", True), _dev(logu, torch.float32, "logu", True),
            _stream()), "sd_langevin_window")

    def sd_langevin_window_phi4(self, B, x, n, chain_id, L, beta, gamma, x_out, adv, rejected=None,
                                logratio=None, logu=None):
        self._check(self._lib.sd_langevin_window_phi4(
            self._h, B, _dev(x, torch.float32, "x"), _dev(n, torch.int32, "n"),
            _dev(chain_id, torch.int64, "chain_id"), L, beta, gamma, _dev(x_out, torch.float32, "x_out"),
            _dev(adv, torch.int32, "adv"), _dev(rejected, torch.uint8, "rejected", True),
            _dev(logratio, torch.float32, "logratio", True), _dev(logu, torch.float32, "logu", True),
            _stream()), "sd_langevin_window_phi4")

    def sd_langevin_run(self, B, x, n, chain_id, means, logw, comp_std, M, gamma, max_windows, x_out, n_out,
                        counters=None):
        self._check(self._lib.sd_langevin_run(
            self._h, B, _dev(x, torch.float32, "x"), _dev(n, torch.int32, "n"),
            _dev(chain_id, torch.int64, "chain_id"), _dev(means, torch.float32, "means"),
            _dev(logw, torch.float32, "logw"), comp_std, M, gamma, max_windows,
            _dev(x_out, torch.float32, "x_out"), _dev(n_out, torch.int32, "n_out"),
            _dev(counters, torch.int64, "counters", True), _stream()), "sd_langevin_run")

    def sd_langevin_run_phi4(self, B, x, n, chain_id, L, beta, gamma, max_windows, x_out, n_out, counters=None):
        self._check(self._lib.sd_langevin_run_phi4(
            self._h, B, _dev(x, torch.float32, "x"), _dev(n, torch.int32, "n"),
            _dev(chain_id, torch.int64, "chain_id"), L, beta, gamma, max_windows,
            _dev(x_out, torch.float32, "x_out"), _dev(n_out, torch.int32, "n_out"),
            _dev(counters, torch.int64, "counters", True), _stream()), "sd_langevin_run_phi4")


class Denoiser:
    """Owns one ``sdden``; built by the ``sdden_*_create`` class methods."""

    def __init__(self, handle, d: int):
        self._lib = load_library()
        self._h = handle
        self.d = d

    @staticmethod
    def _created(rc, h, what):
        lib = load_library()
        if rc != 0:
            raise SDError(f"{what} failed ({rc}): {lib.sdden_last_error(None).decode()}")
        return h

    @classmethod
    def sdden_gmm_create(cls, means, stds, logw, alpha_bar_state):
        lib = load_library()
        mu, sd, lw, ab = (_host(v, np.float32) for v in (means, stds, logw, alpha_bar_state))
        M, d = mu.shape
        h = c_void_p()
        rc = lib.sdden_gmm_create(M, d, mu.ctypes.data, sd.ctypes.data, lw.ctypes.data, ab.shape[0] - 1,
                                  ab.ctypes.data, ctypes.byref(h))
        return cls(cls._created(rc, h, "sdden_gmm_create"), d)

    @classmethod
    def sdden_lowrank_create(cls, mu, U, s2, alpha_bar_state):
        lib = load_library()
        mu, U, ab = (_host(v, np.float32) for v in (mu, U, alpha_bar_state))
        d, r = U.shape
        h = c_void_p()
        rc = lib.sdden_lowrank_create(d, r, mu.ctypes.data, U.ctypes.data, float(s2), ab.shape[0] - 1,
                                      ab.ctypes.data, ctypes.byref(h))
        return cls(cls._created(rc, h, "sdden_lowrank_create"), d)

    @classmethod
    def sdden_mlp_create(cls, p, T: int, Rmax: int):
        lib = load_library()
        W1, W2, W3 = (_host(v, np.uint16) for v in (p.W1, p.W2, p.W3))
        b1, b2, b3 = (_host(v, np.float32) for v in (p.b1, p.b2, p.b3))
        h = c_void_p()
        rc = lib.sdden_mlp_create(p.d, p.H, p.E, W1.ctypes.data, b1.ctypes.data, W2.ctypes.data,
                                  b2.ctypes.data, W3.ctypes.data, b3.ctypes.data, T, Rmax, ctypes.byref(h))
        den = cls(cls._created(rc, h, "sdden_mlp_create"), p.d)
        den.wants_bf16 = True                      # first layer reads bf16: sdden_eval_mirror saves a conversion pass
        return den

    def _check(self, rc, what):
        if rc != 0:
            raise SDError(f"{what} failed ({rc}): {self._lib.sdden_last_error(self._h).decode()}")

    def sdden_eval(self, R, X, krow, out):
        """X, out may be views into larger buffers (their first element is what is passed)."""
        for t, dt, nm in ((X, torch.float32, "X"), (krow, torch.int32, "krow"), (out, torch.float32, "out")):
            if not t.is_cuda or t.dtype != dt or not t.is_contiguous():
                raise SDError(f"{nm}: need a contiguous {dt} CUDA tensor")
        self._check(self._lib.sdden_eval(self._h, R, X.data_ptr(), krow.data_ptr(), out.data_ptr(), _stream()),
                    "sdden_eval")

    def sdden_eval_mirror(self, R, X, Xbf16, krow, out):
        for t, dt, nm in ((X, torch.float32, "X"), (Xbf16, torch.int16, "Xbf16"), (krow, torch.int32, "krow"),
                          (out, torch.float32, "out")):
            if not t.is_cuda or t.dtype != dt or not t.is_contiguous():
                raise SDError(f"{nm}: need a contiguous {dt} CUDA tensor")
        self._check(self._lib.sdden_eval_mirror(self._h, R, X.data_ptr(), Xbf16.data_ptr(), krow.data_ptr(),
                                                out.data_ptr(), _stream()), "sdden_eval_mirror")

    def sdden_reserve(self, Rmax: int):
        self._check(self._lib.sdden_reserve(self._h, Rmax), "sdden_reserve")

    def sdden_profile(self, which: int):
        self._check(self._lib.sdden_profile(self._h, which), "sdden_profile")

    def sdden_profile_min_rows(self, min_rows: int):
        self._check(self._lib.sdden_profile_min_rows(self._h, min_rows), "sdden_profile_min_rows")

    def sdden_profile_collect(self):
        ms, n = ctypes.c_double(), c_int64()
        self._check(self._lib.sdden_profile_collect(self._h, ctypes.byref(ms), ctypes.byref(n)),
                    "sdden_profile_collect")
        return ms.value, n.value

    def sdden_mlp_select_gemm(self, variant: int):
        self._check(self._lib.sdden_mlp_select_gemm(self._h, variant), "sdden_mlp_select_gemm")

    def sdden_set_active_count(self, count: Optional[torch.Tensor], rows_per_chain: int = 1):
        self._keep_count = count
        ptr = _dev(count, torch.int32, "count", allow_none=True)
        self._check(self._lib.sdden_set_active_count(self._h, ptr, rows_per_chain), "sdden_set_active_count")

    def close(self):
        if getattr(self, "_h", None):
            self._lib.sdden_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def sd_measure_stream(src: Optional[torch.Tensor], dst: torch.Tensor, nbytes: int, mode: int, workgroups: int = 0):
    """Measurement kernel (include/sd_measure.h): streaming copy (0), read (1) or fill (2) of nbytes; 3, 4, 5 the
    same with a workgroup walking whole 48 KiB rows."""
    lib = load_library()
    rc = lib.sd_measure_stream(None if src is None else src.data_ptr(), dst.data_ptr(), nbytes, mode, workgroups, _stream())
    if rc != 0:
        raise SDError(f"sd_measure_stream failed ({rc})")


def sd_measure_mfma(shape: int, iters: int, sink: torch.Tensor, workgroups: int = 0) -> float:
    """Measurement kernel (include/sd_measure.h): a loop of MFMAs on register operands; returns its flops."""
    lib = load_library()
    fl = ctypes.c_double()
    rc = lib.sd_measure_mfma(shape, iters, workgroups, sink.data_ptr(), ctypes.byref(fl), _stream())
    if rc != 0:
        raise SDError(f"sd_measure_mfma failed ({rc})")
    return fl.value
