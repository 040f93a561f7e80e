"""sd_advance_static -- the advance entry point for callers that cannot allocate -- against sd_advance.

Both are called through the C ABI (raw ctypes handles, device pointers of torch tensors) on the same
inputs; every output must be bit-identical (integer / index work and row copies).  Two calls in a row on
one context, the second with a smaller batch, so that what the first call left in the library's static
scratch lies behind the second call's data.  No workspace is ever given to the context that calls the
static entry point.
"""
import ctypes

import numpy as np
import pytest
import torch

import workloads as W
from paper_2501_05370_amd import binding

pytestmark = pytest.mark.gpu


def _create(lib, sched, d, K):
    a = np.ascontiguousarray(sched.a, np.float32)
    c = np.ascontiguousarray(sched.c, np.float32)
    s = np.ascontiguousarray(sched.sigma, np.float32)
    fp = ctypes.POINTER(ctypes.c_float)
    sch = binding._Schedule(a.shape[0], a.ctypes.data_as(fp), c.ctypes.data_as(fp), s.ctypes.data_as(fp))
    h = ctypes.c_void_p()
    rc = lib.sd_create(ctypes.byref(sch), d, K, ctypes.byref(h))
    assert rc == 0, lib.sd_last_error(None)
    return h


def _inputs(rng, B, d, T, K):
    n = rng.integers(T - 8, T, size=B).astype(np.int32)
    adv = np.minimum(rng.integers(1, K + 1, size=B), T - n).astype(np.int32)
    rej = rng.integers(0, 2, size=B).astype(np.uint8)
    ids = rng.permutation(B).astype(np.int64)
    y_out = rng.standard_normal((B, d)).astype(np.float32)
    return n, adv, rej, ids, y_out


def _call(fn, lib, h, B, d, n, adv, rej, ids, y_out, Bout):
    """One advance through `fn`; returns every output as host arrays."""
    t = lambda a, dt: torch.as_tensor(a, dtype=dt).cuda().contiguous()
    gy = torch.full((max(B, 1), d), -1.0, dtype=torch.float32, device="cuda")
    gn, gid = t(n, torch.int32), t(ids, torch.int64)
    gyo, gadv, grej = t(y_out, torch.float32), t(adv, torch.int32), t(rej, torch.uint8)
    gout = torch.zeros(max(Bout, 1), d, dtype=torch.float32, device="cuda")
    gB = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(5, dtype=torch.int64, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    rc = fn(h, B, gyo.data_ptr(), gadv.data_ptr(), grej.data_ptr(), gy.data_ptr(), gn.data_ptr(), gid.data_ptr(),
            gout.data_ptr(), gB.data_ptr(), cnt.data_ptr(), stream)
    assert rc == 0, lib.sd_last_error(h)
    torch.cuda.synchronize()
    Ba = int(gB.item())
    return dict(B_active=Ba, y=gy[:Ba].cpu().numpy(), n=gn[:Ba].cpu().numpy(), ids=gid[:Ba].cpu().numpy(),
                out=gout.cpu().numpy(), counters=cnt.cpu().numpy())


@pytest.mark.parametrize("d", [4, 1000, 5])
def test_static_advance_matches_workspace_advance_on_two_calls_in_a_row(d):
    lib = binding.load_library()
    T, K = 50, 6
    sched = W.linear_beta_schedule(T)
    h_ws, h_st = _create(lib, sched, d, K), _create(lib, sched, d, K)
    B1 = binding.SD_STATIC_MAX_CHAINS if d == 4 else (40000 if d < 100 else 3000)   # d = 4: the largest batch the scratch holds
    B2 = 1500 if d < 100 else 70
    ws = torch.empty(lib.sd_workspace_bytes(h_ws, B1), dtype=torch.uint8, device="cuda")
    assert lib.sd_set_workspace(h_ws, ws.data_ptr(), ws.numel()) == 0
    rng = np.random.default_rng(11)
    for B in (B1, B2):                       # the second call is smaller: stale scratch lies behind its data
        n, adv, rej, ids, y_out = _inputs(rng, B, d, T, K)
        want = _call(lib.sd_advance, lib, h_ws, B, d, n, adv, rej, ids, y_out, B)
        got = _call(lib.sd_advance_static, lib, h_st, B, d, n, adv, rej, ids, y_out, B)
        assert got["B_active"] == want["B_active"] and 0 < want["B_active"] < B
        for key in ("y", "n", "ids", "out", "counters"):
            assert np.array_equal(got[key], want[key]), (B, key)
    lib.sd_destroy(h_ws)
    lib.sd_destroy(h_st)


def test_static_advance_rejects_batches_beyond_its_scratch_and_handles_an_empty_batch():
    lib = binding.load_library()
    T, K, d = 50, 6, 4
    h = _create(lib, W.linear_beta_schedule(T), d, K)
    B = binding.SD_STATIC_MAX_CHAINS + 1
    one = torch.zeros(1, dtype=torch.int32, device="cuda")
    p = one.data_ptr()                       # never dereferenced: the size check comes first
    assert lib.sd_advance_static(h, B, p, p, p, p, p, p, p, p, None, None) == -3      # SD_ERR_WORKSPACE
    assert b"static scratch" in lib.sd_last_error(h)
    gB = torch.full((1,), 5, dtype=torch.int32, device="cuda")
    assert lib.sd_advance_static(h, 0, None, None, None, None, None, None, None, gB.data_ptr(), None, None) == 0
    torch.cuda.synchronize()
    assert int(gB.item()) == 0
    lib.sd_destroy(h)
