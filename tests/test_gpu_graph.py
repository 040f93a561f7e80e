"""The window loop with the batch size kept on the device (several windows per host readback) and
with window + advance captured in a HIP graph must give exactly the results of the plain loop:
same kernels, same inputs, noise keyed by chain id and step.  Graph replays are repeated, with
eager work and synchronisations in between, and every run is compared with the eager result.
"""
import numpy as np
import pytest
import torch

import workloads as W

from _gpu import host

pytestmark = pytest.mark.gpu


def _cases():
    return [("c1", dict(), "frozen"), ("c2", dict(B=300, T=60), "frozen"), ("c2", dict(B=200, T=50), "efficient_frozen"),
            ("c5", dict(B=96, d=200, M=4, K=8, T=80), "frozen"), ("phi4", dict(B=150, T=90), "frozen"),
            ("c3", dict(B=40, d=256, r=32, K=6, T=40), "frozen"), ("c4", dict(B=24, d=512, H=256, K=6, T=30), "frozen")]


@pytest.mark.parametrize("name,kw,drafter", _cases())
def test_device_count_and_graph_runs_equal_the_eager_run(name, kw, drafter):
    from paper_2501_05370_amd.runner import make_sampler
    cfg = W.make_config(name, **kw)
    ids = torch.arange(cfg.B, dtype=torch.int64, device="cuda")
    smp = make_sampler(cfg, drafter=drafter)
    out, c0 = smp.run(ids)
    ref = host(out).copy()
    assert c0[0] == cfg.B * cfg.T
    # several windows per readback, batch size read from the device by every kernel
    out, c1 = smp.run(ids, windows_per_sync=5)
    assert np.array_equal(host(out), ref) and c1 == c0
    # graph replays: three runs, eager work and synchronisations between them
    for rep in range(3):
        out, c2 = smp.run(ids, windows_per_sync=3, graph=True)
        assert np.array_equal(host(out), ref), f"replay run {rep}"
        assert c2 == c0
        scratch = torch.randn(1 << 16, device="cuda").sum().item()      # unrelated eager work + a sync
        assert np.isfinite(scratch)
    # and the plain loop still gives the same afterwards (device count switched off again)
    out, c3 = smp.run(ids)
    assert np.array_equal(host(out), ref) and c3 == c0
