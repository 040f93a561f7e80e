"""Host-side checks that need no GPU: the library loads, exports what the headers declare, and
rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2501_05370_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for h in ("sd.h", "sdden.h", "sd_measure.h"):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(sd(?:den)?_[a-z0-9_]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    declared = _declared()
    assert declared == set(binding.exported_symbols())
    for name in declared:
        assert hasattr(lib, name), name


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(binding.SDError):
        binding.load_library(str(tmp_path / "nope.so"))


def test_create_validates_schedule_before_using_the_device():
    lib = binding.load_library()
    T = 4
    a = np.ones(T, np.float32); c = np.full(T, 0.1, np.float32)

    def create(sig, d=8, K=4):
        s = np.asarray(sig, np.float32)
        sch = binding._Schedule(T, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                c.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                s.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
        h = ctypes.c_void_p()
        return lib.sd_create(ctypes.byref(sch), d, K, ctypes.byref(h)), h

    assert create([0.1, 0.0, 0.1, 0.1])[0] == -2            # SD_ERR_SCHEDULE: sigma must be > 0
    assert b"sigma[1]" in lib.sd_last_error(None)
    assert create([0.1, np.nan, 0.1, 0.1])[0] == -2
    assert create([0.1] * 4, K=65)[0] == -1                 # SD_ERR_ARG: window above SD_MAX_WINDOW
    assert create([0.1] * 4, d=0)[0] == -1
    assert lib.sd_create(None, 8, 4, None) == -1
    assert lib.sd_destroy(None) == -1 and lib.sdden_destroy(None) == -1
    rc, h = create([0.1] * 4)
    assert rc in (0, -4)                                    # -4 (SD_ERR_HIP) where there is no GPU
    if rc == 0:
        assert lib.sd_set_temperature(h, 0.0) == -1 and lib.sd_set_draft_mode(h, 7) == -1
        assert lib.sd_workspace_bytes(h, 10) == 10 * 16 + 4 and lib.sd_workspace_bytes(h, 1025) == 1025 * 16 + 8
        lib.sd_destroy(h)


def test_denoiser_create_validates_arguments():
    lib = binding.load_library()
    h = ctypes.c_void_p()
    assert lib.sdden_gmm_create(0, 4, None, None, None, 3, None, ctypes.byref(h)) == -1
    mu = np.zeros((2, 3), np.float32); sd = np.zeros((2, 3), np.float32); lw = np.zeros(2, np.float32)
    ab = np.linspace(0.1, 1, 5).astype(np.float32)
    assert lib.sdden_gmm_create(2, 3, mu.ctypes.data, sd.ctypes.data, lw.ctypes.data, 4, ab.ctypes.data,
                                ctypes.byref(h)) == -1      # stds must be positive
    assert b"stds" in lib.sdden_last_error(None)


def test_bench_refuses_more_than_one_gpu_and_needs_the_library():
    """bench.py is a one-GPU program: --gpus 2 ends with a message before anything touches a device; and the
    product path has no CPU stand-in (without a GPU the run ends with an error, not with oracle numbers)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120, cwd=root)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)
    import torch
    if not torch.cuda.is_available():
        r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--workload", "c1", "--no-cpu-baseline"],
                           capture_output=True, text=True, timeout=300, cwd=root)
        assert r.returncode != 0 and '"metric"' not in r.stdout
