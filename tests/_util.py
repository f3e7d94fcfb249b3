"""Shared helpers of the GPU parity tests."""
import os
import time

import numpy as np
import torch

TOL = 1e-4          # max |err| <= TOL * (1 + |ref|), the bar for fp32 activations and gradients

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def progress(msg):
    """A line for the long full-size tests: printed, and appended to a log that a watcher of the run can
    see growing while pytest holds the output back."""
    line = f"{time.strftime('%H:%M:%S')} {msg}"
    print(line, flush=True)
    try:
        os.makedirs(os.path.join(_ROOT, "gpurun_out"), exist_ok=True)
        with open(os.path.join(_ROOT, "gpurun_out", "test_progress.log"), "a") as f:
            f.write(line + "\n")
    except OSError:
        pass


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def host(t):
    return t.detach().cpu().numpy()


def assert_close(got, ref, name="", tol=TOL):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{name}: non-finite values"
    if got.size == 0:
        return
    excess = np.abs(got - ref) - tol * (1.0 + np.abs(ref))
    worst = np.unravel_index(np.argmax(excess), excess.shape)
    assert excess[worst] <= 0, (
        f"{name}: |err| = {abs(got[worst] - ref[worst]):.3e} at {worst} "
        f"(got {got[worst]:.6e}, ref {ref[worst]:.6e}); "
        f"rel Frobenius err {np.linalg.norm(got - ref) / (np.linalg.norm(ref) + 1e-300):.3e}")


def rel_fro(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / (np.linalg.norm(ref) + 1e-300))
