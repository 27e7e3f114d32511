"""Helpers shared by the GPU parity tests."""
import os
import time

import numpy as np

TOL_F32 = 1e-4     # spec tolerance for fp32 activations and gradients
TOL_BF16 = 2e-2


def rel_errs(got, ref):
    """(max-abs error / max |ref|, Frobenius error / Frobenius norm of ref)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0, 0.0
    diff = np.abs(got - ref)
    den_max = max(np.abs(ref).max(), 1e-30)
    den_fro = max(np.sqrt((ref * ref).sum()), 1e-30)
    return diff.max() / den_max, np.sqrt((diff * diff).sum()) / den_fro


def assert_close(got, ref, tol=TOL_F32, what=""):
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), f"{what}: non-finite values"
    e_max, e_fro = rel_errs(got, ref)
    assert e_max <= tol and e_fro <= tol, f"{what}: rel err max {e_max:.3e} fro {e_fro:.3e} > {tol}"


def to_f64_model(kind, layers):
    return {"kind": kind, "layers": [{k: np.asarray(v, dtype=np.float64) for k, v in l.items()} for l in layers]}


_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_T0 = time.time()


def progress(msg):
    """Progress line of a long test: printed (visible with -s) and appended to test_progress.log in the run's
    output folder, so that a run whose output pytest captures still shows which step it is in."""
    line = f"[{time.time() - _T0:7.1f} s] {msg}"
    print(line, flush=True)
    try:
        d = os.path.join(_ROOT, "gpurun_out")
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "test_progress.log"), "a") as f:
            f.write(line + "\n")
    except OSError:
        pass
