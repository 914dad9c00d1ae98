"""What the GPU parity tests share: the tolerance, the two error measures, and progress lines."""
import os
import sys

import numpy as np

RTOL = 1e-3     # the bar the benchmark spec fixes for fp32, applied per tensor to both measures of errs()

# where the progress lines go besides stdout: POOCH_TEST_LOG_DIR, else the output folder next to tests/ that is listed in .gitignore
_PROGRESS = os.path.join(os.environ.get("POOCH_TEST_LOG_DIR") or
                         os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out"), "gpu_tests_progress.log")


def say(*a):
    """a line per case and step: to stdout (pytest shows it for a failing test) and, because pytest holds stdout
    back while a test runs, appended to a log file as well, so that a long case is seen to be moving"""
    print(*a)
    sys.stdout.flush()
    try:
        os.makedirs(os.path.dirname(_PROGRESS), exist_ok=True)
        with open(_PROGRESS, "a") as f:
            f.write(" ".join(str(v) for v in a) + "\n")
    except OSError:
        pass


def errs(a, b):
    """(||a - b||_2 / ||b||_2, max |a - b| / rms(b)), in float64, chunked so that large tensors are not copied whole"""
    a = np.asarray(a).ravel()
    b = np.asarray(b).ravel()
    assert a.size == b.size
    d2 = b2 = dmax = 0.0
    for lo in range(0, a.size, 1 << 24):
        bb = b[lo:lo + (1 << 24)].astype(np.float64)
        dd = a[lo:lo + (1 << 24)].astype(np.float64) - bb
        d2 += float(dd @ dd)
        b2 += float(bb @ bb)
        dmax = max(dmax, float(np.abs(dd).max()))
    nb = max(np.sqrt(b2), 1e-30)
    return float(np.sqrt(d2) / nb), float(dmax / (nb / np.sqrt(max(a.size, 1))))


def rel(a, b):
    return errs(a, b)[0]


def close(what, a, b, tol=None):
    """both bars of the header; returns the larger of the two errors (each in units of its own bar's scale)"""
    tol = RTOL if tol is None else tol
    assert np.isfinite(np.asarray(a)).all(), (what, "not finite")
    r, m = errs(a, b)
    assert r <= tol, (what, "relative L2 error", r, "bar", tol)
    assert m <= tol, (what, "largest element error / rms of the reference", m, "bar", tol)
    return max(r, m)
