"""Helpers shared by the GPU parity tests: error metric and case announcement."""
import sys

import numpy as np


def announce(msg: str):
    """Name the case on the real stderr before a GPU step or a long checker run.  pytest captures
    at the file-descriptor level, so its capture is suspended for the write: the line then shows
    while the test is still running, which names the case if the run dies and shows that a long
    test is alive."""
    capman = None
    try:
        import conftest
        capman = conftest.CAPTURE_MANAGER
    except ImportError:
        pass
    if capman is not None:
        capman.suspend_global_capture(in_=False)
    try:
        sys.__stderr__.write("[gpu-case] " + msg + "\n")
        sys.__stderr__.flush()
    finally:
        if capman is not None:
            capman.resume_global_capture()


def rel_err(got: np.ndarray, ref: np.ndarray):
    """(relative L2 error, max abs error / max abs ref) of one tensor."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    tiny = 1e-30
    l2 = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), tiny)
    mx = np.abs(got - ref).max() / max(np.abs(ref).max(), tiny) if ref.size else 0.0
    return float(l2), float(mx)


def assert_close(got, ref, tol, what):
    """Relative L2 error and max error (relative to the reference's largest element) within tol."""
    assert np.all(np.isfinite(got)), what + ": non-finite values"
    if not np.any(ref):            # an all-zero reference (e.g. zero-initialised bias gradient) must match exactly-ish
        assert np.abs(got).max() <= 1e-12, what + ": expected zeros"
        return
    l2, mx = rel_err(got, ref)
    assert l2 <= tol and mx <= tol, "%s: rel L2 %.3e, rel max %.3e (tol %.1e)" % (what, l2, mx, tol)
