"""Helpers shared by the GPU parity tests (tolerances from the benchmark spec:
indices bit-exact, log-partition 1e-5 relative, posteriors 1e-5 absolute)."""
import contextlib

import numpy as np
import torch

TOL_D_REL = 1e-5
TOL_POST_ABS = 1e-5


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def announce(*what):
    print("[case]", *what, flush=True)


def assert_dist_close(got, want, what="D"):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    fin = np.isfinite(want)
    assert np.array_equal(np.isfinite(got), fin), (what, got, want)
    assert np.array_equal(got[~fin], want[~fin]) or np.all(np.isnan(want[~fin]) == np.isnan(got[~fin]))
    err = np.abs(got[fin] - want[fin]) / np.maximum(1.0, np.abs(want[fin]))
    assert err.size == 0 or err.max() <= TOL_D_REL, (what, err.max(), got, want)


@contextlib.contextmanager
def library_option(option, value):
    """Set a process-wide option of the library for the duration of a with-block."""
    from paper_2304_13134_amd import binding as lb
    old = lb.set_option(option, value)
    try:
        yield
    finally:
        lb.set_option(option, old)
