import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

TOL = 2.0 ** -10   # parity bound: |Y - Y_ref| <= TOL * (|W| |X|), element-wise


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI)")


def assert_within_scaled_tolerance(Y, Y_ref, S, tol=TOL, what=""):
    """Element-wise |Y - Y_ref| <= tol * S + floor; where S == 0 the result must be 0.

    floor: what the output format itself cannot resolve.  A binary16 output below 2^-14 is
    subnormal, with values 2^-24 apart, so a correctly rounded result may be 2^-25 away from the
    exact one however small S is (a group that keeps one column and meets two small operands);
    float32 outputs (and bfloat16 ones, whose subnormals are 2^-133 apart) have no such floor here."""
    floor = 2.0 ** -25 if np.asarray(Y).dtype == np.float16 else 0.0
    Y = np.asarray(Y, dtype=np.float64)
    err = np.abs(Y - Y_ref)
    assert np.all(np.isfinite(Y)), what + ": non-finite output"
    zero = S == 0
    assert np.all(Y[zero] == 0), what + ": non-zero output where no term contributes"
    ratio = np.where(zero, 0.0, np.maximum(err - floor, 0.0) / np.where(zero, 1.0, S))
    worst = float(ratio.max()) if ratio.size else 0.0
    assert worst <= tol, "%s: max scaled error %.3e > %.3e at %r" % (
        what, worst, tol, np.unravel_index(int(ratio.argmax()), ratio.shape))
    return worst
