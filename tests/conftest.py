import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def rel_err(a, b):
    """Relative Frobenius error ||a-b||_F / max(||b||_F, 1e-30)."""
    import numpy as np
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm((a - b).ravel()) / max(np.linalg.norm(b.ravel()), 1e-30))


def max_err(a, b):
    """Largest element-wise error in units of the reference's root mean square:
    max |a - b| / max(rms(b), 1e-30)."""
    import numpy as np
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    if b.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(b.ravel() ** 2)))
    return float(np.abs(a - b).max() / max(rms, 1e-30))


# An error of relative Frobenius size e spread evenly over N elements has rms e * rms(b); the largest of N
# Gaussian draws is 5-6 rms for N up to 1e8.  Rounding errors are not Gaussian (they grow with the element), so
# the element-wise bar is ELEM x the Frobenius bar: still 30-600 x below "one element is wrong by its own size"
# (max_err >= ~1) for the bars used here (2e-2 ... 1e-5).
ELEM = 16.0
# Gradients of ReLU networks with bf16-stored activations are not continuous in the rounding of a sum: where fp32 and
# fp64 sums fall on different sides of a bf16 rounding boundary the stored activation differs by one bf16 step, and a
# unit whose pre-activation that moves across zero takes the other ReLU decision.  Such a unit adds or removes one
# sample's term in a whole row of a weight gradient - of the order of 1 / sqrt(minibatch) of an element's typical
# size, several times that where the sample's delta and activation are both large - for a handful of units per
# worker.  For those comparisons (`flips=True`) the element-wise bar may be exceeded by at most FLIP_FRACTION of the
# elements, and by none by FLIP_CAP root-mean-squares or more ("wrong by its own typical size").  On the GPU the
# bf16 cases show at most 6e-5 of the elements over the bar and a largest error of 0.51 rms (configs[3], minibatch 32).
FLIP_FRACTION = 1e-3
FLIP_CAP = 1.0


def check_close(a, b, tol, what="", elem=ELEM, flips=False):
    """Both comparators of a parity assertion: relative Frobenius error below `tol` AND every element within
    `elem * tol` root-mean-squares of the reference (with `flips`: all but FLIP_FRACTION of them, and every one
    within FLIP_CAP).  Returns (rel_err, max_err) for printing."""
    import numpy as np
    e, m = rel_err(a, b), max_err(a, b)
    if os.environ.get("DPSGD_TEST_STATS"):
        a64, b64 = np.asarray(a, np.float64), np.asarray(b, np.float64)
        rms = max(float(np.sqrt(np.mean(b64.ravel() ** 2))), 1e-30) if b64.size else 1.0
        over = float(np.mean(np.abs(a64 - b64) > elem * tol * rms)) if b64.size else 0.0
        print(f"    [stats] {what}: frobenius {e:.3e} max {m:.3e} rms, fraction over {elem * tol:.1e}: {over:.3e}, "
              f"size {b64.size}, flips={flips}", flush=True)
    assert e < tol, f"{what}: relative Frobenius error {e:.3e} >= {tol:.1e}"
    if flips and m >= elem * tol:
        a64, b64 = np.asarray(a, np.float64), np.asarray(b, np.float64)
        rms = max(float(np.sqrt(np.mean(b64.ravel() ** 2))), 1e-30)
        over = float(np.mean(np.abs(a64 - b64) > elem * tol * rms))
        assert over <= FLIP_FRACTION, f"{what}: {over:.3e} of the elements are over {elem * tol:.1e} rms (Frobenius {e:.3e})"
        assert m < FLIP_CAP, f"{what}: largest element error {m:.3e} rms >= {FLIP_CAP} (Frobenius {e:.3e})"
        return e, m
    assert m < elem * tol, f"{what}: largest element error {m:.3e} rms >= {elem * tol:.1e} (Frobenius {e:.3e})"
    return e, m
