"""Comparison rules shared by the GPU parity tests (test-side only).

Codes.  The GPU rotates in fp32, the oracle in fp64, so a pre-round value that
sits on a rounding boundary may legitimately round the other way.  A GPU code
may differ from the oracle's by +-1 only where the oracle's pre-round value
t = y / Delta lies within CODE_TOL_REL * (row full scale) of a half-integer,
i.e. within CODE_TOL_REL * max|t| code units.  Everything else must be equal.
Scales are compared at SCALE_RTOL.  fp16 outputs: max |Y_gpu - Y_oracle| <=
OUT_TOL * rms(Y_oracle), with Y_oracle computed from the same codes and scales.
"""
import numpy as np

CODE_TOL_REL = 1e-6
SCALE_RTOL = 1e-6
OUT_TOL = 1e-2


def check_codes(gpu_codes: np.ndarray, ora_codes: np.ndarray, ora_t: np.ndarray, what: str = "codes"):
    """Returns the number of tolerated boundary flips; raises on anything else."""
    gpu_codes = np.asarray(gpu_codes).astype(np.int16)
    ora_codes = np.asarray(ora_codes).astype(np.int16)
    assert gpu_codes.shape == ora_codes.shape, (gpu_codes.shape, ora_codes.shape)
    assert gpu_codes.min(initial=0) >= -8 and gpu_codes.max(initial=0) <= 7
    diff = gpu_codes != ora_codes
    n = int(diff.sum())
    if n == 0:
        return 0
    r, c = np.nonzero(diff)
    d = gpu_codes[r, c] - ora_codes[r, c]
    assert np.all(np.abs(d) == 1), "%s: %d codes differ by more than 1 (first at %s)" % (
        what, int((np.abs(d) > 1).sum()), (r[0], c[0]))
    t = ora_t[r, c]
    tol = CODE_TOL_REL * np.abs(ora_t).max(axis=1)[r]
    dist = np.abs(t - (np.floor(t) + 0.5))                   # distance to the nearest half-integer
    bad = dist > tol
    assert not bad.any(), "%s: %d of %d mismatches are not at a rounding boundary (worst distance %.3g, tol %.3g)" % (
        what, int(bad.sum()), n, float(dist.max()), float(tol.min()))
    # the flip must go towards the other side of that boundary
    assert np.all(np.sign(d) == np.sign(t - ora_codes[r, c])), what + ": flip away from the boundary"
    return n


def check_scales(gpu: np.ndarray, ora: np.ndarray, what: str = "scales"):
    np.testing.assert_allclose(np.asarray(gpu, np.float64), ora, rtol=SCALE_RTOL, atol=0, err_msg=what)


def check_output(y_gpu: np.ndarray, y_ora: np.ndarray, what: str = "Y"):
    y_gpu = np.asarray(y_gpu, np.float64)
    rms = float(np.sqrt(np.mean(y_ora ** 2)))
    err = float(np.abs(y_gpu - y_ora).max(initial=0.0))
    assert err <= OUT_TOL * rms + 1e-30, "%s: max abs err %.4g > %.0e * rms %.4g" % (what, err, OUT_TOL, rms)
    return err / rms if rms else 0.0
