"""Shared helpers of the parity tests (no arithmetic of the method here)."""
import numpy as np

TOL_F32 = 1e-5      # max relative error, fp32 path
TOL_BF16 = 2e-2     # max relative error, bf16 feature variant


def rel_errors(got, ref, ref_abs):
    """Two relative errors of `got` against the fp64 reference:
    normwise  max|got-ref| / max|ref|, and componentwise against the sum of absolute
    terms  max |got-ref| / ref_abs  (the scale that bounds the rounding error of any
    summation order, so it stays meaningful where terms cancel)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    diff = np.abs(got - ref)
    scale = np.abs(ref).max() if ref.size else 0.0
    normwise = float(diff.max() / scale) if scale > 0 else float(diff.max() if diff.size else 0.0)
    pos = ref_abs > 0
    comp = float((diff[pos] / ref_abs[pos]).max()) if pos.any() else 0.0
    zero_ok = bool(np.all(diff[~pos] == 0)) if (~pos).any() else True
    return normwise, comp, zero_ok


def assert_close(got, ref, ref_abs, tol, what=""):
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), what + ": non-finite output"
    normwise, comp, zero_ok = rel_errors(got, ref, ref_abs)
    assert normwise <= tol, "%s: normwise error %.3e > %.1e" % (what, normwise, tol)
    assert comp <= tol, "%s: componentwise error %.3e > %.1e" % (what, comp, tol)
    assert zero_ok, what + ": nonzero output where every term is zero"
