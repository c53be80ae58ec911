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


def check_activation_decisions(dev_hidden, ref, what="", say=None, calls_per_layer=2, scale_floor=0.0):
    """The device's ReLU decisions against the oracle's, per hidden layer.

    ref: an oracle epoch that was GIVEN the device's decisions (device_relu) and used them only
    inside its own ambiguous set (pre-activations that are zero at 1e-5 of the magnitude sum of
    their terms).  Asserts that outside that set the device decided as the oracle does, that the
    set is a small fraction of the entries, and that the hidden activations themselves match:
    layer l is the output of a chain of calls_per_layer * (l + 1) calls, each within 1e-5 of the
    magnitude sums of its terms.  scale_floor (random sweeps only): an entry whose own magnitude
    sum is below that fraction of the layer's largest is measured against that fraction (its
    operands carry the rounding of the calls before, relative to THEIR magnitude sums)."""
    for l, amb in enumerate(ref["relu_ambiguous"]):
        dev = np.asarray(dev_hidden[l], dtype=np.float64)
        own = ref["preact"][l] > 0
        differ = (dev > 0) != own
        if say:
            say("  %s layer %d: %d of %d pre-activations ambiguous at 1e-5 of their magnitude sums, %d device decisions differ"
                % (what, l, int(amb.sum()), amb.size, int(differ.sum())))
        assert not (differ & ~amb).any(), "%s layer %d: %d ReLU decisions differ outside the ambiguous set" % (what, l, int((differ & ~amb).sum()))
        assert amb.mean() <= 1e-3, "%s layer %d: ambiguous set too large (%.2e of the entries)" % (what, l, amb.mean())
        tol = calls_per_layer * (l + 1) * TOL_F32
        mag = ref["preact_mag"][l]
        err = np.abs(dev - ref["hidden"][l]) / np.maximum(np.maximum(mag, scale_floor * mag.max()), np.finfo(np.float64).tiny)
        if say:
            say("  %s layer %d: hidden activations within %.2e of their magnitude sums (bound %.0e)" % (what, l, err.max(), tol))
        assert err.max() <= tol, "%s layer %d: hidden activations off by %.2e of their magnitude sums" % (what, l, err.max())
