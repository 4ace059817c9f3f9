"""Shared helpers of the GPU parity tests: the error metric and the device-side case object."""
import numpy as np

RTOL = 1e-4          # max relative error (the stated bar for fp32 activations, gradients, losses)
ABS_FLOOR = 1e-6     # absolute floor of the denominator
RMS_FLOOR = 1.0      # elements smaller than the reference tensor's rms are judged against the rms: an
                     # fp32 sum of K terms carries an absolute error of about 6e-8 * sqrt(K) * rms(result)
                     # whatever the size of the (possibly cancelling) element itself
RMS_TOL = 1e-5       # bound on rms(x - ref) / rms(ref): catches small systematic errors


def rel_err(x, ref):
    """max_i |x_i - ref_i| / max(|ref_i|, ABS_FLOOR, RMS_FLOOR * rms(ref))."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert x.shape == ref.shape, (x.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    den = np.maximum(np.abs(ref), max(ABS_FLOOR, RMS_FLOOR * rms))
    return float(np.max(np.abs(x - ref) / den))


def strict_rel_err(x, ref):
    """The same metric with the bare 1e-6 floor (reported, not asserted: see the design doc)."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(x - ref) / np.maximum(np.abs(ref), ABS_FLOOR)))


def rms_err(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    den = float(np.sqrt(np.mean(ref * ref)))
    return float(np.sqrt(np.mean((x - ref) ** 2))) / max(den, ABS_FLOOR)


def assert_close(x, ref, what):
    e = rel_err(x, ref)
    assert e <= RTOL, f"{what}: max relative error {e:.3e} > {RTOL:g}"
    r = rms_err(x, ref)
    assert r <= RMS_TOL, f"{what}: rms error {r:.3e} > {RMS_TOL:g}"
    return e


def tie_count(Z, band_rel=1e-5):
    """Pre-activations closer to zero than band_rel * rms: there the ReLU derivative is decided by
    rounding, so gradients further down are not unique."""
    Z = np.asarray(Z)
    rms = float(np.sqrt(np.mean(Z * Z)))
    return int(np.count_nonzero(np.abs(Z) < band_rel * rms))
