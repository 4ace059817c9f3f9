"""Shared helpers of the GPU parity tests: the error metric.

The stated bar for fp32 activations, gradients and losses is a maximum relative error of 1e-4 with
an absolute floor of 1e-6:  |x - ref| <= RTOL * max(|ref|, ABS_FLOOR)              ("bare metric").
Every tensor of the step is a sum of K products, and an fp32 evaluation of such a sum, in any
order, is off by up to a few units of rounding times the sum S of the ABSOLUTE values of its terms,
however small the result itself is by cancellation.  The oracle computes S and K per element
(oracle.bns_oracle.layer_*_bounds, pinned against dense brute force), and the tests assert

    |x - ref| <= RTOL * max(|ref|, ABS_FLOOR) + C_ERR * U * sqrt(K) * S            ("bounded metric")

for every element, plus the bare metric on every element that is not small by cancellation
(|ref| >= S / COND), plus a bound on the rms error of the tensor (systematic errors).

C_ERR: one rounding of a running sum of same-sign terms contributes at most U * S, uniformly
distributed, i.e. a standard deviation of U * S / sqrt(3) per step and U * S * sqrt(K) / 3 for K
steps whose partial sums grow linearly; the maximum over the 1e7..1e8 elements of a tensor sits about
6 standard deviations out: 2 * U * sqrt(K) * S.  A second factor of 2 covers the roundings of the
factors themselves (the product d~_v^-1/2 d~_u^-1/2 / p in fp32, inputs rounded to fp32).
"""
import numpy as np

RTOL = 1e-4          # max relative error (the stated bar for fp32 activations, gradients, losses)
ABS_FLOOR = 1e-6     # absolute floor of the denominator
U = 2.0 ** -24       # unit roundoff of fp32
C_ERR = 4.0          # see the module docstring
COND = 4.0           # an element with |ref| >= S / COND lost at most two bits to cancellation
RMS_TOL = 1e-5       # bound on rms(x - ref) / rms(ref): catches small systematic errors


def tolerance(ref, S, K, stages=1.0):
    """Element-wise bound of the bounded metric.  stages: number of chained layer stages the inputs of
    this tensor went through in fp32 before (1 for a layer fed with exact inputs)."""
    ref = np.asarray(ref, dtype=np.float64)
    return RTOL * np.maximum(np.abs(ref), ABS_FLOOR) + stages * C_ERR * U * np.sqrt(K) * np.asarray(S)


def bare_err(x, ref, where=None):
    """max_i |x_i - ref_i| / max(|ref_i|, ABS_FLOOR), over the elements selected by ``where``."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert x.shape == ref.shape, (x.shape, ref.shape)
    r = np.abs(x - ref) / np.maximum(np.abs(ref), ABS_FLOOR)
    if where is not None:
        r = r[where]
    return float(r.max()) if r.size else 0.0


def rms_err(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    den = float(np.sqrt(np.mean(ref * ref)))
    return float(np.sqrt(np.mean((x - ref) ** 2))) / max(den, ABS_FLOOR)


class Report:
    """Collects what the assertions measured, for the log line of a test."""

    def __init__(self):
        self.worst_ratio = 0.0     # max |x - ref| / tolerance          (bounded metric, must be <= 1)
        self.worst_bare = 0.0      # bare metric over the well-conditioned elements (must be <= RTOL)
        self.worst_bare_all = 0.0  # bare metric over all elements (reported only)
        self.min_cover = 1.0       # smallest fraction of a tensor's elements that is well conditioned

    def line(self):
        return (f"bounded metric: worst |err|/tol {self.worst_ratio:.3f}; bare 1e-4/1e-6 metric on the "
                f"well-conditioned elements {self.worst_bare:.2e} (they are >= {100 * self.min_cover:.1f}% of "
                f"each tensor), on all elements {self.worst_bare_all:.2e}")


def assert_within(x, ref, bound, what, report=None, stages=1.0, rms_tol=RMS_TOL):
    """The three assertions of the module docstring.  bound = (S, K) from the oracle."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert x.shape == ref.shape, (what, x.shape, ref.shape)
    if ref.size == 0:
        return
    S, K = bound
    S = np.broadcast_to(np.asarray(S, dtype=np.float64), ref.shape)
    err = np.abs(x - ref)
    tol = tolerance(ref, S, K, stages)
    ratio = float((err / tol).max())
    assert ratio <= 1.0, (f"{what}: |x - ref| exceeds 1e-4 * max(|ref|, 1e-6) + {stages * C_ERR:g} * 2^-24 * sqrt(K) * S "
                          f"by a factor {ratio:.3g} at {np.unravel_index(np.argmax(err / tol), ref.shape)}")
    well = np.abs(ref) * COND >= S
    bare_well = bare_err(x, ref, well)
    assert bare_well <= RTOL * stages, f"{what}: bare metric {bare_well:.3e} on elements that are not small by cancellation"
    r = rms_err(x, ref)
    assert r <= rms_tol * stages, f"{what}: rms error {r:.3e} > {rms_tol * stages:g}"
    if report is not None:
        report.worst_ratio = max(report.worst_ratio, ratio)
        report.worst_bare = max(report.worst_bare, bare_well)
        report.worst_bare_all = max(report.worst_bare_all, bare_err(x, ref))
        report.min_cover = min(report.min_cover, float(np.count_nonzero(well)) / ref.size)


def assert_bare(x, ref, what):
    """The stated bar without any allowance (losses, weights after an optimiser step, ...)."""
    e = bare_err(x, ref)
    assert e <= RTOL, f"{what}: max relative error {e:.3e} > {RTOL:g} (floor {ABS_FLOOR:g})"
    return e


def tie_count(Z, band_rel=1e-5):
    """Pre-activations closer to zero than band_rel * rms: there the ReLU derivative is decided by
    rounding, so gradients further down are not unique."""
    Z = np.asarray(Z)
    rms = float(np.sqrt(np.mean(Z * Z)))
    return int(np.count_nonzero(np.abs(Z) < band_rel * rms))


def tie_cap(n_hidden, band_rel=1e-5):
    """Upper limit on tie_count for n_hidden pre-activations: at most one hidden unit in ten thousand
    (a Gaussian of the same rms puts 0.8 * band_rel = 8e-6 of its mass into the band; sparse
    non-negative inputs concentrate more of it near zero, measured up to 7e-5), plus a few."""
    return int(8 + 10.0 * band_rel * n_hidden)
