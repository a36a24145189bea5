"""Comparison helpers for the table-interpolated variant, shared by the GPU and the emulation tests."""
import numpy as np

import oracle

KNOT_BAND = 2e-3


def dx_error(dx, x, C, dy, lut):
    """Worst |dx - oracle| / RMS(oracle) over all elements.

    dx uses the difference quotient of the chosen table cell, which jumps at the knots.  An fp32
    implementation takes the cell in fp32, the oracle in fp64: an element whose position lies within
    KNOT_BAND cells of a knot may legitimately use either neighbouring cell, so it is compared with
    both and the smaller error counts.  Every other element is compared with the oracle's cell only.
    """
    ref, _, frac = oracle.backward_lut(x, C, dy, lut, need_dC=False, want_frac=True)
    scale = float(np.sqrt(np.mean(ref * ref)))
    if not np.all(np.isfinite(dx)):
        return float("inf")
    err = np.abs(dx - ref) / scale
    near_lo, near_hi = frac < KNOT_BAND, frac > 1.0 - KNOT_BAND
    near = near_lo | near_hi
    if near.any():
        shift = np.where(near_lo, -1, np.where(near_hi, 1, 0)).astype(np.int8)
        alt, _ = oracle.backward_lut(x, C, dy, lut, need_dC=False, shift=shift)
        err = np.where(near, np.minimum(err, np.abs(dx - alt) / scale), err)
    return float(err.max())
