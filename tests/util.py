"""Helpers shared by the tests."""
import os

import numpy as np


def ensure_built():
    """Load what is built; build only if nothing is."""
    from paper_2511_18297_amd import build as groot_build

    if not os.path.exists(groot_build.LIB_PATH):
        groot_build.build()


def tolerance(S):
    """Accepted fp32-vs-fp64 deviation per element: 1e-5 * sum|a_ij x_jk| + 1e-6."""
    return 1e-5 * S + 1e-6


def assert_close_to_oracle(Y_gpu, Y64, S, what=""):
    Y_gpu = np.asarray(Y_gpu, dtype=np.float64)
    assert Y_gpu.shape == Y64.shape, (Y_gpu.shape, Y64.shape)
    assert np.isfinite(Y_gpu).all(), f"{what}: non-finite output (a row was not written?)"
    err = np.abs(Y_gpu - Y64)
    tol = tolerance(S)
    bad = err > tol
    if bad.any():
        i, k = np.argwhere(bad)[0]
        raise AssertionError(f"{what}: {bad.sum()} elements out of tolerance, first at row {i} col {k}: "
                             f"gpu {Y_gpu[i, k]!r} oracle {Y64[i, k]!r} tol {tol[i, k]!r}")
    return float(np.max(err / tol))


def layer_tolerance(S, scale, absWn, floor=1e-6, pieces=3):
    """Accepted deviation of the fused layer from the fp64 layer, element by element.  The aggregation's own
    bar, 1e-5 * sum|a_ij x_jk| + 1e-6 per element of A_hat X, reaches the output through |Wn|; the dense part
    is an fp32 sum of 2F + 1 <= 129 terms (two products per input feature and the bias) whose rounding error
    is at most (2F + 2) * 2^-24 <= 7.8e-6 of the sum of their magnitudes in any order of summation, each
    product being exact to 2^-23 of itself: together below 1e-5 * scale, scale = |A_hat X| |Wn| + |X| |Ws| + |b|,
    the same coefficient as the aggregation's bar.  With two bf16 pieces per operand instead of three (the
    library's sage_pieces knob) a product is exact to 3 * 2^-18 of itself instead (each operand is represented to
    2^-18, and the product of the two second pieces, at most 2^-18, is dropped), which adds that much of scale."""
    dense = 1e-5 + (3 * 2.0 ** -18 if pieces == 2 else 0.0)
    return (1e-5 * S + floor) @ absWn + dense * scale + floor


def wgrad_tolerance(Sn, Ss, dz_abs_colsum, rows_per_wavefront, pieces=3, floor=1e-6):
    """Accepted deviation of the fused layer's weight gradients dWn = (A_hat X)^T dZ and dWs = X^T dZ from fp64,
    element by element.  Sn = S^T |dZ| with S the aggregation's own sums of absolute terms, Ss = |X|^T |dZ|.  The
    aggregation's bar (1e-5 S + 1e-6 per element of A_hat X) reaches dWn through |dZ|; each product is exact to
    2^-23 of itself (three bf16 pieces per operand; two pieces: 3 * 2^-18); a wavefront adds the products of the
    rows it sweeps in fp32, 16 at a time in the matrix instruction and tile after tile into its accumulator,
    at most (rows + 16) roundings of 2^-24 of the sum of magnitudes; the sums of the wavefronts meet in fp64 and
    the result is rounded to fp32 once."""
    gamma = (rows_per_wavefront + 18) * 2.0 ** -24 + (3 * 2.0 ** -18 if pieces == 2 else 2.0 ** -23)
    return (1e-5 + gamma) * Sn + 1e-6 * dz_abs_colsum[None, :] + floor, gamma * Ss + floor
