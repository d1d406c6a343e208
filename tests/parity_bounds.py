"""Element-wise bounds for the two gradient outputs, used beside the Frobenius-norm tolerance.

A norm over a whole tensor cannot see a wrong one-hot element in a few rows, a dropped vocabulary
column or a mis-scaled low-magnitude column.  Every element is therefore also held to

    |got - ref| <= rel * scale + atol,

with `scale` taken from the ORACLE's tensor: the largest magnitude in the element's token row for
dHidden (a row is g_n (W[:, y] - W p) / temperature: all its elements share the coefficient g_n), and
in the element's vocabulary column for dW (a column is sum_m g_m (1[y_m = v] - p_mv) h_m: all its
elements share the coefficients).

Where the bound comes from (bf16 path): the rows x V intermediate (dz, or the stored exponentials
and the scaled hidden rows of the cache mode) is rounded to bf16 once or twice, unit roundoff 2^-8
each, before an fp32-accumulated contraction; dHidden is rounded to bf16 once more when stored.  A
term's error is therefore at most 2 * 2^-8 = 2^-7 of the term, and no element's terms exceed the
scale above by much (random signs: the errors of a long sum add like a random walk, far below the
sum of magnitudes).  A gradient stored in bf16 (dw_dtype bf16) gets one more rounding: rel 2^-6.
fp32 path: fp64 accumulation, fp32 storage: rel 1e-5 as for the norm.  atol = 1e-30 exempts rows
whose coefficient is so small that fp32/bf16 intermediates leave the normal range.
"""
import numpy as np

REL = {"bf16": 2.0 ** -7, "f32": 1e-5}
ATOL = 1e-30


def worst_excess(got, ref, axis, rel):
    """max over elements of |got - ref| / (rel * scale + ATOL), scale = max |ref| along `axis`.
    <= 1 means every element is inside its bound.  Also returns the index of the worst element."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    scale = np.abs(ref).max(axis=axis, keepdims=True)
    ratio = np.abs(got - ref) / (rel * scale + ATOL)
    if ratio.size == 0:
        return 0.0, ()
    idx = np.unravel_index(int(np.argmax(ratio)), ratio.shape)
    return float(ratio[idx]), idx


def assert_dhidden_close(got, ref, dtype="bf16", rel=None):
    """got, ref: [..., d]; every element within rel of its token row's largest magnitude."""
    worst, idx = worst_excess(got, ref, -1, REL[dtype] if rel is None else rel)
    assert worst <= 1.0, f"dHidden element {idx}: error is {worst:.2f} x its bound"
    assert np.isfinite(np.asarray(got, np.float64)).all()


def assert_dw_close(got, ref, dtype="bf16", rel=None):
    """got, ref: [d, V] (logical layout); every element within rel of its vocabulary column's largest
    magnitude."""
    worst, idx = worst_excess(got, ref, 0, REL[dtype] if rel is None else rel)
    assert worst <= 1.0, f"dW element {idx}: error is {worst:.2f} x its bound"
    assert np.isfinite(np.asarray(got, np.float64)).all()
