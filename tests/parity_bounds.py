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
each, before an fp32-accumulated contraction; dHidden is rounded to bf16 once more when stored.  An
element never sees more than two of these roundings, so the error of its dominant term is at most
2 * 2^-8 of the term (reached when both roundings fall at the end of their interval on the same side:
seen at 0.9 of that among the 10^7 elements of a full-size slice), and no element's terms exceed the
scale above by much (random signs: the errors of a long sum add like a random walk, far below the
sum of magnitudes).  One more 2^-8 covers the rest: the other terms of the sum and the coefficient's
own error (the ratio's, 1e-3 at most).  rel = 3 * 2^-8.  A gradient stored in bf16 (dw_dtype bf16) gets
one more rounding: rel 2^-6.
fp32 path: fp64 accumulation, fp32 storage: rel 1e-5 as for the norm.  atol = 1e-30 exempts rows
whose coefficient is so small that fp32/bf16 intermediates leave the normal range.

One more term, from the data and not from the kernels (coefficient_slack below): log-probabilities are
stored as float (the behaviour pass stores them so; the current pass rounds the same way, which is what
makes equal policies give ratios of exactly 1).  The oracle keeps its current log-probs in float64, so
a generation's log ratio s_n differs from the oracle's by ds <= L_n 2^-24 max|logp|.  That moves the
weight of every member of the group by the same relative amount, the baseline b = (1/N_k) sum w R by
at most ds b, and the coefficient g_n ~ rho_n (R_n - b) by ds (1 + b / |A_n|) relative: an advantage
that is a difference of nearly equal numbers amplifies it.  Each generation's rows get that much more.
"""
import numpy as np

REL = {"bf16": 3 * 2.0 ** -8, "f32": 1e-5}
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


def coefficient_slack(oracle_out, rewards, mask):
    """Per generation: ds (1 + b / |A_n|), the relative error its coefficient may carry because stored
    log-probs are floats (see above); 0 where the advantage is 0 (the coefficient is an exact 0).
    oracle_out: the oracle's result dict (adv, weight, logp_cur)."""
    adv = np.asarray(oracle_out["adv"], np.float64)
    R = np.asarray(rewards, np.float64)
    lengths = (np.asarray(mask) != 0).sum(axis=1)
    ds = lengths * 2.0 ** -24 * max(float(np.abs(oracle_out["logp_cur"]).max()), 1.0)
    b = np.abs(R - adv)                              # the baseline the generation's reward was compared with
    slack = np.zeros_like(adv)
    nz = adv != 0
    slack[nz] = ds[nz] + ds.max() * b[nz] / np.abs(adv[nz])     # own ratio; the group's weights in the baseline
    return slack


def token_coefficient_slack(coef_of_logp, logp_cur, mask, tokens, V):
    """The same effect for estimators whose coefficient is per token (the baselines' clipped surrogate): the
    library's current log-probs are floats, the oracle's are not, and a coefficient such as the KL term's
    beta (1 - exp(ref - cur)) is a difference of nearly equal numbers now and then.  coef_of_logp(logp) must
    return the oracle's coefficients [N,T] for current log-probs `logp`; it is evaluated at the oracle's
    log-probs and at both ends of the float rounding interval around them.  Returns (relative slack per
    token [N,T], relative slack per vocabulary column [V]): a token's rows of dHidden get the first; a
    column of dW gets the largest slack among the tokens sampled there (it is their one-hot terms that
    make up the column), and where nothing was sampled the coefficient-weighted mean."""
    lp = np.asarray(logp_cur, np.float64)
    msk = np.asarray(mask) != 0
    ulp = 2.0 ** -24 * np.maximum(np.abs(lp), 1.0) * 1.001            # half a float spacing, a little generous
    g0 = coef_of_logp(lp)
    dg = np.maximum(np.abs(coef_of_logp(lp + ulp) - g0), np.abs(coef_of_logp(lp - ulp) - g0)) * msk
    rel = np.zeros_like(g0)
    nz = (g0 != 0) & msk
    rel[nz] = dg[nz] / np.abs(g0[nz])
    mean = float(dg.sum() / max(np.abs(g0).sum(), 1e-300))
    col = np.full(V, mean)
    tok = np.asarray(tokens)
    np.maximum.at(col, tok[msk], rel[msk])
    return rel, col


def assert_dhidden_close(got, ref, dtype="bf16", rel=None):
    """got, ref: [..., d]; every element within rel of its token row's largest magnitude.  rel may be an
    array that broadcasts against the rows (one tolerance per generation: shape [N, 1, 1])."""
    worst, idx = worst_excess(got, ref, -1, REL[dtype] if rel is None else rel)
    assert worst <= 1.0, f"dHidden element {idx}: error is {worst:.2f} x its bound"
    assert np.isfinite(np.asarray(got, np.float64)).all()


def assert_dw_close(got, ref, dtype="bf16", rel=None):
    """got, ref: [d, V] (logical layout); every element within rel of its vocabulary column's largest
    magnitude.  rel may be an array over the columns (shape [V])."""
    worst, idx = worst_excess(got, ref, 0, REL[dtype] if rel is None else rel)
    assert worst <= 1.0, f"dW element {idx}: error is {worst:.2f} x its bound"
    assert np.isfinite(np.asarray(got, np.float64)).all()
