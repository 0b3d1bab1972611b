"""Which FP8 attention outputs count as correct: the accepted set around the oracle's result.

Test code, NumPy only.  Everything here is computed from the ORACLE's own intermediate quantities
(the `parts` of fps_oracle.attention) and two stated constants of the hardware's arithmetic; nothing
the GPU reports enters it.

Why a set and not a point.  P is rounded to E4M3 (Sec. 3.2, fixed scale 1/448): a score that moves
by one part in 10^4 can carry 448 p across a rounding boundary and change that P element by a whole
grid step (6-12 %).  An implementation that evaluates Eq. 3 on FP8 matrix hardware does not
reproduce the exact dot products: the gfx950 instruction adds the 128 products in groups, aligned
to each group's largest exponent, and drops the bits about 13 places below it.  What is known about
its result is the bound

    |S_hw - S_exact| <= ACC_EPS * sum_c |q_c k_c|            (raw code products, before scaling)

which the GPU tests assert on the kernel's own accumulators, pair by pair, against the oracle's
exact products.  Given only that bound, every score lies in an interval around the oracle's value,
and so does every 448 p; wherever a rounding boundary falls inside the interval both neighbouring
codes are correct results.  `fp8_slack` turns that into a per-output bound: how far a correct
output can lie from the oracle's.  An element whose interval contains no boundary contributes
nothing, whatever the kernel did with it.
"""
import numpy as np

from oracle import e4m3

# Accumulation accuracy of the E4M3 matrix instruction relative to sum_c |q_c k_c|.  Measured on the
# box: the error is symmetric around zero, about 2^-16.5 of that sum on average, and its largest
# values follow the largest single product of the row (up to 5.5 * 2^-13 of it: an outlier-channel
# product beside 127 small ones), which on Gaussian data with x8 outlier channels reaches
# 1.5 * 2^-12 of the sum.  The GPU tests assert the bound below on every tile they compare.
ACC_EPS = 2.0 ** -11
# The kernel evaluates 448 * 2^(S' - m) in float32: the product of three scales, one fma and the
# hardware exponential.  Exponent error <= |S'| * EXP_ABS (scale product and fma roundings), and a
# relative error EXP_REL on the result (v_exp_f32 is accurate to about one ulp).
EXP_ABS = 2.0 ** -22
EXP_REL = 2.0 ** -20
SUB_SPACING = 2.0 ** -9          # E4M3 spacing below 2^-6
MIN_NORMAL = 2.0 ** -6


def score_halfwidth(part, acc_eps=ACC_EPS):
    """Half-width, in the base-2 score units of S', of the interval a hardware score lies in."""
    return acc_eps * part["absraw"] * part["pair_scale"]


def fp8_slack(part, ref_rows, acc_eps=ACC_EPS, exp_abs=EXP_ABS, exp_rel=EXP_REL, pv_eps=None):
    """Per output element of one query tile: the largest distance from the oracle's output
    `ref_rows` that a result can have when every score is only known to lie within the hardware's
    accumulation bound of the oracle's exact score.  Returns (slack [TS, d], stats dict,
    may_differ [TS, keys]: the P elements for which more than one value is acceptable).

    Terms.  (a) P codes: y = 448 p lies in [y_lo, y_hi]; rounding is monotone, so the codes a
    correct implementation may produce are those between round(y_lo) and round(y_hi).  (b) An
    online kernel rounds an element against the row reference it has when the element's key tile
    arrives, which may be lower than the final one: for values that end below the format's normal
    range that is a finer grid than the oracle's.  (c) If the row maximum's interval reaches past
    the integer the oracle's reference is snapped to, the kernel's reference may be one higher,
    which doubles the grid spacing of the smallest values.  (d) The denominator sums the unrounded
    weights, each inside its interval.  (e) The PV product runs on the same matrix instruction and
    carries the same relative accumulation bound.
    """
    fmax = e4m3.FP8_MAX
    pv_eps = acc_eps if pv_eps is None else pv_eps
    delta = score_halfwidth(part, acc_eps) + np.abs(part["S"]) * exp_abs
    grow = np.exp2(delta) * (1.0 + exp_rel)
    y = fmax * part["p"]
    yq = fmax * part["ph"]
    y_hi_open = y * grow                                     # not clipped: used for the denominator
    y_hi = np.minimum(y_hi_open, fmax)                       # within one reference nothing exceeds 448
    y_lo = y / grow
    r_hi = e4m3.round_to_e4m3(y_hi)
    r_lo = e4m3.round_to_e4m3(y_lo)
    d = np.maximum(np.abs(r_hi - yq), np.abs(r_lo - yq))     # (a)
    ambiguous = r_hi != r_lo
    reach = np.maximum(np.maximum(y_hi - yq, yq - y_lo), 0.0)
    # (b) a grid at least twice as fine: the rounded value is within a quarter spacing of the value
    sub = y_lo < MIN_NORMAL
    d = np.where(sub, np.maximum(d, reach + SUB_SPACING / 4), d)
    # (c) reference one higher: spacing 2^-8 in the oracle's units for everything below 2^-5
    up_rows = (part["S"] + delta).max(axis=1) > part["m"]
    sub_up = up_rows[:, None] & (y_lo < 2 * MIN_NORMAL)
    d = np.where(sub_up, np.maximum(d, reach + SUB_SPACING), d)
    may_differ = d > 0
    d /= fmax
    # (d) denominator
    l = part["l"]
    l_lo = (y_lo / fmax).sum(axis=1)
    l_hi = (y_hi_open / fmax).sum(axis=1)
    absv = np.abs(part["v"])
    slack = (d @ absv) / l_lo[:, None]
    slack += np.abs(ref_rows) * (np.maximum(l_hi - l, l - l_lo) / l_lo)[:, None]
    slack += pv_eps * ((part["ph"] + d) @ absv) / l_lo[:, None]         # (e)
    slack[~part["rows_valid"]] = 0.0
    stats = dict(p_elems=int(y.size), ambiguous=int(np.count_nonzero(ambiguous)),
                 rows_ref_may_rise=int(np.count_nonzero(up_rows & part["rows_valid"])))
    return slack, stats, may_differ


def scores_within_model(raw_hw, part, acc_eps=ACC_EPS):
    """Largest |S_hw - S_exact| / (acc_eps * sum_c |q_c k_c|) over one query tile's window (<= 1
    means every hardware score lies inside the interval fp8_slack assumes).  Where the sum of
    absolute products is zero the hardware score must be exactly zero."""
    err = np.abs(np.asarray(raw_hw, dtype=np.float64) - part["raw"])
    bound = acc_eps * part["absraw"]
    if np.any((bound == 0) & (err != 0)):
        return np.inf
    return float(np.max(err / np.maximum(bound, 1e-300)))
