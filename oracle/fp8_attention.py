"""CPU oracle of the FP8 variant of the pattern-specific sparse attention.

TEST INFRASTRUCTURE ONLY.  Imported by the tests, the smoke check and the
benchmark's CPU-baseline leg, and by nothing else; it shares no code with the
HIP library and never imports it.

What it follows in the paper
----------------------------
Appendix B (Table 4, "Sparse-vDiT + FP8") combines the sparse kernels of
Section 4.2 with FP8 quantisation.  The paper gives no recipe: neither the FP8
format, nor which operands are quantised, nor the granularity of the scales.
This oracle therefore fixes one (every choice below is a reading of this build,
not of the paper) and states it as a quantise-dequantise definition on top of Eq. 1:

* format: OCP FP8 E4M3 (4 exponent bits, bias 7, 3 mantissa bits, largest finite
  value 448, subnormals down to 2^-9, no infinities), round to nearest even,
  values beyond +-448 saturate;
* operands: Q, K, V and the probabilities P are quantised; scores, row sums and
  the output accumulate exactly (float64 here, fp32 on the GPU);
* scales: fixed powers of two, no data-dependent calibration.
      Q8 = e4m3( fp32(q) * fp32(4 * log2(e) / sqrt(d)) )      (product in fp32)
      K8 = e4m3( k / 4 ),   V8 = e4m3( v )
  so that Q8 . K8 is the score of Eq. 1 in units of log 2;
* probabilities: with s2 = Q8 . K8 over the kept keys of the row and the integer
  reference m = ceil(max s2) - 8,  P8 = e4m3( 2^(s2 - m) )  (so the largest
  probability of a row lies in (128, 256], well inside the normal range and
  below 448), and  O = (P8 V8) / sum(P8).
  An integer reference makes the rounding of P independent of the order in which
  a blocked implementation meets the keys, up to the subnormal range: moving the
  reference by an integer multiplies every P8 by an exact power of two.

Masks, modes and the zero output of M_1 are taken from the bf16 oracle's
definitions; only the arithmetic of a row differs.

Several results are correct for a row whose probabilities sit on a rounding
boundary: P8 is a rounding decision on a score that an fp32 implementation sums
in an order of its own, so a probability within the score's error bound of the
midpoint between two E4M3 values may take either neighbour.
attention_rows_fp8_alternatives states that set: per row the results of every
combination of the heaviest such decisions, plus a bound on what the lighter
ones can move.

Pins (tests/test_oracle_fp8.py): the rounding against the format's own code
table (brute-force nearest value, ties to even) and against a library
conversion; the attention against closed forms (constant V, zero Q), a
pure-Python loop over the code table, invariance under an integer shift of the
reference, and closeness to the unquantised oracle; the score-error bound against
fp32 sums taken in random orders with truncation; the set of alternatives against
a hand-worked row, against rows without any ambiguity, and against the results
of simulated implementations whose scores are off by up to the bound.  No
function here is "parity unpinned".
"""
from __future__ import annotations

import math

import numpy as np

from . import sparse_attention as SA

E4M3_MAX = 448.0
Q_PRESCALE = 4.0     # power of two moved from K to Q: Q8 carries 4*log2(e)/sqrt(d), K8 carries 1/4
P_HEADROOM = 8       # the reference sits this many binary orders below ceil(row max)


def round_e4m3(x):
    """Nearest OCP E4M3 value of every element (ties to even mantissa, saturating).

    Written from the format: a value with binade e = floor(log2|x|), clipped below
    at the smallest normal exponent -6, is a multiple of the spacing 2^(e-3).
    """
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), E4M3_MAX)
    e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    e = np.maximum(e, -6.0)
    step = np.exp2(e - 3.0)
    q = np.rint(a / step) * step          # rint: ties to even; a/step is exact (power of two)
    return np.copysign(q, x)


def rounding_margin(x):
    """Relative distance of every element to the nearest point where round_e4m3
    changes its result (the midpoint between two neighbouring E4M3 values);
    infinite for zero.  A blocked fp32 implementation whose value differs from
    the exact one by less than this margin takes the same rounding decision."""
    a = np.minimum(np.abs(np.asarray(x, dtype=np.float64)), E4M3_MAX)
    e = np.maximum(np.floor(np.log2(np.where(a > 0, a, 1.0))), -6.0)
    units = a / np.exp2(e - 3.0)          # in [8, 16) for normal numbers, [0, 8) for subnormal ones
    lo = np.floor(units)
    up = lo + 0.5                          # midpoint towards the next value
    # midpoint towards the previous value: the spacing halves below the bottom of a normal binade
    down = np.where((lo == 8.0) & (e > -6.0), 7.75, lo - 0.5)
    with np.errstate(divide="ignore", invalid="ignore"):
        m = np.minimum(np.abs(up - units), units - down) / units
    return np.where(a > 0, m, np.inf)


def quantise_q(q):
    """Q8 of the header: the score scale and log2(e) are folded in before rounding."""
    d = q.shape[-1]
    c = np.float32(Q_PRESCALE * math.log2(math.e) / math.sqrt(d))
    return round_e4m3((np.asarray(q, dtype=np.float32) * c).astype(np.float64))


def quantise_k(k):
    return round_e4m3(np.asarray(k, dtype=np.float64) / Q_PRESCALE)


def quantise_v(v):
    return round_e4m3(np.asarray(v, dtype=np.float64))


def attention_rows_fp8(q8_rows, k8, v8, mask, shift=0):
    """The quantised row arithmetic of the header for operands already in E4M3.

    q8_rows [R, D], k8 [L, D], v8 [L, D] float64 holding E4M3 values, mask [R, L].
    shift: integer added to the reference (0 in the definition; the tests use it
    to show that the result does not depend on it).
    """
    if not mask.any(axis=1).all():
        raise ValueError("a query row keeps no key")
    s2 = q8_rows @ k8.T
    s2[~mask] = -np.inf
    m = np.ceil(s2.max(axis=1, keepdims=True)) - P_HEADROOM + int(shift)
    p8 = round_e4m3(np.exp2(s2 - m))
    return (p8 @ v8) / p8.sum(axis=1, keepdims=True)


def score_error_bound(q8_rows, k8):
    """Bound on |s2 of an fp32 implementation - exact s2|, per (row, key).

    A product of two E4M3 values has an 8-bit significand and is exact in fp32.
    Summing the d products of a score in fp32, in any order and with rounding or
    truncation at every step, commits at most 2 units in the last place
    (2 * 2^-24 relative) on a partial sum that never exceeds sum_d |q8 k8| in
    magnitude, d times at most: |error| <= d * 2^-23 * sum_d |q8_d k8_d|.
    A matrix unit that aligns the products of a step to the largest one keeps to
    this bound as long as it carries 24 bits below that one.
    """
    d = q8_rows.shape[-1]
    return d * 2.0 ** -23 * (np.abs(q8_rows) @ np.abs(k8).T)


EXP2_REL_ERR = 2.0 ** -21    # relative error granted to the implementation's exp2 (a few fp32 ulp)
MAX_FLIPS = 6                # rounding decisions enumerated per row (2^6 candidate results)


def attention_rows_fp8_alternatives(q8_rows, k8, v8, mask, max_flips=MAX_FLIPS):
    """The set of correct results of attention_rows_fp8, row by row.

    A probability p = 2^(s2 - m) is AMBIGUOUS when the relative distance of p to a
    midpoint between two E4M3 values is at most log(2) * score_error_bound +
    EXP2_REL_ERR: an fp32 implementation may then round it to either neighbour.
    Returns (out, candidates, slack):
      out         [R, D]  the nominal result (every decision taken on the exact score);
      candidates  list of R arrays [n_r, D]: the results for every combination of the
                  max_flips ambiguous probabilities with the largest |change of P8|
                  (n_r = 2^k, row 0 = the nominal result; n_r = 1 without ambiguity);
      slack       [R, D]  element-wise bound on what flipping any subset of the
                  remaining (lighter) ambiguous probabilities moves a candidate by.
    A result is correct iff it lies within slack (plus the accumulation error of
    the implementation) of one of the row's candidates.
    """
    if not mask.any(axis=1).all():
        raise ValueError("a query row keeps no key")
    s2 = q8_rows @ k8.T
    s2[~mask] = -np.inf
    m = np.ceil(s2.max(axis=1, keepdims=True)) - P_HEADROOM
    p = np.exp2(s2 - m)
    p8 = round_e4m3(p)
    den = p8.sum(axis=1)
    num = p8 @ v8
    out = num / den[:, None]
    rel = math.log(2.0) * score_error_bound(q8_rows, k8) + EXP2_REL_ERR
    ambiguous = mask & (rounding_margin(p) <= rel)
    candidates = [out[r:r + 1] for r in range(out.shape[0])]
    slack = np.zeros_like(out)
    for r in np.nonzero(ambiguous.any(axis=1))[0]:
        j = np.nonzero(ambiguous[r])[0]
        pj, ej = p[r, j], rel[r, j]
        up, down = round_e4m3(pj * (1.0 + 2.0 * ej)), round_e4m3(pj * (1.0 - 2.0 * ej))   # the two neighbours
        other = np.where(up != p8[r, j], up, down)
        dp = other - p8[r, j]
        keep = dp != 0
        j, dp = j[keep], dp[keep]
        order = np.argsort(-np.abs(dp), kind="stable")
        j, dp = j[order], dp[order]
        top_j, top_dp = j[:max_flips], dp[:max_flips]
        k_top = top_j.size
        bits = (np.arange(1 << k_top)[:, None] >> np.arange(k_top)[None, :]) & 1      # [2^k, k], row 0 = no flip
        num_c = num[r][None, :] + (bits * top_dp[None, :]) @ v8[top_j]
        den_c = den[r] + bits @ top_dp
        cand = num_c / den_c[:, None]
        candidates[r] = cand
        rest_j, rest_dp = j[max_flips:], np.abs(dp[max_flips:])
        if rest_j.size:
            reach = np.abs(v8[rest_j]) + np.abs(cand).max(axis=0)[None, :]
            slack[r] = (rest_dp[:, None] * reach).sum(axis=0) / (den_c.min() - rest_dp.sum())
    return out, candidates, slack


def attention_head_fp8_alternatives(q, k, v, mode, params, rows=None, chunk=128):
    """attention_rows_fp8_alternatives for one head (all rows or the given rows): (out, candidates, slack)."""
    L, d = q.shape
    rows = np.arange(L, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.zeros((rows.size, d), dtype=np.float64)
    slack = np.zeros_like(out)
    candidates = [out[r:r + 1] for r in range(rows.size)]
    if mode != SA.MODE_SKIP:
        q8, k8, v8 = quantise_q(q), quantise_k(k), quantise_v(v)
        for s in range(0, rows.size, chunk):
            r = rows[s:s + chunk]
            o, c, sl = attention_rows_fp8_alternatives(q8[r], k8, v8, SA.allowed_mask(mode, params, L, r))
            out[s:s + chunk], slack[s:s + chunk] = o, sl
            candidates[s:s + chunk] = c
    return out, candidates, slack


def attention_head_fp8(q, k, v, mode, params, rows=None, chunk=128):
    """One head in the FP8 variant, all rows or the given rows.  q, k, v: [L, D]."""
    L, d = q.shape
    rows = np.arange(L, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.zeros((rows.size, d), dtype=np.float64)
    if mode != SA.MODE_SKIP:
        q8, k8, v8 = quantise_q(q), quantise_k(k), quantise_v(v)
        for s in range(0, rows.size, chunk):
            r = rows[s:s + chunk]
            out[s:s + chunk] = attention_rows_fp8(q8[r], k8, v8, SA.allowed_mask(mode, params, L, r))
    return out
