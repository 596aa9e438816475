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

Pins (tests/test_oracle_fp8.py): the rounding against the format's own code
table (brute-force nearest value, ties to even) and against a library
conversion; the attention against closed forms (constant V, zero Q), a
pure-Python loop over the code table, invariance under an integer shift of the
reference, and closeness to the unquantised oracle.  No function here is
"parity unpinned".
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


WEIGHT_FLOOR = 5e-3   # share of the row sum below which a probability is too light to matter for the margin


def attention_rows_fp8(q8_rows, k8, v8, mask, shift=0, with_margin=False):
    """The quantised row arithmetic of the header for operands already in E4M3.

    q8_rows [R, D], k8 [L, D], v8 [L, D] float64 holding E4M3 values, mask [R, L].
    shift: integer added to the reference (0 in the definition; the tests use it
    to show that the result does not depend on it).
    with_margin: also return, per row, the smallest rounding_margin of the
    probabilities that carry more than WEIGHT_FLOOR of the row's weight: how far
    the row's result is from depending on the last bits of a score.  (A lighter
    probability that rounds the other way moves the row by less than
    WEIGHT_FLOOR / 8 * |v - o|.)
    """
    if not mask.any(axis=1).all():
        raise ValueError("a query row keeps no key")
    s2 = q8_rows @ k8.T
    s2[~mask] = -np.inf
    m = np.ceil(s2.max(axis=1, keepdims=True)) - P_HEADROOM + int(shift)
    p = np.exp2(s2 - m)
    p8 = round_e4m3(p)
    den = p8.sum(axis=1, keepdims=True)
    out = (p8 @ v8) / den
    if not with_margin:
        return out
    margin = np.where(p8 > WEIGHT_FLOOR * den, rounding_margin(p), np.inf).min(axis=1)
    return out, margin


def attention_head_fp8(q, k, v, mode, params, rows=None, chunk=128, with_margin=False):
    """One head in the FP8 variant, all rows or the given rows.  q, k, v: [L, D].
    with_margin: also return the per-row margin of attention_rows_fp8."""
    L, d = q.shape
    rows = np.arange(L, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.zeros((rows.size, d), dtype=np.float64)
    margin = np.full(rows.size, np.inf)
    if mode != SA.MODE_SKIP:
        q8, k8, v8 = quantise_q(q), quantise_k(k), quantise_v(v)
        for s in range(0, rows.size, chunk):
            r = rows[s:s + chunk]
            out[s:s + chunk], margin[s:s + chunk] = attention_rows_fp8(
                q8[r], k8, v8, SA.allowed_mask(mode, params, L, r), with_margin=True)
    return (out, margin) if with_margin else out
