"""Pins of the FP8 oracle against things other than itself: the E4M3 code table
written out from the format, a library conversion, closed forms, a pure-Python
loop, the shift invariance its header claims, and the unquantised oracle."""
import math

import numpy as np
import pytest
import torch

from oracle import fp8_attention as F8
from oracle import sparse_attention as SA


def e4m3_table():
    """All finite non-negative E4M3 values from the bit fields: sign 1, exponent 4
    (bias 7), mantissa 3; exponent 0 is subnormal; 0x7f is NaN."""
    vals = []
    for code in range(0x7f):
        e, m = code >> 3, code & 7
        vals.append(m / 8 * 2.0 ** -6 if e == 0 else (1 + m / 8) * 2.0 ** (e - 7))
    return np.array(vals)


def nearest_in_table(x, table):
    """Brute force: nearest table value, ties to the even code, saturating."""
    a = min(abs(x), table[-1])
    d = np.abs(table - a)
    best = np.flatnonzero(d == d.min())
    code = best[0] if len(best) == 1 else [c for c in best if c % 2 == 0][0]
    return math.copysign(table[code], x)


def test_table_has_the_formats_landmarks():
    t = e4m3_table()
    assert t[-1] == 448.0 and t[1] == 2.0 ** -9 and t[8] == 2.0 ** -6 and t[0x38] == 1.0
    assert (np.diff(t) > 0).all()


def test_rounding_matches_brute_force_over_the_code_table():
    t = e4m3_table()
    rng = np.random.default_rng(0)
    x = np.concatenate([
        rng.standard_normal(2000), rng.standard_normal(2000) * 0.01, rng.standard_normal(500) * 300,
        t, -t, (t[1:] + t[:-1]) / 2,                     # every value and every midpoint
        (t[1:] + t[:-1]) / 2 * (1 + 1e-12), (t[1:] + t[:-1]) / 2 * (1 - 1e-12),
        [0.0, 1e-9, 2.0 ** -10, 2.0 ** -10 * 1.0001, 448.0, 449.0, 1e6, -1e6]])
    want = np.array([nearest_in_table(v, t) for v in x])
    np.testing.assert_array_equal(F8.round_e4m3(x), want)


def test_rounding_matches_library_conversion():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(20000) * s for s in (1e-3, 0.05, 1.0, 40.0)]).astype(np.float32)
    x = x[np.abs(x) <= 448]
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).to(torch.float64).numpy()
    np.testing.assert_array_equal(F8.round_e4m3(x.astype(np.float64)), lib)


def test_rounding_is_idempotent_and_odd():
    rng = np.random.default_rng(2)
    x = rng.standard_normal(5000) * 10
    r = F8.round_e4m3(x)
    np.testing.assert_array_equal(F8.round_e4m3(r), r)
    np.testing.assert_array_equal(F8.round_e4m3(-x), -r)


def test_rounding_margin_is_the_distance_to_a_change_of_the_result():
    rng = np.random.default_rng(8)
    x = np.abs(rng.standard_normal(4000)) * np.exp2(rng.integers(-8, 8, 4000))
    x = x[(x > 2.0 ** -9) & (x < 440)]
    m = F8.rounding_margin(x)
    r = F8.round_e4m3(x)
    # inside the margin nothing changes, just beyond it (on one side) the result does
    np.testing.assert_array_equal(F8.round_e4m3(x * (1 + 0.999 * m)), r)
    np.testing.assert_array_equal(F8.round_e4m3(x * (1 - 0.999 * m)), r)
    moved = (F8.round_e4m3(x * (1 + 1.001 * m)) != r) | (F8.round_e4m3(x * (1 - 1.001 * m)) != r)
    assert moved.all()
    assert F8.rounding_margin(np.array([0.0]))[0] == np.inf


def test_operand_scales():
    rng = np.random.default_rng(3)
    d = 64
    q = rng.standard_normal((5, d))
    # representable inputs stay what they are up to the stated scale
    k = F8.round_e4m3(rng.standard_normal((7, d))) * 4
    np.testing.assert_array_equal(F8.quantise_k(k), k / 4)
    v = F8.round_e4m3(rng.standard_normal((7, d)))
    np.testing.assert_array_equal(F8.quantise_v(v), v)
    # Q8 . K8 approximates the Eq. 1 score in units of log 2
    k1 = rng.standard_normal((7, d))
    s_exact = (q @ k1.T) / math.sqrt(d) * math.log2(math.e)
    s_q = F8.quantise_q(q) @ F8.quantise_k(k1).T
    assert np.abs(s_q - s_exact).max() < 0.2
    assert np.abs(s_exact).max() > 2


def test_constant_v_and_zero_q_closed_forms():
    rng = np.random.default_rng(4)
    L, d = 96, 32
    q, k = rng.standard_normal((L, d)), rng.standard_normal((L, d))
    row = F8.round_e4m3(rng.standard_normal(d))
    v = np.tile(row, (L, 1))
    params = {"half_width": 9}
    out = F8.attention_head_fp8(q, k, v, SA.MODE_DIAG, params)
    np.testing.assert_allclose(out, v, rtol=1e-14, atol=0)
    # zero queries: every kept key has probability 2^8 exactly, the output is the plain mean of V8
    v = rng.standard_normal((L, d))
    out = F8.attention_head_fp8(np.zeros((L, d)), k, v, SA.MODE_DIAG, params)
    v8 = F8.quantise_v(v)
    for i in (0, 5, 50, 95):
        lo, hi = max(0, i - 9), min(L, i + 10)
        np.testing.assert_allclose(out[i], v8[lo:hi].mean(axis=0), rtol=1e-13, atol=1e-15)


def test_against_a_pure_python_loop_over_the_code_table():
    t = e4m3_table()
    rng = np.random.default_rng(5)
    L, d = 12, 8
    q, k, v = (rng.standard_normal((L, d)) for _ in range(3))
    params = {"offsets": [-4, 0, 5], "half_width": 1}
    got = F8.attention_head_fp8(q, k, v, SA.MODE_MULTIDIAG, params)
    c = np.float32(4 * math.log2(math.e) / math.sqrt(d))
    for i in range(L):
        kept = [j for j in range(L) if any(abs(j - i - o) <= 1 for o in params["offsets"])]
        q8 = [nearest_in_table(float(np.float32(q[i, x]) * c), t) for x in range(d)]
        s = {}
        for j in kept:
            s[j] = sum(q8[x] * nearest_in_table(k[j, x] / 4, t) for x in range(d))
        m = math.ceil(max(s.values())) - 8
        p = {j: nearest_in_table(2.0 ** (s[j] - m), t) for j in kept}
        den = sum(p.values())
        for x in range(d):
            want = sum(p[j] * nearest_in_table(v[j, x], t) for j in kept) / den
            assert abs(got[i, x] - want) <= 1e-12 * max(1.0, abs(want))


def test_integer_shift_of_the_reference_changes_nothing_in_the_normal_range():
    rng = np.random.default_rng(6)
    L, d = 64, 32
    q8 = F8.quantise_q(rng.standard_normal((L, d)))
    k8 = F8.quantise_k(rng.standard_normal((L, d)))
    v8 = F8.quantise_v(rng.standard_normal((L, d)))
    mask = np.ones((L, L), dtype=bool)
    base = F8.attention_rows_fp8(q8, k8, v8, mask)
    s2 = q8 @ k8.T
    spread = (np.ceil(s2.max(axis=1)) - s2.min(axis=1)).max()
    assert spread < 8 + 6 - 3          # every P stays a normal number under the shifts below
    for shift in (1, 2, 3):           # a higher reference: what the final one is to a block met earlier
        np.testing.assert_allclose(F8.attention_rows_fp8(q8, k8, v8, mask, shift=shift), base, rtol=1e-13, atol=1e-15)
    # with a long tail in the subnormal range the dependence stays far below the parity tolerance
    q8 = F8.quantise_q(rng.standard_normal((L, d)) * 4)
    wide = F8.attention_rows_fp8(q8, k8, v8, mask)
    assert np.abs(F8.attention_rows_fp8(q8, k8, v8, mask, shift=2) - wide).max() < 2e-3


@pytest.mark.parametrize("mode,params", [
    (SA.MODE_DENSE, {}),
    (SA.MODE_DIAG, {"half_width": 40}),
    (SA.MODE_MULTIDIAG, {"offsets": [-100, 0, 100], "half_width": 12}),
    (SA.MODE_VSTRIPE, {"cols": list(range(3, 300, 7))}),
    (SA.MODE_SKIP, {}),
])
def test_close_to_the_unquantised_oracle(mode, params):
    rng = np.random.default_rng(7)
    L, d = 300, 64
    q, k, v = (rng.standard_normal((L, d)) for _ in range(3))
    want = SA.attention_head(q, k, v, mode, params)
    got = F8.attention_head_fp8(q, k, v, mode, params)
    if mode == SA.MODE_SKIP:
        assert not got.any()
        return
    rel = np.sqrt(((got - want) ** 2).sum() / (want ** 2).sum())
    assert rel < 0.08, rel      # E4M3 carries 4 significant bits: a few percent is the expected level
    # and a wrong mask, a transposed operand or a dropped scale would give an error of order one
    assert rel > 1e-4


# ---- the set of correct results (attention_rows_fp8_alternatives) ----

def test_score_error_bound_covers_fp32_sums_in_any_order():
    """fp32 sums of the d exact products, in random orders, rounded or truncated at every step, stay inside the bound."""
    rng = np.random.default_rng(5)
    for d in (64, 128):
        q8 = F8.quantise_q(rng.standard_normal((16, d)) * 2.0)
        k8 = F8.quantise_k(rng.standard_normal((40, d)) * 2.0)
        bound = F8.score_error_bound(q8, k8)
        exact = q8 @ k8.T
        assert (bound > 0).all() and bound.max() < 1e-3
        for trial in range(6):
            perm = rng.permutation(d)
            acc = np.zeros((16, 40), dtype=np.float32)
            for t in perm:
                term = (q8[:, t:t + 1] * k8[None, :, t]).astype(np.float32)          # exact in fp32
                wide = acc.astype(np.float64) + term.astype(np.float64)
                if trial % 2:                                                       # truncation towards zero
                    r = wide.astype(np.float32)
                    away = np.abs(r.astype(np.float64)) > np.abs(wide)
                    r = np.where(away, np.nextafter(r, np.float32(0)), r).astype(np.float32)
                    acc = r
                else:
                    acc = wide.astype(np.float32)
            assert (np.abs(acc.astype(np.float64) - exact) <= bound).all()
    # the closed form on a case worked by hand: d = 64 terms of 0.5 * 0.25
    one = F8.score_error_bound(np.full((1, 64), 0.5), np.full((1, 64), 0.25))
    assert one[0, 0] == 64 * 2.0 ** -23 * 8.0


def test_alternatives_of_a_hand_worked_row():
    """Two keys.  Key 0 carries the row maximum 0 (P = 256 exactly), key 1 a score that puts P one part in 10^6
    below 11.5, the midpoint of the E4M3 neighbours 11 and 12: the nominal rounding is 11, the alternative 12."""
    d = 64
    target = math.log2(11.5 * (1.0 - 1e-5)) - 8.0        # score of key 1 relative to the reference -8
    # the score is spelt out over eight coordinates of falling weight (2^-9 is the smallest E4M3 value), each
    # taking the E4M3 value nearest to what is left
    q8 = np.zeros((1, d))
    k8 = np.zeros((2, d))
    rest = target
    for c, weight in enumerate([1.0, 2.0 ** -3, 2.0 ** -6] + [2.0 ** -9] * 5):
        q8[0, c] = weight
        k8[1, c] = F8.round_e4m3(np.array([rest / weight]))[0]
        rest -= k8[1, c] * weight
    assert np.array_equal(F8.round_e4m3(q8), q8) and abs(rest) < 3e-6
    s = float(q8[0] @ k8[1])
    p = 2.0 ** (s + 8.0)
    assert 2e-6 < 1.0 - p / 11.5 < 2e-5, p               # on the low side of the midpoint, inside the error bound
    v8 = np.array([[1.0] + [0.0] * (d - 1), [-2.0] + [0.5] * (d - 1)])
    mask = np.ones((1, 2), dtype=bool)
    out, cands, slack = F8.attention_rows_fp8_alternatives(q8, k8, v8, mask)
    assert np.array_equal(out, F8.attention_rows_fp8(q8, k8, v8, mask))
    assert cands[0].shape == (2, d) and not slack.any()
    want_nominal = (256.0 * v8[0] + 11.0 * v8[1]) / 267.0
    want_other = (256.0 * v8[0] + 12.0 * v8[1]) / 268.0
    assert np.allclose(cands[0][0], want_nominal, rtol=0, atol=1e-15)
    assert np.allclose(cands[0][1], want_other, rtol=0, atol=1e-15)


def test_no_alternatives_without_a_rounding_boundary_in_reach():
    """Zero queries: every score is 0, every P is 256 exactly, nothing is ambiguous."""
    rng = np.random.default_rng(6)
    k8, v8 = F8.quantise_k(rng.standard_normal((50, 64))), F8.quantise_v(rng.standard_normal((50, 64)))
    mask = rng.random((7, 50)) < 0.5
    mask[:, 0] = True
    out, cands, slack = F8.attention_rows_fp8_alternatives(np.zeros((7, 64)), k8, v8, mask)
    assert all(c.shape[0] == 1 for c in cands) and not slack.any()
    assert np.array_equal(np.concatenate(cands), out)


@pytest.mark.parametrize("d,max_flips", [(64, 6), (128, 6), (128, 1), (128, 0)])
def test_alternatives_cover_every_result_within_the_score_error(d, max_flips):
    """Simulated implementations: the exact scores moved by up to the bound (random, and all to one side), then
    the definition's own rounding.  Every such result lies within the row's slack of one of its candidates -
    also when few or no decisions are enumerated and the rest goes to the slack."""
    rng = np.random.default_rng(7 + d)
    L, R = 3000, 96
    q8 = F8.quantise_q(rng.standard_normal((R, d)))
    k8, v8 = F8.quantise_k(rng.standard_normal((L, d))), F8.quantise_v(rng.standard_normal((L, d)))
    mask = np.ones((R, L), dtype=bool)
    out, cands, slack = F8.attention_rows_fp8_alternatives(q8, k8, v8, mask, max_flips=max_flips)
    assert sum(c.shape[0] > 1 for c in cands) >= (R // 4 if max_flips else 0)      # the case is not empty
    bound = F8.score_error_bound(q8, k8)
    s2 = q8 @ k8.T
    m = np.ceil(s2.max(axis=1, keepdims=True)) - F8.P_HEADROOM
    flipped_rows = 0
    for trial in range(8):
        err = {0: bound, 1: -bound}.get(trial, bound * rng.uniform(-1.0, 1.0, size=bound.shape))
        p8 = F8.round_e4m3(np.exp2(s2 + err - m))
        got = (p8 @ v8) / p8.sum(axis=1, keepdims=True)
        for r in range(R):
            over = np.abs(got[r][None, :] - cands[r]) - slack[r][None, :]
            assert over.max(axis=1).min() <= 1e-12, (trial, r, over.max(axis=1).min())
        flipped_rows += int((np.abs(got - out).max(axis=1) > 1e-12).sum())
    assert flipped_rows > R                                                         # the simulated errors do flip decisions
