"""Pins of the CPU oracle's attention values against things other than itself.

Each pin names what fixes the expected value: a library routine (torch's
scaled_dot_product_attention with an explicit mask), a pure-Python triple loop
written straight from Eq. 1, or a closed form that holds for any mask.
"""
import math

import numpy as np
import pytest
import torch

from oracle import sparse_attention as O
from paper_2506_03065_amd import workloads as W


def _np(t):
    return t.to(torch.float64).numpy()


def _brute_mask(mode, p, L, i, j):
    if mode == O.MODE_DENSE:
        return True
    if mode == O.MODE_DIAG:
        return abs(i - j) <= p["half_width"]
    if mode == O.MODE_MULTIDIAG:
        return any(abs(j - i - o) <= p["half_width"] for o in p["offsets"])
    if mode == O.MODE_VSTRIPE:
        return j in set(p["cols"])
    raise AssertionError


def _brute_attention(q, k, v, mode, p):
    """Eq. 1 restricted to the kept keys, one scalar at a time."""
    L, D = q.shape
    out = [[0.0] * D for _ in range(L)]
    if mode == O.MODE_SKIP:
        return np.asarray(out)
    for i in range(L):
        keep = [j for j in range(L) if _brute_mask(mode, p, L, i, j)]
        s = [sum(float(q[i, d]) * float(k[j, d]) for d in range(D)) / math.sqrt(D) for j in keep]
        m = max(s)
        e = [math.exp(x - m) for x in s]
        z = sum(e)
        for d in range(D):
            out[i][d] = sum(e[t] * float(v[keep[t], d]) for t in range(len(keep))) / z
    return np.asarray(out)


CASES = [
    (O.MODE_DENSE, {}),
    (O.MODE_SKIP, {}),
    (O.MODE_DIAG, {"half_width": 3}),
    (O.MODE_DIAG, {"half_width": 0}),            # only the diagonal itself
    (O.MODE_DIAG, {"half_width": 100}),          # wider than the sequence
    (O.MODE_MULTIDIAG, {"half_width": 1, "offsets": (-8, 0, 8)}),
    (O.MODE_MULTIDIAG, {"half_width": 2, "offsets": (0, 5, -70, 70)}),  # bands outside [-L, L]
    (O.MODE_MULTIDIAG, {"half_width": 3, "offsets": (0, 4, -4)}),       # overlapping bands
    (O.MODE_MULTIDIAG, {"half_width": 1, "offsets": (0, 3)}),           # asymmetric: pins the sign
    (O.MODE_VSTRIPE, {"cols": (5,)}),
    (O.MODE_VSTRIPE, {"cols": (0, 7, 8, 23)}),
]


@pytest.mark.parametrize("mode,p", CASES)
def test_brute_force_triple_loop(mode, p):
    rng = np.random.default_rng(3)
    L, D = 24, 4
    q, k, v = (rng.standard_normal((L, D)) for _ in range(3))
    want = _brute_attention(q, k, v, mode, p)
    got = O.attention_head(q, k, v, mode, p, chunk=7)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_sign_of_offsets_matters_and_is_j_minus_i():
    """A single band at offset +3 keeps j = i + 3 (a key after the query)."""
    m = O.allowed_mask(O.MODE_MULTIDIAG, {"half_width": 0, "offsets": (3,)}, 8, np.arange(5))
    want = np.zeros((5, 8), dtype=bool)
    for i in range(5):
        want[i, i + 3] = True
    assert (m == want).all()


@pytest.mark.parametrize("wl", [W.tiny(), W.small(L=333, D=64), W.small(L=200, D=128, seed=11)],
                         ids=lambda w: w.name)
def test_library_sdpa_with_explicit_mask(wl):
    """Eq. 1 is textbook softmax attention: torch's CPU routine in float64, given
    a mask built here with torch index arithmetic, must agree."""
    q, k, v = W.make_qkv(wl)
    got = O.attention_layer(_np(q), _np(k), _np(v), wl.strategy_table, wl.pattern_params)
    i = torch.arange(wl.L)[:, None]
    j = torch.arange(wl.L)[None, :]
    for h in range(wl.H):
        mode, p = int(wl.strategy_table[h]), wl.pattern_params[h]
        if mode == W.SKIP:
            assert not got[0, h].any()
            continue
        if mode == W.DENSE:
            mask = torch.ones(wl.L, wl.L, dtype=torch.bool)
        elif mode in (W.DIAG, W.MULTIDIAG):
            mask = torch.zeros(wl.L, wl.L, dtype=torch.bool)
            for o in p["offsets"]:
                mask |= ((j - i - o) <= p["half_width"]) & ((j - i - o) >= -p["half_width"])
        else:
            mask = torch.zeros(wl.L, wl.L, dtype=torch.bool)
            mask[:, torch.tensor(p["cols"])] = True
        want = torch.nn.functional.scaled_dot_product_attention(
            q[0, h].double()[None], k[0, h].double()[None], v[0, h].double()[None], attn_mask=mask[None])
        np.testing.assert_allclose(got[0, h], want[0].numpy(), rtol=0, atol=1e-10)


def test_full_width_patterns_equal_dense():
    rng = np.random.default_rng(5)
    L, D = 97, 8
    q, k, v = (rng.standard_normal((L, D)) for _ in range(3))
    dense = O.attention_head(q, k, v, O.MODE_DENSE, {})
    wide = O.attention_head(q, k, v, O.MODE_DIAG, {"half_width": L - 1})
    multi = O.attention_head(q, k, v, O.MODE_MULTIDIAG,
                             {"half_width": 10, "offsets": tuple(range(-100, 101, 20))})
    stripes = O.attention_head(q, k, v, O.MODE_VSTRIPE, {"cols": tuple(range(L))})
    for other in (wide, multi, stripes):
        assert np.array_equal(dense, other)
    narrow = O.attention_head(q, k, v, O.MODE_DIAG, {"half_width": L - 2})
    assert not np.array_equal(dense[0], narrow[0])       # row 0 loses key L-1
    assert np.array_equal(dense[1:-1], narrow[1:-1])


def test_constant_values_give_constant_output():
    """Softmax weights over the kept keys sum to one: V == c gives O == c."""
    wl = W.small(L=150, D=64)
    q, k, _ = W.make_qkv(wl)
    v = np.full((1, wl.H, wl.L, wl.D), 0.625)
    out = O.attention_layer(_np(q), _np(k), v, wl.strategy_table, wl.pattern_params)
    for h in range(wl.H):
        want = 0.0 if wl.strategy_table[h] == W.SKIP else 0.625
        np.testing.assert_allclose(out[0, h], want, rtol=0, atol=1e-14)


def test_zero_queries_give_windowed_mean_of_values():
    """Q == 0 makes all kept scores equal, so O[i] is the mean of V over the kept
    keys of row i; for bands this is a difference of prefix sums."""
    rng = np.random.default_rng(9)
    L, D = 211, 6
    k, v = rng.standard_normal((L, D)), rng.standard_normal((L, D))
    q = np.zeros((L, D))
    prefix = np.concatenate([np.zeros((1, D)), np.cumsum(v, axis=0)])
    w = 17
    got = O.attention_head(q, k, v, O.MODE_DIAG, {"half_width": w})
    for i in range(L):
        lo, hi = max(0, i - w), min(L, i + w + 1)
        np.testing.assert_allclose(got[i], (prefix[hi] - prefix[lo]) / (hi - lo), atol=1e-12)
    offs, w = (-60, 0, 60), 5
    got = O.attention_head(q, k, v, O.MODE_MULTIDIAG, {"half_width": w, "offsets": offs})
    for i in range(L):
        tot, cnt = np.zeros(D), 0
        for o in offs:
            lo, hi = max(0, i + o - w), min(L, i + o + w + 1)
            if hi > lo:
                tot += prefix[hi] - prefix[lo]
                cnt += hi - lo
        np.testing.assert_allclose(got[i], tot / cnt, atol=1e-12)
    cols = (3, 50, 51, 200)
    got = O.attention_head(q, k, v, O.MODE_VSTRIPE, {"cols": cols})
    np.testing.assert_allclose(got, np.broadcast_to(v[list(cols)].mean(axis=0), (L, D)), atol=1e-12)


def test_structure_invariances():
    wl = W.small(L=120, D=64, H=5)
    q, k, v = (_np(t) for t in W.make_qkv(wl))
    base = O.attention_layer(q, k, v, wl.strategy_table, wl.pattern_params)
    # column order does not matter
    h = int(np.nonzero(wl.strategy_table == W.VSTRIPE)[0][0])
    shuffled = [dict(p) for p in wl.pattern_params]
    shuffled[h]["cols"] = tuple(reversed(shuffled[h]["cols"]))
    again = O.attention_layer(q, k, v, wl.strategy_table, shuffled)
    assert np.array_equal(base[0, h], again[0, h])
    # heads are independent: changing head 0's inputs and mode leaves the others alone
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[0, 0] += 1.0
    k2[0, 0] *= 2.0
    v2[0, 0] -= 3.0
    table2 = wl.strategy_table.copy()
    table2[0] = W.SKIP
    other = O.attention_layer(q2, k2, v2, table2, wl.pattern_params)
    assert np.array_equal(base[0, 1:], other[0, 1:])
    assert not other[0, 0].any()
    # permuting kept keys together with their values changes nothing (dense head)
    perm = np.random.default_rng(1).permutation(wl.L)
    a = O.attention_head(q[0, 0], k[0, 0], v[0, 0], O.MODE_DENSE, {})
    b = O.attention_head(q[0, 0], k[0, 0][perm], v[0, 0][perm], O.MODE_DENSE, {})
    np.testing.assert_allclose(a, b, atol=1e-13)
    # a sampled-row call returns exactly the rows of the full call
    rows = np.asarray([0, 5, 77, 119])
    part = O.attention_layer(q, k, v, wl.strategy_table, wl.pattern_params, rows=rows)
    assert np.array_equal(part, base[:, :, rows])


def test_rows_without_keys_and_bad_parameters_are_errors():
    q = np.zeros((16, 4))
    with pytest.raises(ValueError):
        O.attention_head(q, q, q, O.MODE_MULTIDIAG, {"half_width": 1, "offsets": (6,)})
    with pytest.raises(ValueError):
        O.attention_head(q, q, q, O.MODE_VSTRIPE, {"cols": ()})
    with pytest.raises(ValueError):
        O.attention_head(q, q, q, O.MODE_VSTRIPE, {"cols": (3, 3)})
    with pytest.raises(ValueError):
        O.attention_head(q, q, q, O.MODE_VSTRIPE, {"cols": (16,)})
    with pytest.raises(ValueError):
        O.attention_head(q, q, q, O.MODE_DIAG, {"half_width": -1})


def test_scale_is_one_over_sqrt_d():
    """Two keys, D = 4: the weight of key 0 is sigmoid((s0 - s1) / sqrt(4))."""
    q = np.asarray([[1.0, 2.0, 0.0, -1.0], [0.0, 0.0, 0.0, 0.0]])
    k = np.asarray([[0.5, 1.0, 3.0, 0.0], [-1.0, 0.25, 2.0, 2.0]])
    v = np.asarray([[1.0, 0.0, 0.0, 0.0], [0.0, 1.0, 0.0, 0.0]])
    out = O.attention_head(q, k, v, O.MODE_DENSE, {})
    s0, s1 = 2.5, -2.5
    w0 = 1.0 / (1.0 + math.exp(-(s0 - s1) / 2.0))
    np.testing.assert_allclose(out[0], [w0, 1 - w0, 0, 0], atol=1e-15)
    np.testing.assert_allclose(out[1], [0.5, 0.5, 0, 0], atol=1e-15)
