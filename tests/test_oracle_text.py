"""Pins of the text-prefix borders (Section 4.1.1: T-T, T-V and V-T stay dense
around the sparse V-V pattern) in the oracle: an element-wise definition, closed
form pair counts, a library attention with an independently built mask, and a
plain-loop tile scan for the block lists."""
import math

import numpy as np
import pytest
import torch

from oracle import sparse_attention as O


def kept(mode, p, T, i, j):
    """The definition, one element at a time."""
    if i < T or j < T:
        return True
    if mode == O.MODE_VSTRIPE:
        return j in p["cols"]
    offs = (0,) if mode == O.MODE_DIAG else p["offsets"]
    return any(abs(j - i - o) <= p["half_width"] for o in offs)


CASES = [
    (O.MODE_DIAG, {"half_width": 5, "text_tokens": 8}, 40),
    (O.MODE_MULTIDIAG, {"half_width": 2, "offsets": (-16, 0, 16), "text_tokens": 8}, 56),
    (O.MODE_VSTRIPE, {"cols": (9, 20, 33), "text_tokens": 8}, 40),
    (O.MODE_VSTRIPE, {"cols": (0, 3, 20), "text_tokens": 4}, 24),      # listed text columns change nothing
]


@pytest.mark.parametrize("mode,p,L", CASES)
def test_mask_is_the_union_of_pattern_and_borders(mode, p, L):
    T = p["text_tokens"]
    rows = np.arange(L)
    got = O.allowed_mask(mode, p, L, rows)
    want = np.array([[kept(mode, p, T, i, j) for j in range(L)] for i in range(L)])
    np.testing.assert_array_equal(got, want)
    # sub-selection of rows gives the same rows
    np.testing.assert_array_equal(O.allowed_mask(mode, p, L, rows[5::7]), want[5::7])
    # without the prefix the V-V part is untouched
    bare = {k: v for k, v in p.items() if k != "text_tokens"}
    np.testing.assert_array_equal(O.allowed_mask(mode, bare, L, rows)[T:, T:], want[T:, T:])


def test_pair_counts_closed_form():
    L, T, w = 300, 32, 7
    band = lambda n, offs: sum(max(0, n - abs(d)) for d in set(d for o in offs for d in range(o - w, o + w + 1)))
    n = O.mask_popcount(O.MODE_DIAG, {"half_width": w, "text_tokens": T}, L)
    assert n == T * L + (L - T) * T + band(L - T, (0,))
    offs = (-60, 0, 60)
    n = O.mask_popcount(O.MODE_MULTIDIAG, {"half_width": w, "offsets": offs, "text_tokens": T}, L)
    assert n == T * L + (L - T) * T + band(L - T, offs)
    cols = (40, 41, 100, 299)
    n = O.mask_popcount(O.MODE_VSTRIPE, {"cols": cols, "text_tokens": T}, L)
    assert n == L * (T + len(cols)) + T * (L - T - len(cols))


def test_dense_and_skip_ignore_the_prefix_and_bad_prefixes_are_errors():
    rows = np.arange(10)
    assert O.allowed_mask(O.MODE_DENSE, {"text_tokens": 4}, 10, rows).all()
    q = np.ones((10, 4))
    assert not O.attention_head(q, q, q, O.MODE_SKIP, {"text_tokens": 4}).any()
    for T in (10, 11, -1):
        with pytest.raises(ValueError):
            O.allowed_mask(O.MODE_DIAG, {"half_width": 1, "text_tokens": T}, 10, rows)


@pytest.mark.parametrize("mode,p,L", CASES)
def test_attention_against_library_softmax_with_an_independent_mask(mode, p, L):
    rng = np.random.default_rng(3)
    d = 16
    q, k, v = (rng.standard_normal((L, d)) for _ in range(3))
    got = O.attention_head(q, k, v, mode, p)
    T = p["text_tokens"]
    m = torch.tensor([[kept(mode, p, T, i, j) for j in range(L)] for i in range(L)])
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None], attn_mask=m[None])[0].numpy()
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)
    # text rows are plain dense attention
    dense = O.attention_head(q, k, v, O.MODE_DENSE, {})
    np.testing.assert_allclose(got[:T], dense[:T], rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("mode,p", [(O.MODE_DIAG, {"half_width": 5, "text_tokens": 16}),
                                    (O.MODE_MULTIDIAG, {"half_width": 3, "offsets": (-40, 0, 40), "text_tokens": 16}),
                                    (O.MODE_DIAG, {"half_width": 0, "text_tokens": 32})])
def test_block_lists_by_plain_tile_scan(mode, p):
    L, bq, bk = 150, 16, 8
    T = p["text_tokens"]
    lists = O.block_lists(mode, p, L, bq, bk)
    runs = [tuple(r) for r in lists["runs"]]
    assert lists["row_ptr"][0] == 0
    for qb in range(-(-L // bq)):
        ent = range(lists["row_ptr"][qb], lists["row_ptr"][qb + 1])
        rows = range(qb * bq, min(L, (qb + 1) * bq))
        if rows[0] < T:
            assert len(ent) == 0
            continue
        want = []
        for kb in range(-(-L // bk)):
            cells = [(i, j) for i in rows for j in range(kb * bk, kb * bk + bk)]
            k_ = [(i, j) for (i, j) in cells if j < L and kept(mode, p, T, i, j)]
            if not k_:
                continue
            touched = sorted({r for (i, j) in k_ for r, (lo, hi) in enumerate(runs) if lo <= j - i <= hi
                              and kept(mode, {**p, "text_tokens": 0}, 0, i, j)})
            first, count = (touched[0], touched[-1] - touched[0] + 1) if touched else (0, 0)
            want.append((kb, int(len(k_) == len(cells)), first, count))
        got = [(int(lists["kv_block_idx"][e]), int(lists["flags"][e]), int(lists["run_first"][e]),
                int(lists["run_count"][e])) for e in ent]
        assert got == want, qb
        # the text tiles come first and are kept whole
        assert [g[:2] for g in got[:T // bk]] == [(kb, 1) for kb in range(T // bk)]


def test_lists_need_an_aligned_prefix_and_columns_gain_the_text():
    with pytest.raises(ValueError):
        O.block_lists(O.MODE_DIAG, {"half_width": 3, "text_tokens": 12}, 100, 16, 8)
    with pytest.raises(ValueError):
        O.block_lists(O.MODE_DIAG, {"half_width": 3, "text_tokens": 16}, 100, 16, 12)
    cl = O.column_list({"cols": (40, 3, 77), "text_tokens": 8}, 100, 16)
    assert cl.tolist() == list(range(8)) + [40, 77] + [-1] * 6
    g = O.head_groups([2, 2, 4, 4], [{"half_width": 3, "text_tokens": 16}, {"half_width": 3},
                                     {"cols": (1,), "text_tokens": 16}, {"cols": (1,), "text_tokens": 16}])
    assert g[0]["list_id"] == [0, 1] and g[1]["list_id"] == [0, 0]
