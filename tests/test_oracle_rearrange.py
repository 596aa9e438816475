"""Pins of the rearrangement oracle: the index map against explicit loops, the
claims of its header, and the theorem the GPU path rests on (window attention in
position-major order = diagonal attention on rearranged tensors)."""
import numpy as np
import pytest

from oracle import rearrange as R
from oracle import sparse_attention as SA


@pytest.mark.parametrize("L,first,N,F", [(30, 0, 5, 6), (40, 4, 6, 5), (23, 3, 4, 5), (12, 0, 12, 1), (12, 0, 1, 12)])
def test_index_map_by_explicit_loops_and_bijective(L, first, N, F):
    pi = R.position_major_index(L, first, N, F)
    want = list(range(L))
    for f in range(F):
        for p in range(N):
            want[first + f * N + p] = first + p * F + f
    assert pi.tolist() == want
    assert sorted(pi.tolist()) == list(range(L))
    if F == 1 or N == 1:
        assert pi.tolist() == list(range(L))
    x = np.arange(L * 3).reshape(L, 3)
    y = R.rearrange(x, first, N, F)
    for i in range(L):
        assert (y[pi[i]] == x[i]).all()
    assert (R.rearrange(y, first, N, F, inverse=True) == x).all()


def test_bad_video_blocks_are_errors():
    for args in ((10, 0, 4, 3), (10, -1, 3, 3), (10, 0, 0, 3), (10, 2, 3, 3)):
        with pytest.raises(ValueError):
            R.position_major_index(*args)


def test_window_contains_all_nearby_positions_of_all_frames_and_does_not_wrap():
    L, first, N, F, w = 4 + 7 * 6, 4, 7, 6, 2
    W = w * F + F - 1
    m = R.window_mask(L, first, N, F, W, np.arange(L))
    for fi in range(F):
        for pi_ in range(N):
            for fj in range(F):
                for pj in range(N):
                    i, j = first + fi * N + pi_, first + fj * N + pj
                    if abs(pi_ - pj) <= w:
                        assert m[i, j]
                    if abs(pi_ - pj) > w + 1:
                        assert not m[i, j]
    # the last position of a frame and the first position of the next are far apart
    assert not m[first + 0 * N + (N - 1), first + 1 * N + 0]
    # a band on the frame-major index would keep that pair
    assert SA.allowed_mask(SA.MODE_DIAG, {"half_width": w}, L, [first + N - 1])[0, first + N]
    assert (m == m.T).all() and m.diagonal().all()


def test_pair_count_closed_form():
    # no leading tokens: the mask is a plain band of half width W in the rearranged order
    L, N, F, W = 60, 10, 6, 9
    m = R.window_mask(L, 0, N, F, W, np.arange(L))
    assert int(m.sum()) == sum(L - abs(d) for d in range(-W, W + 1))


@pytest.mark.parametrize("first,N,F,W", [(0, 8, 5, 7), (6, 7, 4, 9), (3, 5, 6, 0)])
def test_equals_diagonal_attention_on_rearranged_tensors(first, N, F, W):
    L, d = first + N * F + 2, 8
    rng = np.random.default_rng(11)
    q, k, v = (rng.standard_normal((L, d)) for _ in range(3))
    direct = R.attention_head_rearranged(q, k, v, first, N, F, W)
    qp, kp, vp = (R.rearrange(x, first, N, F) for x in (q, k, v))
    band = SA.attention_head(qp, kp, vp, SA.MODE_DIAG, {"half_width": W})
    np.testing.assert_allclose(R.rearrange(band, first, N, F, inverse=True), direct, rtol=1e-12, atol=1e-14)
    # and on sampled rows
    rows = [0, first, L - 1, first + N]
    np.testing.assert_allclose(R.attention_head_rearranged(q, k, v, first, N, F, W, rows=rows), direct[rows],
                               rtol=1e-12, atol=1e-14)


def test_rearranged_multi_diagonal_head_in_the_attention_oracle():
    L, first, N, F, W = 70, 6, 8, 7, 9
    p = {"half_width": W, "rearranged": (first, N, F), "offsets": ()}
    rows = np.arange(L)
    np.testing.assert_array_equal(SA.allowed_mask(SA.MODE_MULTIDIAG, p, L, rows), R.window_mask(L, first, N, F, W, rows))
    rng = np.random.default_rng(5)
    q, k, v = (rng.standard_normal((L, 8)) for _ in range(3))
    np.testing.assert_allclose(SA.attention_head(q, k, v, SA.MODE_MULTIDIAG, p),
                               R.attention_head_rearranged(q, k, v, first, N, F, W), rtol=1e-13, atol=1e-15)
    # its lists are those of the plain band in the rearranged order; row_map inverts the index map
    lists = SA.block_lists(SA.MODE_MULTIDIAG, p, L, 16, 8)
    band = SA.block_lists(SA.MODE_DIAG, {"half_width": W}, L, 16, 8)
    for key in ("row_ptr", "kv_block_idx", "flags", "run_first", "run_count", "runs"):
        np.testing.assert_array_equal(lists[key], band[key])
    pi = SA.position_major_index(L, first, N, F)
    rm = lists["row_map"]
    assert rm.size == 72 and rm.dtype == np.int32 and (rm[L:] == -1).all()
    assert all(rm[pi[i]] == i for i in range(L))
    with pytest.raises(ValueError):
        SA.allowed_mask(SA.MODE_MULTIDIAG, dict(p, text_tokens=8), L, rows)
    with pytest.raises(ValueError):
        SA.block_lists(SA.MODE_MULTIDIAG, dict(p, rearranged=(first, N, 9)), L, 16, 8)


def test_rearranged_heads_form_their_own_group():
    table = [3, 3, 2, 3, 3]
    plain = {"half_width": 2, "offsets": (0, 10)}
    re1 = {"half_width": 5, "rearranged": (0, 10, 4)}
    re2 = {"half_width": 6, "rearranged": (0, 10, 4)}
    g = SA.head_groups(table, [plain, re1, {"half_width": 3}, re2, re1])
    assert [(x["mode"], x["heads"], x["list_id"], x["rearranged"]) for x in g] == \
        [(2, [2], [0], False), (3, [0], [0], False), (3, [1, 3, 4], [0, 1, 0], True)]
