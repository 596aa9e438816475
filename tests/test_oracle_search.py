"""Pins of the search-step oracle (Section 4.2, Eq. 2-3, Algorithm 1) against
things other than itself: hand-worked selections, closed forms of the MSE and
of the sparsity, and special cases whose answer the definition fixes."""
import numpy as np
import pytest

from oracle import sparse_attention as A
from oracle import sparse_search as S


def test_selection_rule_hand_worked():
    # rows = modes 1..4, columns = heads; epsilon = 1
    loss = np.array([[5.0, 0.9, 2.0, 1.0],     # skip
                     [3.0, 0.5, 0.3, 1.0],     # diagonal
                     [2.0, 0.7, 0.3, 1.5],     # multi-diagonal
                     [1.1, 0.6, 4.0, 9.0]])    # vertical
    # head 0: all four above 1 -> dense.  head 1: min 0.5 -> diagonal.  head 2: tie
    # 0.3 / 0.3 -> the lower mode id (diagonal).  head 3: losses equal to epsilon are
    # not "above" it -> a sparse mode is taken, the first minimum is skip.
    assert S.select_modes(loss, 1.0).tolist() == [0, 2, 2, 1]
    # a threshold below every loss keeps every head dense; a huge one changes nothing else
    assert S.select_modes(loss, 0.2).tolist() == [0, 0, 0, 0]
    assert S.select_modes(loss, 100.0).tolist() == [4, 2, 2, 1]


def test_loss_is_mse_plus_penalty_on_kept_share():
    mse = np.array([[0.0], [0.1], [0.2], [0.3]])
    sparsity = np.array([[1.0], [0.9], [0.5], [0.0]])
    got = S.losses(mse, sparsity, 0.5)
    assert np.allclose(got[:, 0], [0.0, 0.1 + 0.05, 0.2 + 0.25, 0.3 + 0.5])
    # lambda = 0: the loss is the MSE alone (the first row of the lambda ablation)
    assert np.array_equal(S.losses(mse, sparsity, 0.0), mse)


def test_sparsity_closed_forms():
    L = 97
    assert S.head_sparsity(A.MODE_SKIP, {}, L) == 1.0
    assert S.head_sparsity(A.MODE_DENSE, {}, L) == 0.0
    w = 5      # band at offset 0: L(2w+1) - w(w+1) kept pairs
    assert np.isclose(S.head_sparsity(A.MODE_DIAG, {"half_width": w}, L), 1 - (L * (2 * w + 1) - w * (w + 1)) / L ** 2)
    cols = (3, 10, 11, 50)
    assert np.isclose(S.head_sparsity(A.MODE_VSTRIPE, {"cols": cols}, L), 1 - len(cols) / L)
    o, w = 20, 4   # one band away from the diagonal: (2w+1)(L - |o|)
    assert np.isclose(S.head_sparsity(A.MODE_MULTIDIAG, {"half_width": w, "offsets": (o,)}, L),
                      1 - (2 * w + 1) * (L - o) / L ** 2)


def test_mse_closed_forms():
    gen = np.random.default_rng(3)
    ref = gen.standard_normal((2, 3, 11, 4))
    assert np.allclose(S.head_mse(ref, ref), 0.0)
    # against zeros (the skip mode) the MSE is the mean square of the reference, per head
    want = np.array([(ref[:, h] ** 2).sum() / (2 * 11 * 4) for h in range(3)])
    assert np.allclose(S.head_mse(np.zeros_like(ref), ref), want)
    # a constant shift c gives c^2 whatever the data
    assert np.allclose(S.head_mse(ref + 0.25, ref), 0.0625)


def _layer(seed, B=1, H=3, L=48, D=8):
    gen = np.random.default_rng(seed)
    q, k, v = (gen.standard_normal((B, H, L, D)) for _ in range(3))
    params = {A.MODE_DIAG: [{"half_width": 6}] * H,
              A.MODE_MULTIDIAG: [{"half_width": 2, "offsets": (-16, 0, 16)}] * H,
              A.MODE_VSTRIPE: [{"cols": tuple(range(0, L, 6))}] * H}
    return q, k, v, params


def test_search_layer_pieces_and_output_assembly():
    q, k, v, params = _layer(11)
    table, loss, mse, sparsity, x_o = S.search_layer(q, k, v, params, lam=0.5, eps=1.0)
    H, L = q.shape[1], q.shape[2]
    dense = A.attention_layer(q, k, v, np.zeros(H, dtype=np.int32), [dict()] * H)
    # row 0 is the skip mode: its MSE is the mean square of the dense output and its loss has no penalty
    assert np.allclose(mse[0], (dense ** 2).mean(axis=(0, 2, 3)))
    assert np.allclose(loss[0], mse[0])
    assert np.allclose(sparsity[1], 1 - (L * 13 - 6 * 7) / L ** 2)
    # the output carries, head by head, the output of the chosen mode
    for h in range(H):
        one = np.full(H, table[h], dtype=np.int32)
        want = A.attention_layer(q, k, v, one, params.get(int(table[h]), [dict()] * H))[:, h]
        assert np.array_equal(x_o[:, h], want)


def test_full_width_patterns_cost_nothing_but_the_penalty():
    # patterns that keep the whole map reproduce dense exactly: MSE 0, loss = lambda * 1
    q, k, v, _ = _layer(12, L=20)
    H, L = q.shape[1], q.shape[2]
    params = {A.MODE_DIAG: [{"half_width": L}] * H,
              A.MODE_MULTIDIAG: [{"half_width": L, "offsets": (0,)}] * H,
              A.MODE_VSTRIPE: [{"cols": tuple(range(L))}] * H}
    table, loss, mse, sparsity, x_o = S.search_layer(q, k, v, params, lam=0.25, eps=10.0)
    assert np.allclose(mse[1:], 0.0) and np.allclose(sparsity[1:], 0.0)
    assert np.allclose(loss[1:], 0.25)
    # V of unit scale: the skip mode's MSE (about 1/L per element after averaging) is below the
    # penalty here only if it is; the rule must pick the smaller of the two
    for h in range(H):
        assert table[h] == (1 if loss[0, h] <= 0.25 else 2)


def test_epsilon_zero_and_lambda_large_keep_every_head_dense():
    q, k, v, params = _layer(13)
    table, loss, *_ = S.search_layer(q, k, v, params, lam=0.5, eps=0.0)
    assert (loss[1:] > 0).all()          # every sparse mode here has a positive loss ...
    assert (loss[0] > 0).all()           # ... and so has skipping
    assert table.tolist() == [0, 0, 0]


def test_block_sparsity_closed_forms_and_its_limit():
    L = 200
    assert S.head_block_sparsity(A.MODE_SKIP, {}, L, 16, 16) == 1.0 and S.head_block_sparsity(A.MODE_DENSE, {}, L, 16, 16) == 0.0
    # vertical stripes: 21 columns are two column tiles of 16 for each of the 13 query tiles
    cols = tuple(range(3, 200, 10))[:21] + (7,)
    cols = tuple(sorted(set(cols)))[:21]
    assert len(cols) == 21
    assert np.isclose(S.head_block_sparsity(A.MODE_VSTRIPE, {"cols": cols}, L, 16, 16), 1 - 2 / 13)
    # a diagonal of half width 0 with square tiles that divide L: exactly the n diagonal tiles
    assert np.isclose(S.head_block_sparsity(A.MODE_DIAG, {"half_width": 0}, 192, 16, 16), 1 - 12 / 144)
    # half width 16: rows 16a..16a+15 reach keys 16a-16..16a+31, the diagonal tile and both neighbours
    assert np.isclose(S.head_block_sparsity(A.MODE_DIAG, {"half_width": 16}, 192, 16, 16), 1 - (12 + 2 * 11) / 144)
    # half width 17: one key further, into the tiles two away
    assert np.isclose(S.head_block_sparsity(A.MODE_DIAG, {"half_width": 17}, 192, 16, 16), 1 - (12 + 2 * 11 + 2 * 10) / 144)
    # tiles of one element: the block count is the element count
    for mode, p in ((A.MODE_DIAG, {"half_width": 9}), (A.MODE_MULTIDIAG, {"half_width": 3, "offsets": (-40, 0, 25)}),
                    (A.MODE_VSTRIPE, {"cols": (1, 5, 77)})):
        assert np.isclose(S.head_block_sparsity(mode, p, 90, 1, 1), S.head_sparsity(mode, p, 90))
    # coarser tiles can only compute more
    for bs in (2, 4, 8, 16):
        assert S.head_block_sparsity(A.MODE_DIAG, {"half_width": 9}, 90, bs, bs) <= S.head_sparsity(A.MODE_DIAG, {"half_width": 9}, 90) + 1e-12
