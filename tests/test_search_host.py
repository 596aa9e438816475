"""Host logic of the search step through the C ABI (no GPU): Eq. 2-3 selection
and the per-head sparsity of a plan, against the oracle."""
import numpy as np
import pytest

from oracle import sparse_attention as A
from oracle import sparse_search as S
from paper_2506_03065_amd import binding as svd
from paper_2506_03065_amd import workloads as W


def test_select_matches_the_oracle_on_random_and_tied_losses():
    gen = np.random.default_rng(5)
    for trial in range(50):
        H = int(gen.integers(1, 40))
        mse = (gen.random((4, H)) * gen.choice([0.1, 1.0, 10.0])).astype(np.float32)
        sparsity = gen.random((4, H))
        sparsity[0] = 1.0
        if trial % 5 == 0:          # exact ties between modes and with the threshold
            mse[:] = np.float32(0.25)
            sparsity[:] = 1.0
        lam, eps = float(gen.choice([0.0, 0.1, 0.5, 1.0])), float(gen.choice([0.25, 0.5, 1.0, 3.0]))
        table, loss = svd.svd_search_select(mse, sparsity, lam, eps)
        # the library may fuse the multiply-add of Eq. 2: last-bit differences are allowed in the
        # loss, the selection is checked exactly on the loss the library reports
        assert np.allclose(loss, S.losses(mse, sparsity, lam), rtol=1e-14, atol=0)
        assert np.array_equal(table, S.select_modes(loss, eps))


def test_select_rejects_bad_arguments():
    # the raw entry point returns a status and touches nothing
    assert svd.lib().svd_search_select(3, None, None, 0.5, 1.0, None, None) == 1   # SVD_ERR_NULL
    with pytest.raises(svd.SvdError):
        svd.svd_search_select(np.zeros((4, 0)), np.zeros((4, 0)), 0.5, 1.0)


@pytest.mark.parametrize("name", ["tiny"])
def test_plan_head_sparsity_matches_the_explicit_mask(name):
    wl = W.BY_NAME[name]()
    plan = svd.svd_plan_create(svd.tensor_desc(wl.B, wl.H, wl.L, wl.D), wl.strategy_table, wl.pattern_params)
    got = plan.head_sparsity()
    plan.close()
    want = [S.head_sparsity(int(wl.strategy_table[h]), wl.pattern_params[h], wl.L) for h in range(wl.H)]
    assert np.allclose(got, want, rtol=0, atol=1e-15)


def test_plan_head_sparsity_small_mixed_layer():
    wl = W.small(L=333, D=64, H=10, seed=3)
    plan = svd.svd_plan_create(svd.tensor_desc(wl.B, wl.H, wl.L, wl.D), wl.strategy_table, wl.pattern_params)
    got = plan.head_sparsity()
    plan.close()
    want = [S.head_sparsity(int(wl.strategy_table[h]), wl.pattern_params[h], wl.L) for h in range(wl.H)]
    assert np.allclose(got, want, rtol=0, atol=1e-15)
