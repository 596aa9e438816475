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


def test_search_entry_points_validate_before_any_launch():
    """Bad arguments are turned into status codes on the host (fake 16-byte aligned
    'device' addresses are never dereferenced)."""
    import ctypes as C
    lib = svd.lib()
    d = svd.tensor_desc(1, 4, 100, 64)
    p16, p8 = C.c_void_p(0x1000), C.c_void_p(0x1008)
    n = C.c_size_t()
    assert lib.svd_head_mse_workspace_bytes(C.byref(d), C.byref(n)) == 0 and n.value >= 16
    assert lib.svd_head_mse_workspace_bytes(None, C.byref(n)) == 1
    bad = svd.tensor_desc(1, 4, 100, 96)
    assert lib.svd_head_mse_workspace_bytes(C.byref(bad), C.byref(n)) == 2
    # svd_head_mse: null pointers, alignment, workspace too small
    assert lib.svd_head_mse(None, p16, C.byref(d), p16, p16, 1 << 20, None) == 1
    assert lib.svd_head_mse(p8, p16, C.byref(d), p16, p16, 1 << 20, None) == 4
    assert lib.svd_head_mse(p16, p16, C.byref(d), p16, p16, 4, None) == 8
    assert lib.svd_head_mse(p16, p16, C.byref(d), p16, None, 0, None) == 8
    # svd_select_heads: bad mode id, missing source of a used mode, shape mismatch, too many heads
    ptrs = (C.c_void_p * 5)(p16, p16, p16, None, p16)
    table = np.array([0, 1, 2, 4], dtype=np.int32)
    tp = table.ctypes.data_as(C.POINTER(C.c_int32))
    bad_table = np.array([0, 1, 2, 7], dtype=np.int32)
    assert lib.svd_select_heads(ptrs, C.byref(d), bad_table.ctypes.data_as(C.POINTER(C.c_int32)), p16, C.byref(d), None) == 5
    need3 = np.array([0, 1, 3, 4], dtype=np.int32)
    assert lib.svd_select_heads(ptrs, C.byref(d), need3.ctypes.data_as(C.POINTER(C.c_int32)), p16, C.byref(d), None) == 1
    other = svd.tensor_desc(1, 4, 101, 64)
    assert lib.svd_select_heads(ptrs, C.byref(d), tp, p16, C.byref(other), None) == 2
    assert lib.svd_select_heads(ptrs, C.byref(d), tp, p8, C.byref(d), None) == 4
    many = svd.tensor_desc(1, 1025, 16, 64)
    big_table = np.zeros(1025, dtype=np.int32)
    assert lib.svd_select_heads(ptrs, C.byref(many), big_table.ctypes.data_as(C.POINTER(C.c_int32)), p16,
                                C.byref(many), None) == 9
    # svd_search_layer: workspace size comes from the host; too small or misaligned workspaces and
    # non-contiguous tensors are refused
    params = {2: [{"half_width": 5}] * 4, 3: [{"half_width": 2, "offsets": (-30, 0, 30)}] * 4,
              4: [{"cols": (1, 2, 3)}] * 4}
    need = svd.svd_search_layer_workspace_bytes(d, params)
    assert need >= 5 * 4 * 100 * 64 * 2
    arr, keep = svd._params_by_mode(params, 4)
    out_table = np.zeros(4, dtype=np.int32)
    call = lambda desc, ws, nbytes: lib.svd_search_layer(p16, p16, p16, C.byref(desc), arr, 0.5, 1.0,
                                                         out_table.ctypes.data_as(C.POINTER(C.c_int32)), None, p16,
                                                         ws, nbytes, None)
    assert call(d, C.c_void_p(0x10000), need - 1) == 8
    assert call(d, C.c_void_p(0x10010), need) == 8          # not 256-byte aligned
    assert call(d, None, need) == 8
    strided = svd.tensor_desc(1, 4, 100, 64, stride_b=4 * 100 * 64, stride_h=64, stride_l=4 * 64)
    assert call(strided, C.c_void_p(0x10000), 1 << 30) == 9
    # a parameter set that leaves a row without keys is reported as such
    empty = dict(params)
    empty[3] = [{"half_width": 1, "offsets": (40,)}] * 4
    with pytest.raises(svd.SvdError) as e:
        svd.svd_search_layer_workspace_bytes(d, empty)
    assert e.value.status == 7


def test_fp8_entry_points_validate_before_any_launch():
    """Sizes come from the host; bad arguments become status codes without a launch."""
    import ctypes as C
    lib = svd.lib()
    d = svd.tensor_desc(2, 4, 300, 64)
    n = C.c_size_t()
    assert lib.svd_fp8_workspace_bytes(C.byref(d), C.byref(n)) == 0
    assert n.value == 2 * 2 * 4 * 384 * 64          # K8 and V8, L rounded up to a multiple of 128
    assert lib.svd_fp8_workspace_bytes(None, C.byref(n)) == 1
    assert lib.svd_fp8_workspace_bytes(C.byref(d), None) == 1
    bad = svd.tensor_desc(1, 4, 100, 96)
    assert lib.svd_fp8_workspace_bytes(C.byref(bad), C.byref(n)) == 2
    p16 = C.c_void_p(0x1000)
    # without a plan nothing is dereferenced
    assert lib.svd_attn_forward_fp8(None, p16, p16, p16, p16, C.c_void_p(0x10000), 1 << 30, None) == 1
    assert lib.svd_attn_forward_fp8_group(None, 0, p16, p16, p16, p16, C.c_void_p(0x10000), 1 << 30, None) == 1
    # a plan without device workspace can be inspected but not launched
    table = np.array([0, 2, 3, 4], dtype=np.int32)
    params = [{}, {"half_width": 5}, {"half_width": 2, "offsets": (-30, 0, 30)}, {"cols": (1, 2, 3)}]
    plan = svd.svd_plan_create(d, table, params)
    assert lib.svd_attn_forward_fp8(plan.handle, p16, p16, p16, p16, C.c_void_p(0x10000), 1 << 30, None) == 8
    assert lib.svd_attn_forward_fp8(plan.handle, None, p16, p16, p16, C.c_void_p(0x10000), 1 << 30, None) == 1
    plan.close()


@pytest.mark.parametrize("L,D,text", [(333, 64, 0), (1000, 128, 0), (900, 128, 256), (1300, 64, 512)])
def test_plan_head_block_sparsity_matches_the_explicit_mask_tiles(L, D, text):
    """The block-level S_i (Section 4.2's wording) from the plan's lists against the oracle's count over explicit-mask tiles."""
    wl = W.small(L=L, D=D, H=5, seed=29)
    if text:
        wl = W.with_text_borders(wl, text)
    plan = svd.svd_plan_create(svd.tensor_desc(wl.B, wl.H, wl.L, wl.D), wl.strategy_table, wl.pattern_params)
    got = plan.head_block_sparsity()
    for g in plan.groups():
        for h in g["heads"]:
            want = S.head_block_sparsity(int(wl.strategy_table[h]), wl.pattern_params[h], wl.L, g["block_q"], g["block_k"])
            assert abs(got[h] - want) <= 1e-15, (h, g["mode"], got[h], want)
    plan.close()


def test_probe_entry_points_validate_on_the_host():
    """The calibration probes refuse bad arguments before any launch (no GPU needed for that)."""
    import ctypes as C
    lib = svd.lib()
    flops = C.c_double()
    assert lib.svd_probe_mfma(None, 0, 1, 1, C.byref(flops), None) == 1                    # SVD_ERR_NULL
    assert lib.svd_probe_mfma(C.c_void_p(256), 4096, 0, 1, C.byref(flops), None) == 2      # SVD_ERR_SHAPE: no iterations
    assert lib.svd_probe_mfma(C.c_void_p(256), 100, 1, 1, C.byref(flops), None) == 8       # SVD_ERR_WORKSPACE: scratch too small
    assert lib.svd_probe_copy(None, C.c_void_p(256), 16, None) == 1
    assert lib.svd_probe_copy(C.c_void_p(256), C.c_void_p(512), 24, None) == 2             # not a multiple of 16 bytes
    assert lib.svd_probe_copy(C.c_void_p(8), C.c_void_p(512), 32, None) == 4               # SVD_ERR_ALIGN
