"""GPU parity of the token rearrangement (Section 4.1.2) and of the path it
enables: rearrange q, k, v, run the diagonal mode, rearrange the output back;
against the oracle that states the kept set in the original order."""
import numpy as np
import pytest
import torch

from oracle import rearrange as R
from paper_2506_03065_amd import binding as svd
from paper_2506_03065_amd import workloads as W
from parity_util import assert_close, f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("B,H,L,D,first,N,F", [(1, 3, 1000, 64, 0, 100, 10), (2, 2, 777, 128, 17, 40, 19),
                                               (1, 1, 2100, 64, 256, 461, 4), (1, 2, 64, 128, 0, 1, 64)])
def test_rows_move_bit_for_bit(B, H, L, D, first, N, F):
    g = torch.Generator().manual_seed(5)
    x = torch.randn(B, H, L, D, generator=g).to(torch.bfloat16).to(DEV)
    y = torch.full_like(x, float("nan"))
    svd.svd_rearrange_tokens(x, y, first, N, F)
    pi = torch.from_numpy(R.position_major_index(L, first, N, F)).to(DEV)
    want = torch.empty_like(x)
    want[:, :, pi] = x
    assert torch.equal(y.view(torch.int16), want.view(torch.int16))
    z = torch.full_like(x, float("nan"))
    svd.svd_rearrange_tokens(y, z, first, N, F, inverse=True)
    assert torch.equal(z.view(torch.int16), x.view(torch.int16))
    # strided (token-major storage) tensors
    xs = x.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    ys = torch.full_like(xs, float("nan"))
    svd.svd_rearrange_tokens(xs, ys, first, N, F)
    assert torch.equal(ys.contiguous().view(torch.int16), want.view(torch.int16))


def test_validation():
    x = torch.zeros(1, 1, 100, 64, dtype=torch.bfloat16, device=DEV)
    y = torch.full_like(x, 3.0)
    for args, status in (((0, 30, 4), 6), ((-1, 10, 4), 6), ((0, 0, 4), 6), ((90, 5, 3), 6)):
        with pytest.raises(svd.SvdError) as e:
            svd.svd_rearrange_tokens(x, y, *args)
        assert e.value.status == status
    with pytest.raises(svd.SvdError) as e:
        svd.svd_rearrange_tokens(x, x, 0, 10, 10)
    assert e.value.status == 9
    torch.cuda.synchronize()
    assert (y == 3.0).all()


def rearranged_window_attention(q, k, v, first, N, F, W):
    """The path of the header comment: three rearrangements, the diagonal mode, one back."""
    B, H, L, D = q.shape
    qp, kp, vp, op, out = (torch.empty_like(q) for _ in range(5))
    for src, dst in ((q, qp), (k, kp), (v, vp)):
        svd.svd_rearrange_tokens(src, dst, first, N, F)
    table = np.full(H, W_DIAG, dtype=np.int32)
    params = [{"half_width": W}] * H
    desc = svd.desc_of(q)
    ws = torch.empty(svd.svd_plan_workspace_bytes(desc, table, params), dtype=torch.uint8, device=q.device)
    plan = svd.svd_plan_create(desc, table, params, workspace=ws)
    svd.svd_attn_forward_planned(plan, qp, kp, vp, op)
    svd.svd_rearrange_tokens(op, out, first, N, F, inverse=True)
    torch.cuda.synchronize()
    plan.close()
    return out


W_DIAG = W.DIAG


@pytest.mark.parametrize("L,D,first,N,F,w", [(1000, 64, 0, 100, 10, 3), (1300, 128, 256, 87, 12, 2)])
def test_window_in_position_major_order_all_rows(L, D, first, N, F, w):
    g = torch.Generator().manual_seed(9)
    q, k, v = (torch.randn(1, 2, L, D, generator=g).to(torch.bfloat16).to(DEV) for _ in range(3))
    Wd = w * F + F - 1
    out = rearranged_window_attention(q, k, v, first, N, F, Wd)
    for h in range(2):
        want = R.attention_head_rearranged(f64(q[0, h]), f64(k[0, h]), f64(v[0, h]), first, N, F, Wd)
        assert_close(f64(out[0, h]), want, f"rearranged window head {h}")


def test_wan_shape_sampled_rows():
    L, D, N, F, w = 75600, 128, 3600, 21, 40
    g = torch.Generator().manual_seed(13)
    q, k, v = (torch.randn(1, 2, L, D, generator=g).to(torch.bfloat16).to(DEV) for _ in range(3))
    Wd = w * F + F - 1
    out = rearranged_window_attention(q, k, v, 0, N, F, Wd)
    rows = np.unique(np.concatenate([np.arange(0, 4), np.arange(L - 4, L), [N - 1, N, 20 * N, 20 * N + N - 1],
                                     np.random.default_rng(2).integers(0, L, 24)]))
    for h in range(2):
        want = R.attention_head_rearranged(f64(q[0, h]), f64(k[0, h]), f64(v[0, h]), 0, N, F, Wd, rows=rows)
        assert_close(f64(out[0, h][torch.as_tensor(rows)]), want, f"rearranged window, Wan shape, head {h}")


# ---- the rearranged form inside the strategy table: no copies, rows reached through the row map ----

@pytest.mark.parametrize("L,D,B,first,N,F,w", [(1000, 64, 1, 0, 100, 10, 3), (1300, 128, 2, 256, 87, 12, 2),
                                                (777, 64, 1, 17, 40, 19, 0), (520, 128, 1, 0, 520, 1, 30)])
def test_rearranged_heads_in_a_layer_all_rows(L, D, B, first, N, F, w):
    from parity_util import check_layer, run_planned
    wl = W.small(L=L, D=D, H=10, seed=21, B=B)
    params = [dict(p) for p in wl.pattern_params]
    multi = [h for h in range(wl.H) if wl.strategy_table[h] == W.MULTIDIAG]
    params[multi[0]] = {"half_width": w * F + F - 1, "offsets": (), "cols": (), "rearranged": (first, N, F)}
    wl.pattern_params = params
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    out = run_planned(wl, q, k, v)
    check_layer(wl, q, k, v, out)
    # the same head through the explicit path: identical kept set, same kernel family
    h = multi[0]
    ref = rearranged_window_attention(q[:, h:h + 1].contiguous(), k[:, h:h + 1].contiguous(), v[:, h:h + 1].contiguous(),
                                      first, N, F, w * F + F - 1)
    assert_close(f64(out[0, h]), f64(ref[0, 0]), "row-map path against the copy path")
    # FP8 variant: the pre-pass writes K8 and V8 in the rearranged order
    from test_gpu_fp8 import check_layer_fp8, run_fp8
    out8, _ = run_fp8(wl, q, k, v)
    check_layer_fp8(wl, q, k, v, out8)


def test_rearranged_heads_wan_shape_sampled_rows():
    from parity_util import check_layer, run_planned
    L, D, N, F, w = 75600, 128, 3600, 21, 40
    table = np.asarray([W.MULTIDIAG, W.MULTIDIAG, W.DIAG], dtype=np.int32)
    params = [{"half_width": w * F + F - 1, "rearranged": (0, N, F)}, {"half_width": 900, "offsets": (-N, 0, N)},
              {"half_width": 3600}]
    wl = W.Workload("wan-rearranged", -1, 1, 3, L, D, N, F, 0, table, params, 77)
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    out = run_planned(wl, q, k, v)
    rows = np.unique(np.concatenate([np.arange(0, 4), np.arange(L - 4, L), [N - 1, N, 20 * N, 20 * N + N - 1],
                                     np.random.default_rng(3).integers(0, L, 20)]))
    check_layer(wl, q, k, v, out, rows=rows)
    from test_gpu_fp8 import check_layer_fp8, run_fp8
    out8, _ = run_fp8(wl, q, k, v)
    check_layer_fp8(wl, q, k, v, out8, rows=rows)
