"""GPU parity of the offline search step (Section 4.2, Eq. 2-3, Algorithm 1)
through the C ABI, against the oracle."""
import numpy as np
import pytest
import torch

from oracle import sparse_attention as A
from oracle import sparse_search as S
from paper_2506_03065_amd import binding as svd
from paper_2506_03065_amd import workloads as W
from parity_util import f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("B,H,L,D", [(1, 3, 1000, 64), (2, 5, 333, 128), (1, 1, 31, 64), (1, 4, 9000, 128)])
def test_head_mse_matches_the_definition(B, H, L, D):
    gen = torch.Generator().manual_seed(100 + L)
    a = torch.randn(B, H, L, D, generator=gen).to(torch.bfloat16)
    b = (a.float() + 0.1 * torch.randn(B, H, L, D, generator=gen)).to(torch.bfloat16)
    b[:, 0] = a[:, 0]                       # one head identical: exactly zero
    want = S.head_mse(f64(a), f64(b))
    a, b = a.to(DEV), b.to(DEV)
    ws = torch.empty(max(svd.svd_head_mse_workspace_bytes(svd.desc_of(a)), 4), dtype=torch.uint8, device=DEV)
    mse = torch.full((H,), float("nan"), dtype=torch.float32, device=DEV)
    svd.svd_head_mse(a, b, mse, ws)
    first = mse.cpu().numpy().copy()
    svd.svd_head_mse(a, b, mse, ws)
    torch.cuda.synchronize()
    got = mse.cpu().numpy()
    assert got[0] == 0.0
    # fp32 products and partial sums, double final sum: a few ulps of float32
    assert np.allclose(got, want, rtol=2e-5, atol=0), (got, want)
    assert np.array_equal(got, first), "the reduction must give the same bits on every run"


def test_head_mse_strided_layout():
    B, H, L, D = 2, 4, 200, 64
    gen = torch.Generator().manual_seed(7)
    a_blhd = torch.randn(B, L, H, D, generator=gen).to(torch.bfloat16).to(DEV)
    b_blhd = torch.randn(B, L, H, D, generator=gen).to(torch.bfloat16).to(DEV)
    a, b = a_blhd.permute(0, 2, 1, 3), b_blhd.permute(0, 2, 1, 3)      # [B, H, L, D] views
    ws = torch.empty(max(svd.svd_head_mse_workspace_bytes(svd.desc_of(a)), 4), dtype=torch.uint8, device=DEV)
    mse = torch.empty(H, dtype=torch.float32, device=DEV)
    svd.svd_head_mse(a, b, mse, ws)
    torch.cuda.synchronize()
    assert np.allclose(mse.cpu().numpy(), S.head_mse(f64(a), f64(b)), rtol=2e-5, atol=0)


def test_select_heads_copies_the_chosen_mode_bit_for_bit():
    B, H, L, D = 2, 6, 130, 64
    gen = torch.Generator().manual_seed(9)
    modes = [torch.randn(B, H, L, D, generator=gen).to(torch.bfloat16).to(DEV) for _ in range(5)]
    table = np.array([0, 4, 2, 2, 1, 3], dtype=np.int32)
    out_blhd = torch.zeros(B, L, H, D, dtype=torch.bfloat16, device=DEV)
    out = out_blhd.permute(0, 2, 1, 3)                                  # strided destination
    svd.svd_select_heads(modes, table, out)
    torch.cuda.synchronize()
    for h in range(H):
        assert torch.equal(out[:, h], modes[int(table[h])][:, h])
    # a mode the table does not use may be missing
    modes[3] = None
    table2 = np.array([0, 4, 2, 2, 1, 1], dtype=np.int32)
    svd.svd_select_heads(modes, table2, out)
    torch.cuda.synchronize()
    assert torch.equal(out[:, 5], modes[1][:, 5])
    with pytest.raises(svd.SvdError):
        svd.svd_select_heads(modes, table, out)                         # mode 3 is needed now


def _search_case(seed, H, L, D):
    wl = W.small(L=L, D=D, H=H, seed=seed)
    q, k, v = W.make_qkv(wl)
    gen = np.random.default_rng(seed)
    params = {A.MODE_DIAG: [{"half_width": int(gen.integers(L // 16, L // 4))} for _ in range(H)],
              A.MODE_MULTIDIAG: [{"half_width": int(gen.integers(2, L // 20 + 3)), "offsets": (-L // 3, 0, L // 3)}
                                 for _ in range(H)],
              A.MODE_VSTRIPE: [{"cols": tuple(sorted(gen.choice(L, size=L // 8, replace=False).tolist()))}
                               for _ in range(H)]}
    return q, k, v, params


@pytest.mark.parametrize("seed,H,L,D,lam,eps", [(61, 4, 500, 64, 0.5, 1.0), (62, 3, 300, 128, 0.1, 0.05),
                                               (63, 4, 700, 64, 0.0, 0.02), (64, 2, 260, 128, 1.0, 0.5)])
def test_search_layer_against_the_oracle(seed, H, L, D, lam, eps):
    q, k, v, params = _search_case(seed, H, L, D)
    want_table, want_loss, want_mse, want_sparsity, want_xo = S.search_layer(f64(q), f64(k), f64(v), params, lam, eps)
    q, k, v = (t.to(DEV) for t in (q, k, v))
    desc = svd.desc_of(q)
    ws = torch.empty(svd.svd_search_layer_workspace_bytes(desc, params), dtype=torch.uint8, device=DEV)
    out = torch.full_like(q, float("nan"))
    table, loss = svd.svd_search_layer(q, k, v, params, lam, eps, out, ws)
    # losses: the sparsity part is exact, the MSE part carries the bf16 error of the outputs
    # (relative 1e-2 on the difference of two outputs, so on the MSE about 2e-2 plus a floor)
    assert np.allclose(loss, want_loss, rtol=3e-2, atol=2e-5), (loss, want_loss)
    # the table must be the rule applied to the losses the library saw ...
    assert np.array_equal(table, S.select_modes(loss, eps))
    # ... and equal to the oracle's wherever its decision has a margin
    for h in range(H):
        col = np.sort(want_loss[:, h])
        clear = (col[1] - col[0] > 0.05 * col[0] + 1e-4) and np.all(np.abs(want_loss[:, h] - eps) > 0.05 * eps + 1e-4)
        if clear:
            assert table[h] == want_table[h], (h, loss[:, h], want_loss[:, h])
    # the output carries the chosen mode's output head by head (compare with the oracle run of that mode)
    got = f64(out)
    for h in range(H):
        one = np.full(H, table[h], dtype=np.int32)
        ref = A.attention_layer(f64(q), f64(k), f64(v), one, params.get(int(table[h]), [dict()] * H))[:, h]
        assert np.abs(got[:, h] - ref).max() <= 2e-2
