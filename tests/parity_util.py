"""Shared helpers of the GPU parity tests: run the HIP path through the C-ABI
binding and compare with the CPU oracle on the same seeded inputs."""
import numpy as np
import torch

from oracle import sparse_attention as O
from paper_2506_03065_amd import binding as svd

# The contract: max abs error <= 2e-2 and mean abs error <= 2e-3 against the
# oracle.  With N(0,1) inputs the outputs of long heads are small, so two
# scale-free gates are added per head: relative L2 error <= 1e-2 and
# max abs error <= 8e-2 * rms(reference) + 1e-3.  Where the 8e-2 comes from:
# the precision this build specifies (bf16 pre-scaled Q, bf16 P, bf16 output,
# everything else exact), carried out on the CPU, already deviates from the
# exact definition by up to 6.6 % of a head's rms on a single element of a
# narrow-band head (tests/test_tolerance_derivation.py, which also holds the
# gate to at most 1.5 times that); the kernel adds the order of its tiles.
MAX_ABS, MEAN_ABS, REL_L2, MAX_OVER_RMS = 2e-2, 2e-3, 1e-2, 8e-2


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def run_planned(wl, q, k, v, out=None, dense_split=0):
    """q, k, v: CUDA bf16 [B, H, L, D] (any strides with contiguous D)."""
    desc = svd.desc_of(q)
    nbytes = svd.svd_plan_workspace_bytes(desc, wl.strategy_table, wl.pattern_params, dense_split=dense_split)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=q.device)
    plan = svd.svd_plan_create(desc, wl.strategy_table, wl.pattern_params, workspace=ws, dense_split=dense_split)
    if dense_split > 1:
        assert plan.dense_split() >= 1
    if out is None:
        out = torch.full_like(q, float("nan"))
    svd.svd_attn_forward_planned(plan, q, k, v, out)
    torch.cuda.synchronize()
    plan.close()
    return out


def assert_close(got, want, what=""):
    """got, want: float64 arrays of one head, [R, D]."""
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    diff = np.abs(got - want)
    rms = float(np.sqrt((want ** 2).mean()))
    assert diff.max() <= MAX_ABS, f"{what}: max abs {diff.max():.3e}"
    assert diff.mean() <= MEAN_ABS, f"{what}: mean abs {diff.mean():.3e}"
    if rms > 0:
        rel = float(np.sqrt((diff ** 2).sum() / (want ** 2).sum()))
        assert rel <= REL_L2, f"{what}: relative L2 {rel:.3e}"
        assert diff.max() <= MAX_OVER_RMS * rms + 1e-3, f"{what}: max abs {diff.max():.3e} vs rms {rms:.3e}"
    else:
        assert not got.any(), f"{what}: expected exact zeros"


def check_layer(wl, q, k, v, out, rows=None, heads=None):
    """Compare out (CUDA) with the oracle for every head (or `heads`), on all
    rows or on `rows`."""
    qc, kc, vc = q.cpu(), k.cpu(), v.cpu()
    oc = out.cpu()
    for b in range(wl.B):
        for h in (range(wl.H) if heads is None else heads):
            mode, p = int(wl.strategy_table[h]), wl.pattern_params[h]
            want = O.attention_head(f64(qc[b, h]), f64(kc[b, h]), f64(vc[b, h]), mode, p, rows=rows)
            got = f64(oc[b, h]) if rows is None else f64(oc[b, h][torch.as_tensor(rows)])
            assert_close(got, want, f"{wl.name} b{b} h{h} mode{mode}")
