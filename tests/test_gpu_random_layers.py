"""Seeded random layers: lengths, head sizes, mode mixes, band widths, offsets,
column sets, batch, text prefix and dense split drawn at random; bf16 and FP8
paths against their oracles on all rows."""
import numpy as np
import pytest
import torch

from paper_2506_03065_amd import workloads as W
from parity_util import check_layer, run_planned
from test_gpu_fp8 import check_layer_fp8, run_fp8

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def random_layer(seed):
    rng = np.random.default_rng(1000 + seed)
    D = int(rng.choice([64, 128]))
    L = int(rng.integers(260, 2200))
    H = int(rng.integers(3, 9))
    B = int(rng.choice([1, 1, 2]))
    text = int(rng.choice([0, 0, 256])) if L > 600 else 0
    table = rng.integers(0, 5, H).astype(np.int32)
    table[rng.integers(0, H)] = W.MULTIDIAG          # at least one of the harder modes
    params = []
    for m in table:
        p = {"half_width": 0, "offsets": (), "cols": ()}
        if m == W.DIAG:
            p["half_width"] = int(rng.integers(0, L // 2))
            p["offsets"] = (0,)
        elif m == W.MULTIDIAG:
            step = int(rng.integers(20, max(21, L // 3)))
            ks = rng.choice(np.arange(-4, 5), size=int(rng.integers(1, 6)), replace=False)
            offs = sorted({0} | {int(k) * step for k in ks})      # offset 0 keeps every row non-empty
            p["half_width"] = int(rng.integers(0, max(1, step // 2)))
            p["offsets"] = tuple(offs)
        elif m == W.VSTRIPE:
            n = int(rng.integers(1, max(2, L // 4)))
            p["cols"] = tuple(int(c) for c in np.sort(rng.choice(L, size=n, replace=False)))
        if text and m >= W.DIAG:
            p["text_tokens"] = text
        params.append(p)
    split = int(rng.choice([0, 0, 1, 2, 5]))
    wl = W.Workload(f"random{seed}", -1, B, H, L, D, max(8, L // 5), 5, text, table, params, 4000 + seed)
    return wl, split


@pytest.mark.parametrize("seed", list(range(12)) + [23, 45])   # the last two: narrow-band heads with the largest single-element deviations seen
def test_random_layer(seed):
    wl, split = random_layer(seed)
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    out = run_planned(wl, q, k, v, dense_split=split)
    check_layer(wl, q, k, v, out)
    out8, _ = run_fp8(wl, q, k, v, dense_split=split)
    check_layer_fp8(wl, q, k, v, out8)
    for h in range(wl.H):
        if wl.strategy_table[h] == W.SKIP:
            assert not out[:, h].view(torch.int16).any() and not out8[:, h].view(torch.int16).any()
