"""GPU parity at the benchmark shapes, in the launch configuration bench.py
times: sampled query rows of every head against the explicit-mask oracle, and
every row of selected heads against the zero-query closed form."""
import numpy as np
import pytest
import torch

from paper_2506_03065_amd import binding as svd
from paper_2506_03065_amd import workloads as W
from parity_util import assert_close, check_layer, f64, run_planned

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _windowed_means(v, mode, p, L):
    """Mean of V over the kept keys of every row (what Q == 0 must give)."""
    prefix = np.concatenate([np.zeros((1, v.shape[1])), np.cumsum(v, axis=0)])
    if mode == W.DENSE:
        return np.broadcast_to(v.mean(axis=0), v.shape)
    if mode == W.VSTRIPE:
        return np.broadcast_to(v[list(p["cols"])].mean(axis=0), v.shape)
    i = np.arange(L)
    tot, cnt = np.zeros_like(v), np.zeros(L)
    for o in p["offsets"]:
        lo = np.clip(i + o - p["half_width"], 0, L)
        hi = np.clip(i + o + p["half_width"] + 1, 0, L)
        hi = np.maximum(hi, lo)
        tot += prefix[hi] - prefix[lo]
        cnt += hi - lo
    return tot / cnt[:, None]


@pytest.mark.parametrize("name", ["cogvideox1.5", "hunyuanvideo", "wan2.1"])
def test_benchmark_shape_sampled_rows_and_closed_form(name):
    wl = W.BY_NAME[name]()
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    out = run_planned(wl, q, k, v)
    assert torch.isfinite(out.float()).all()
    rows = W.sample_rows(wl, n_random=48)
    # rows of the ragged last tile and of the tile before it
    bq, _ = svd.svd_default_blocks(wl.D)
    rows = np.unique(np.concatenate([rows, np.arange(max(0, wl.L - 2 * bq - 3), wl.L, 37)]))
    check_layer(wl, q, k, v, out, rows=rows)
    for h in range(wl.H):
        if wl.strategy_table[h] == W.SKIP:
            assert not out[0, h].view(torch.int16).any()
    # zero queries: every row of the first head of each mode against prefix sums of V
    out0 = run_planned(wl, torch.zeros_like(q), k, v)
    for mode in (W.DENSE, W.DIAG, W.MULTIDIAG, W.VSTRIPE):
        h = int(np.nonzero(wl.strategy_table == mode)[0][0])
        want = _windowed_means(f64(v[0, h]), mode, wl.pattern_params[h], wl.L)
        assert_close(f64(out0[0, h]), want, f"{name} zero-q head {h} mode {mode}")


_STACK_QKV = {}


def _stack_qkv(wl):
    """Every layer of the stack draws Q, K, V from the same seed: generated once."""
    if wl.seed not in _STACK_QKV:
        _STACK_QKV.clear()
        _STACK_QKV[wl.seed] = [t.to(DEV) for t in W.make_qkv(wl)]
    return _STACK_QKV[wl.seed]


@pytest.mark.parametrize("layer", [0, 5, 10, 15, 20, 25, 30, 35, 39])
def test_stack_layers(layer):
    """Layers of the 40-layer stack (Wan2.1 shape, dense share falling with depth): every head on sampled rows.
    (All 40 tables are compiled against the oracle's groups and lists on the CPU, tests/test_pattern_compiler.py.)"""
    wl = W.stack_layer(layer)
    counts = W.stack_layer_counts(layer)
    assert sum(counts.values()) == wl.H and counts[W.DENSE] == int(round(40 * (0.8 - 0.7 * layer / 39)))
    q, k, v = _stack_qkv(wl)
    out = run_planned(wl, q, k, v)
    rows = W.sample_rows(wl, n_random=16, seed=layer)
    check_layer(wl, q, k, v, out, rows=rows)
    for h in range(wl.H):
        if wl.strategy_table[h] == W.SKIP:
            assert not out[0, h].view(torch.int16).any()
    if layer == 39:
        _STACK_QKV.clear()
