"""The whole layer in ONE launch (plan option single_launch): resident work-groups
pulling items off per-XCD work queues.  Same arithmetic per query row as the
grouped launches, so the result must equal that of a grouped plan with
dense_split = 1 bit for bit; and it must meet the oracle's bars."""
import numpy as np
import pytest
import torch

from paper_2506_03065_amd import binding as svd
from paper_2506_03065_amd import workloads as W
from parity_util import check_layer
from test_gpu_random_layers import random_layer

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_plan(wl, q, k, v, **options):
    desc = svd.desc_of(q)
    ws = torch.empty(svd.svd_plan_workspace_bytes(desc, wl.strategy_table, wl.pattern_params, **options),
                     dtype=torch.uint8, device=DEV)
    ws.fill_(0xA5)                                # the queue positions must not depend on what the workspace held
    plan = svd.svd_plan_create(desc, wl.strategy_table, wl.pattern_params, workspace=ws, **options)
    assert plan.single_launch() == (options.get("single_launch", 0) in (1, 3))
    out = torch.full_like(q, float("nan"))
    svd.svd_attn_forward_planned(plan, q, k, v, out)
    torch.cuda.synchronize()
    return out, plan, ws


def bits(t):
    return t.view(torch.int16)


def assert_same_bits(a, b, first_row=0):
    """Rows first_row.. of every head; a short message instead of two tensors."""
    diff = bits(a)[:, :, first_row:] != bits(b)[:, :, first_row:]
    assert not diff.any(), f"{int(diff.sum())} elements differ, first at {diff.nonzero()[0].tolist()}"


@pytest.mark.parametrize("L,D,H,seed,B", [(333, 64, 5, 7, 1), (200, 128, 5, 11, 1), (1000, 64, 5, 3, 2),
                                           (1500, 128, 10, 4, 2), (31, 64, 4, 6, 1), (1, 128, 5, 12, 1),
                                           (2600, 64, 7, 8, 1)])
def test_small_layers_all_rows_equal_the_grouped_launches(L, D, H, seed, B):
    wl = W.small(L=L, D=D, H=H, seed=seed, B=B)
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    one, plan, ws = run_plan(wl, q, k, v, single_launch=1)
    grouped, plan_g, _ = run_plan(wl, q, k, v, single_launch=2, dense_split=1)
    assert_same_bits(one, grouped)
    check_layer(wl, q, k, v, one)
    # a second and third pass with the same plan (the queue positions are reset by the call itself)
    for _ in range(2):
        again = torch.full_like(q, float("nan"))
        svd.svd_attn_forward_planned(plan, q, k, v, again)
        torch.cuda.synchronize()
        assert torch.equal(bits(again), bits(one))
    plan.close()
    plan_g.close()


@pytest.mark.parametrize("seed", [0, 2, 3, 5, 7, 9])
def test_random_layers(seed):
    """Random mode mixes, widths, column sets, batch and text prefix.  Text rows become dense items here, while the
    grouped launches may cut their key range and merge (another rounding): those rows are held to the oracle only."""
    wl, _ = random_layer(seed)
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    one, plan, _ = run_plan(wl, q, k, v, single_launch=1)
    grouped, plan_g, _ = run_plan(wl, q, k, v, single_launch=2, dense_split=1)
    assert_same_bits(one, grouped, first_row=wl.text_tokens)
    dense = [h for h in range(wl.H) if wl.strategy_table[h] in (W.DENSE, W.SKIP)]
    assert_same_bits(one[:, dense], grouped[:, dense])
    check_layer(wl, q, k, v, one)
    plan.close()
    plan_g.close()


def test_rearranged_heads_and_strided_layout():
    wl = W.small(L=900, D=128, H=6, seed=17)
    wl.pattern_params[2] = {"half_width": 2 * 5 + 4, "rearranged": (0, 180, 5)}       # the multi-diagonal head in rearranged form
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    q, k, v = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (q, k, v))   # token-major storage
    one, plan, _ = run_plan(wl, q, k, v, single_launch=1)
    grouped, plan_g, _ = run_plan(wl, q, k, v, single_launch=2, dense_split=1)
    assert_same_bits(one, grouped)
    plan.close()
    plan_g.close()


@pytest.mark.parametrize("L,D,form", [(1500, 64, 1), (9000, 128, 0)])
def test_captured_single_launch_replays_to_the_eager_bits(L, D, form):
    """form 0 at D = 128 on a layer whose items are long enough: the library's own choice is the layer kernel
    (gather pre-pass, fill, layer kernel)."""
    wl = W.small(L=L, D=D, H=6, seed=71, B=2 if form else 1)
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    if form:
        eager, plan, _ = run_plan(wl, q, k, v, single_launch=form)
    else:
        desc = svd.desc_of(q)
        ws = torch.empty(svd.svd_plan_workspace_bytes(desc, wl.strategy_table, wl.pattern_params), dtype=torch.uint8, device=DEV)
        plan = svd.svd_plan_create(desc, wl.strategy_table, wl.pattern_params, workspace=ws)
        assert plan.single_launch()
        eager = torch.full_like(q, float("nan"))
        svd.svd_attn_forward_planned(plan, q, k, v, eager)
        torch.cuda.synchronize()
    out = torch.full_like(q, float("nan"))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        svd.svd_attn_forward_planned(plan, q, k, v, out)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        svd.svd_attn_forward_planned(plan, q, k, v, out)
    scratch = torch.empty(1 << 20, device=DEV)
    for rep in range(4):
        out.fill_(float("nan"))
        scratch.normal_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(bits(out), bits(eager)), f"replay {rep}"
    del graph
    plan.close()


@pytest.mark.parametrize("B", [1, 2])
def test_dense_head_start_covers_whole_rounds_and_leaves_the_rest_to_the_queues(B):
    """26 dense heads of 11 256-row tiles: 286 dense items per batch entry, of which 256 (B = 2: 512 of 572) go
    through the dense kernel, whole rounds of the 256 compute units; the queues' dense segment starts in the middle
    of a head (B = 2: of a head of the second batch entry), at a 128-row item."""
    wl = W.small(L=2600, D=64, H=30, seed=19, B=B)
    for h in range(4, 30):
        wl.strategy_table[h] = W.DENSE
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    one, plan, _ = run_plan(wl, q, k, v, single_launch=3)
    grouped, plan_g, _ = run_plan(wl, q, k, v, single_launch=2, dense_split=1)
    assert_same_bits(one, grouped)
    check_layer(wl, q, k, v, one, heads=[0, 1, 2, 3, 4, 17, 26, 27, 28, 29])
    plan.close()
    plan_g.close()


@pytest.mark.parametrize("name", ["cogvideox1.5", "hunyuanvideo", "wan2.1"])
def test_benchmark_shapes_sampled_rows(name):
    """Both forms (the layer kernel alone, and after the dense head start) at the benchmark shapes."""
    wl = W.BY_NAME[name]()
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    grouped, plan_g, _ = run_plan(wl, q, k, v, single_launch=2, dense_split=1)
    plan_g.close()
    rows = W.sample_rows(wl, n_random=24)
    for form in (1, 3):
        one, plan, _ = run_plan(wl, q, k, v, single_launch=form)
        assert torch.isfinite(one.float()).all()
        assert_same_bits(one, grouped)
        if form == 3:
            check_layer(wl, q, k, v, one, rows=rows)
        plan.close()


@pytest.mark.parametrize("form", [1, 3])
@pytest.mark.parametrize("modes", [[W.SKIP] * 3, [W.DENSE] * 2, [W.VSTRIPE] * 3, [W.DIAG], [W.SKIP, W.MULTIDIAG]])
def test_degenerate_tables(modes, form):
    """Layers made of one mode only (a single segment, or none that computes), one head, skip plus one pattern."""
    L, D = 700, 128
    base = W.small(L=L, D=D, H=5, seed=23)                      # one parameter set per mode to borrow from
    by_mode = {int(m): p for m, p in zip(base.strategy_table, base.pattern_params)}
    wl = W.Workload("degenerate", -1, 1, len(modes), L, D, base.frame_tokens, base.n_frames, 0,
                    np.asarray(modes, dtype=np.int32), [dict(by_mode[int(m)]) for m in modes], 99)
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    one, plan, _ = run_plan(wl, q, k, v, single_launch=form)
    grouped, plan_g, _ = run_plan(wl, q, k, v, single_launch=2, dense_split=1)
    assert_same_bits(one, grouped)
    check_layer(wl, q, k, v, one)
    plan.close()
    plan_g.close()
