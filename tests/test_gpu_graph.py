"""The forward pass recorded into a HIP graph: only kernel launches and
event-based fork/join are enqueued, so a captured layer must replay to the
same bits as the eager call, also with eager work between the replays."""
import numpy as np
import pytest
import torch

from paper_2506_03065_amd import binding as svd
from paper_2506_03065_amd import workloads as W
from parity_util import check_layer

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _difference(rep, out, eager, wl):
    """Failure message: where a replay differs from the eager result."""
    diff = out.view(torch.int16) != eager.view(torch.int16)
    idx = diff.nonzero()[:4000]
    heads = sorted({(int(i[0]), int(i[1])) for i in idx})
    rows = sorted({int(i[2]) for i in idx})
    return (f"replay {rep} differs from the eager result: {int(diff.sum())} elements, "
            f"{int(torch.isnan(out.float()).sum())} NaN, (batch, head) {heads[:8]} "
            f"modes {[int(wl.strategy_table[h]) for _, h in heads[:8]]}, rows {rows[:4]}..{rows[-4:]}")


@pytest.mark.parametrize("L,D,split", [(1500, 64, 0), (900, 128, 2)])
def test_captured_forward_replays_to_the_eager_bits(L, D, split):
    wl = W.small(L=L, D=D, H=6, seed=71, B=2)
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    desc = svd.desc_of(q)
    ws = torch.empty(svd.svd_plan_workspace_bytes(desc, wl.strategy_table, wl.pattern_params, dense_split=split),
                     dtype=torch.uint8, device=DEV)
    plan = svd.svd_plan_create(desc, wl.strategy_table, wl.pattern_params, workspace=ws, dense_split=split)
    eager = torch.full_like(q, float("nan"))
    svd.svd_attn_forward_planned(plan, q, k, v, eager)
    torch.cuda.synchronize()
    check_layer(wl, q, k, v, eager)

    out = torch.full_like(q, float("nan"))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        svd.svd_attn_forward_planned(plan, q, k, v, out)       # warm-up on the capture stream
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        svd.svd_attn_forward_planned(plan, q, k, v, out)       # the binding picks up the capturing stream
    scratch = torch.empty(1 << 20, device=DEV)
    for rep in range(4):
        out.fill_(float("nan"))
        scratch.normal_()                                      # eager work and a synchronisation between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), _difference(rep, out, eager, wl)
    del graph
    plan.close()


def test_captured_fp8_forward_replays_to_the_eager_bits():
    """The FP8 layer (pre-pass, attention, merge of a split dense launch) enqueues
    kernel launches only."""
    wl = W.small(L=900, D=128, H=6, seed=73, B=2)
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    desc = svd.desc_of(q)
    ws = torch.empty(svd.svd_plan_workspace_bytes(desc, wl.strategy_table, wl.pattern_params, dense_split=2),
                     dtype=torch.uint8, device=DEV)
    plan = svd.svd_plan_create(desc, wl.strategy_table, wl.pattern_params, workspace=ws, dense_split=2)
    ws8 = torch.empty(svd.svd_fp8_workspace_bytes(desc), dtype=torch.uint8, device=DEV)
    eager = torch.full_like(q, float("nan"))
    svd.svd_attn_forward_fp8(plan, q, k, v, eager, ws8)
    torch.cuda.synchronize()
    assert torch.isfinite(eager.float()).all()

    out = torch.full_like(q, float("nan"))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        svd.svd_attn_forward_fp8(plan, q, k, v, out, ws8)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        svd.svd_attn_forward_fp8(plan, q, k, v, out, ws8)
    scratch = torch.empty(1 << 20, device=DEV)
    for rep in range(3):
        out.fill_(float("nan"))
        ws8.fill_(0x7f)                                        # the replay must refill the quantised arrays
        scratch.normal_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), _difference(rep, out, eager, wl)
    del graph
    plan.close()


@pytest.mark.skip(reason="capture of a layer with a text prefix is switched off in the library (it returns "
                         "SVD_ERR_UNSUPPORTED before enqueuing anything): a capture-and-replay run over random "
                         "layers ended in a host-side heap abort at its first layer with a split text-row launch "
                         "(L 998, D 128, 256 text tokens, five-way dense split); the library's host code replays "
                         "that sequence cleanly under AddressSanitizer on a model of the runtime "
                         "(tests/test_host_launch_model.py), so the cause is not known and the case stays off the GPU")
def test_captured_text_prefix_forward_replays_to_the_eager_bits():
    from test_gpu_random_layers import random_layer
    wl, split = random_layer(2)     # L 998, D 128, text 256, dense_split 5
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    desc = svd.desc_of(q)
    ws = torch.empty(svd.svd_plan_workspace_bytes(desc, wl.strategy_table, wl.pattern_params, dense_split=split),
                     dtype=torch.uint8, device=DEV)
    plan = svd.svd_plan_create(desc, wl.strategy_table, wl.pattern_params, workspace=ws, dense_split=split)
    eager = torch.full_like(q, float("nan"))
    svd.svd_attn_forward_planned(plan, q, k, v, eager)
    torch.cuda.synchronize()
    out = torch.full_like(q, float("nan"))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        svd.svd_attn_forward_planned(plan, q, k, v, out)
    for rep in range(3):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), _difference(rep, out, eager, wl)
    del graph
    plan.close()
