"""The one-shot entry point that allocates nothing (its plan workspace is the
library's static device buffer) against the one-shot entry point that takes a
caller workspace: same bits, on two calls in a row, the second with a smaller
layer, then the first layer again (the buffer keeps the last call's contents)."""
import pytest
import torch

from paper_2506_03065_amd import binding as svd
from paper_2506_03065_amd import workloads as W
from parity_util import check_layer

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(wl):
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    desc = svd.desc_of(q)
    ws = torch.empty(svd.svd_plan_workspace_bytes(desc, wl.strategy_table, wl.pattern_params),
                     dtype=torch.uint8, device=DEV)
    want = torch.full_like(q, float("nan"))
    svd.sparse_vdit_attn_forward(q, k, v, wl.strategy_table, wl.pattern_params, want, ws)
    torch.cuda.synchronize()
    got = torch.full_like(q, float("nan"))
    svd.sparse_vdit_attn_forward_static(q, k, v, wl.strategy_table, wl.pattern_params, got)
    torch.cuda.synchronize()
    return q, k, v, want, got


def test_static_entry_point_matches_the_workspace_entry_point():
    big = W.small(L=1500, D=128, H=7, seed=91, B=2)      # all five modes, ragged, split dense heads
    little = W.small(L=333, D=64, H=5, seed=92)
    for wl in (big, little, big):
        q, k, v, want, got = _both(wl)
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), wl.name
        check_layer(wl, q, k, v, got)
    # the cached plan: a second call with the same layer, on another stream
    q, k, v, want, _ = _both(big)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    got = torch.full_like(q, float("nan"))
    with torch.cuda.stream(side):
        svd.sparse_vdit_attn_forward_static(q, k, v, big.strategy_table, big.pattern_params, got)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
