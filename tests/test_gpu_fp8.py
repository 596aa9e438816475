"""GPU parity of the FP8 variant: the HIP path, called through the C ABI, against
the quantise-dequantise oracle; the quantised arrays byte by byte."""
import numpy as np
import pytest
import torch

from oracle import fp8_attention as F8
from oracle import sparse_attention as O
from paper_2506_03065_amd import binding as svd
from paper_2506_03065_amd import workloads as W
from parity_util import MAX_ABS, MAX_OVER_RMS, MEAN_ABS, REL_L2, assert_close, f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _cuda(ts):
    return [t.to(DEV) for t in ts]


def run_fp8(wl, q, k, v, dense_split=0, out=None):
    desc = svd.desc_of(q)
    nbytes = svd.svd_plan_workspace_bytes(desc, wl.strategy_table, wl.pattern_params, dense_split=dense_split)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=q.device)
    plan = svd.svd_plan_create(desc, wl.strategy_table, wl.pattern_params, workspace=ws, dense_split=dense_split)
    ws8 = torch.full((svd.svd_fp8_workspace_bytes(desc),), 0x7f, dtype=torch.uint8, device=q.device)   # NaN bytes
    if out is None:
        out = torch.full_like(q, float("nan"))
    svd.svd_attn_forward_fp8(plan, q, k, v, out, ws8)
    torch.cuda.synchronize()
    plan.close()
    return out, ws8


def best_candidates(got, candidates, slack):
    """Per row, the correct result (see attention_rows_fp8_alternatives) closest to `got`, and what is left of
    |got - it| after the row's slack: the deviation that no admissible rounding decision explains."""
    want = np.empty_like(got)
    excess = np.empty_like(got)
    for r, cand in enumerate(candidates):
        over = np.maximum(np.abs(got[r][None, :] - cand) - slack[r][None, :], 0.0)
        best = int(np.argmin(over.max(axis=1)))
        want[r], excess[r] = cand[best], over[best]
    return want, excess


def check_layer_fp8(wl, q, k, v, out, rows=None, heads=None, slack_share=0.25):
    """Against the FP8 oracle.  Where several results are correct - a probability within the fp32 score-error
    bound of a midpoint between two E4M3 values may round either way - the oracle lists them: every combination
    of the (up to six) heaviest such decisions of a row, plus an element-wise bound (slack) on what the lighter
    ones can move.  A row passes iff, for ONE of its candidates, every element lies within slack plus the
    element bar of the bf16 path; the bars are those of parity_util, applied to what exceeds the slack."""
    qc, kc, vc, oc = q.cpu(), k.cpu(), v.cpu(), out.cpu()
    for b in range(wl.B):
        for h in (range(wl.H) if heads is None else heads):
            mode, p = int(wl.strategy_table[h]), wl.pattern_params[h]
            what = f"fp8 {wl.name} b{b} h{h} mode{mode}"
            nominal, candidates, slack = F8.attention_head_fp8_alternatives(f64(qc[b, h]), f64(kc[b, h]), f64(vc[b, h]),
                                                                            mode, p, rows=rows)
            got = f64(oc[b, h]) if rows is None else f64(oc[b, h][torch.as_tensor(rows)])
            assert np.isfinite(got).all(), f"{what}: non-finite output"
            want, excess = best_candidates(got, candidates, slack)
            rms = float(np.sqrt((nominal ** 2).mean()))
            # the slack must stay a small part of the element bar, or the check would be empty (not asserted for
            # score profiles built to have large score errors: there the bound itself is what is being granted)
            if slack_share is not None:
                assert slack.max() <= slack_share * (MAX_OVER_RMS * rms + 1e-3), f"{what}: slack {slack.max():.3e} vs rms {rms:.3e}"
            assert excess.max() <= MAX_ABS, f"{what}: max abs {excess.max():.3e}"
            assert excess.mean() <= MEAN_ABS, f"{what}: mean abs {excess.mean():.3e}"
            if rms > 0:
                rel = float(np.sqrt((excess ** 2).sum() / (nominal ** 2).sum()))
                assert rel <= REL_L2, f"{what}: relative L2 {rel:.3e}"
                assert excess.max() <= MAX_OVER_RMS * rms + 1e-3, f"{what}: max abs {excess.max():.3e} vs rms {rms:.3e}"
            else:
                assert not got.any(), f"{what}: expected exact zeros"


def decode(bytes_u8):
    return bytes_u8.view(torch.float8_e4m3fn).to(torch.float64).cpu().numpy()


@pytest.mark.parametrize("L,D", [(333, 64), (200, 128), (450, 128)])
def test_quantised_arrays_byte_for_byte(L, D):
    wl = W.small(L=L, D=D, H=5, seed=13, B=2)
    q, k, v = _cuda(W.make_qkv(wl))
    _, ws8 = run_fp8(wl, q, k, v)
    Lp = (L + 127) // 128 * 128
    k8 = decode(ws8[: ws8.numel() // 2]).reshape(wl.B, wl.H, Lp, D)
    v8 = decode(ws8[ws8.numel() // 2:]).reshape(wl.B, wl.H, Lp // 64, D, 64)
    # key of byte position 32*h + 16*blk + 4*g + r inside a group of 64
    pos = np.arange(64)
    h_, blk, g, r = pos // 32, (pos // 16) % 2, (pos // 4) % 4, pos % 4
    key_of_pos = 32 * blk + 8 * g + 4 * h_ + r
    assert sorted(key_of_pos) == list(range(64))
    kc, vc = k.cpu(), v.cpu()
    for b in range(wl.B):
        for h in range(wl.H):
            mode, p = int(wl.strategy_table[h]), wl.pattern_params[h]
            if mode == W.SKIP:
                continue
            src = np.unique(np.asarray(p["cols"])) if mode == W.VSTRIPE else np.arange(L)
            n = len(src)
            want_k = np.zeros((Lp, D))
            want_v = np.zeros((Lp, D))
            want_k[:n] = F8.quantise_k(f64(kc[b, h]))[src]
            want_v[:n] = F8.quantise_v(f64(vc[b, h]))[src]
            bk = svd.svd_default_blocks(D)[1]
            n_pad = Lp if mode != W.VSTRIPE else (n + bk - 1) // bk * bk
            np.testing.assert_array_equal(k8[b, h, :n_pad], want_k[:n_pad], err_msg=f"K8 b{b} h{h}")
            got_v = np.zeros((Lp, D))
            for G in range(n_pad // 64):
                got_v[G * 64 + key_of_pos] = v8[b, h, G].T     # [64 positions, D] -> rows by key
            np.testing.assert_array_equal(got_v[:n_pad], want_v[:n_pad], err_msg=f"V8 b{b} h{h}")


def test_tiny_all_rows():
    wl = W.tiny()
    q, k, v = _cuda(W.make_qkv(wl))
    out, _ = run_fp8(wl, q, k, v)
    check_layer_fp8(wl, q, k, v, out)


@pytest.mark.parametrize("L,D,H,seed,B", [(333, 64, 5, 7, 1), (200, 128, 5, 11, 1), (1000, 64, 5, 3, 1),
                                           (1000, 128, 5, 4, 1), (77, 128, 4, 5, 1), (31, 64, 4, 6, 1),
                                           (520, 128, 10, 8, 2), (700, 64, 5, 9, 2),
                                           (1, 64, 5, 12, 1), (2, 128, 5, 13, 2), (16, 64, 5, 14, 1)])
def test_small_ragged_all_rows(L, D, H, seed, B):
    wl = W.small(L=L, D=D, H=H, seed=seed, B=B)
    q, k, v = _cuda(W.make_qkv(wl))
    out, _ = run_fp8(wl, q, k, v)
    check_layer_fp8(wl, q, k, v, out)
    for h in range(wl.H):
        if wl.strategy_table[h] == W.SKIP:
            assert not out[:, h].view(torch.int16).any(), "skipped head must be exact zeros"


def test_close_to_the_unquantised_attention():
    wl = W.small(L=600, D=128, H=5, seed=23)
    q, k, v = _cuda(W.make_qkv(wl))
    out, _ = run_fp8(wl, q, k, v)
    qc, kc, vc, oc = q.cpu(), k.cpu(), v.cpu(), out.cpu()
    for h in range(wl.H):
        mode, p = int(wl.strategy_table[h]), wl.pattern_params[h]
        if mode == W.SKIP:
            continue
        want = O.attention_head(f64(qc[0, h]), f64(kc[0, h]), f64(vc[0, h]), mode, p)
        got = f64(oc[0, h])
        rel = np.sqrt(((got - want) ** 2).sum() / (want ** 2).sum())
        assert rel < 0.08, (h, mode, rel)


def test_closed_forms_constant_v_and_zero_q():
    wl = W.small(L=900, D=128, H=5, seed=61)
    q, k, v = _cuda(W.make_qkv(wl))
    vc = torch.full_like(v, 0.625)      # representable in E4M3
    out, _ = run_fp8(wl, q, k, vc)
    for h in range(wl.H):
        want = 0.0 if wl.strategy_table[h] == W.SKIP else 0.625
        assert torch.allclose(out[0, h].float(), torch.full_like(out[0, h].float(), want), atol=4e-3)
    # zero queries: every kept key has the same P, the output is the mean of the quantised V
    out, _ = run_fp8(wl, torch.zeros_like(q), k, v)
    v8 = F8.quantise_v(f64(v[0].cpu()))
    for h in range(wl.H):
        mode, p = int(wl.strategy_table[h]), wl.pattern_params[h]
        if mode == W.DENSE:
            want = np.tile(v8[h].mean(axis=0), (wl.L, 1))
        elif mode == W.VSTRIPE:
            want = np.tile(v8[h][list(p["cols"])].mean(axis=0), (wl.L, 1))
        else:
            continue
        assert_close(f64(out[0, h].cpu()), want, f"zero-q mean, head {h}")


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("profile", ["rising", "falling", "late_outlier", "very_negative"])
def test_peaked_scores_move_the_reference(D, profile):
    """Score profiles that move the integer reference many times, never after the
    first tile, once by a large jump near the end, or that sit far below zero."""
    L, H = 1500, 5
    wl = W.small(L=L, D=D, H=H, seed=41)
    q, k, v = W.make_qkv(wl)
    j = torch.arange(L, dtype=torch.float32)
    if profile == "rising":
        gain = 0.25 + 2.75 * j / L
    elif profile == "falling":
        gain = 3.0 - 2.75 * j / L
    elif profile == "late_outlier":
        gain = torch.ones(L)
        gain[L - 37] = 5.0
    else:
        gain = torch.full((L,), 8.0)
    u = torch.nn.functional.normalize(torch.ones(D), dim=0) * (D ** 0.5)
    sign = -1.0 if profile == "very_negative" else 1.0
    q = (0.3 * q.float() + 2.0 * u).to(torch.bfloat16)
    k = (0.3 * k.float() + sign * gain[None, None, :, None] * u).to(torch.bfloat16)
    q, k, v = _cuda([q, k, v])
    out, _ = run_fp8(wl, q, k, v)
    # queries and keys share a large common component here: sum |q8 k8|, and with it the fp32 error bound of a
    # score, is one to two orders of magnitude above that of unit-variance inputs, so a large share of the
    # probabilities of a row is open; the worst-case slack (all of them flipping one way) reaches 7e-3
    check_layer_fp8(wl, q, k, v, out, slack_share=None)


@pytest.mark.parametrize("L,D,split", [(1000, 64, 3), (1000, 128, 5), (130, 64, 8)])
def test_dense_key_range_split(L, D, split):
    wl = W.small(L=L, D=D, H=5, seed=51, B=2)
    q, k, v = _cuda(W.make_qkv(wl))
    out, _ = run_fp8(wl, q, k, v, dense_split=split)
    check_layer_fp8(wl, q, k, v, out)


def test_strided_token_major_layout():
    wl = W.small(L=450, D=64, H=5, seed=41)
    q, k, v = _cuda(W.make_qkv(wl))
    qs, ks, vs = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (q, k, v))
    out = torch.full_like(qs, float("nan"))
    run_fp8(wl, qs, ks, vs, out=out)
    check_layer_fp8(wl, q, k, v, out)


def test_workspace_validation():
    wl = W.small(L=300, D=64, H=5, seed=71)
    q, k, v = _cuda(W.make_qkv(wl))
    desc = svd.desc_of(q)
    ws = torch.empty(svd.svd_plan_workspace_bytes(desc, wl.strategy_table, wl.pattern_params), dtype=torch.uint8, device=DEV)
    plan = svd.svd_plan_create(desc, wl.strategy_table, wl.pattern_params, workspace=ws)
    out = torch.full_like(q, 3.0)
    need = svd.svd_fp8_workspace_bytes(desc)
    assert need == 2 * wl.B * wl.H * 384 * 64
    ws8 = torch.empty(need + 256, dtype=torch.uint8, device=DEV)
    for bad in (ws8[: need - 1], ws8[16: 16 + need]):      # too small, misaligned
        with pytest.raises(svd.SvdError) as e:
            svd.svd_attn_forward_fp8(plan, q, k, v, out, bad)
        assert e.value.status == 8
    torch.cuda.synchronize()
    assert (out == 3.0).all()
    plan.close()


def test_group_entry_point_matches_the_layer_call():
    wl = W.small(L=700, D=128, H=10, seed=81, B=2)
    q, k, v = _cuda(W.make_qkv(wl))
    want, _ = run_fp8(wl, q, k, v)
    desc = svd.desc_of(q)
    ws = torch.empty(svd.svd_plan_workspace_bytes(desc, wl.strategy_table, wl.pattern_params), dtype=torch.uint8, device=DEV)
    plan = svd.svd_plan_create(desc, wl.strategy_table, wl.pattern_params, workspace=ws)
    ws8 = torch.empty(svd.svd_fp8_workspace_bytes(desc), dtype=torch.uint8, device=DEV)
    out = torch.full_like(q, float("nan"))
    for gi in range(len(plan.groups())):
        svd.svd_attn_forward_fp8_group(plan, gi, q, k, v, out, ws8)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), want.view(torch.int16))
    with pytest.raises(svd.SvdError) as e:
        svd.svd_attn_forward_fp8_group(plan, len(plan.groups()), q, k, v, out, ws8)
    assert e.value.status == 2
    plan.close()


@pytest.mark.parametrize("name", ["cogvideox1.5", "hunyuanvideo", "wan2.1"])
def test_benchmark_shape_sampled_rows_and_closed_form(name):
    """The FP8 path at the benchmark shapes, in the launch configuration bench.py
    times with --precision fp8: sampled rows of every head against the FP8 oracle,
    every row of one head per mode against the zero-query closed form."""
    from test_gpu_full_size import _windowed_means
    wl = W.BY_NAME[name]()
    q, k, v = (t.to(DEV) for t in W.make_qkv(wl))
    out, _ = run_fp8(wl, q, k, v)
    assert torch.isfinite(out.float()).all()
    rows = W.sample_rows(wl, n_random=24)
    bq, _ = svd.svd_default_blocks(wl.D)
    rows = np.unique(np.concatenate([rows, np.arange(max(0, wl.L - 2 * bq - 3), wl.L, 61)]))
    check_layer_fp8(wl, q, k, v, out, rows=rows)
    for h in range(wl.H):
        if wl.strategy_table[h] == W.SKIP:
            assert not out[0, h].view(torch.int16).any()
    out0, _ = run_fp8(wl, torch.zeros_like(q), k, v)
    for mode in (W.DENSE, W.DIAG, W.MULTIDIAG, W.VSTRIPE):
        h = int(np.nonzero(wl.strategy_table == mode)[0][0])
        want = _windowed_means(F8.quantise_v(f64(v[0, h].cpu())), mode, wl.pattern_params[h], wl.L)
        assert_close(f64(out0[0, h].cpu()), want, f"fp8 {name} zero-q head {h} mode {mode}")


@pytest.mark.parametrize("D", [64, 128])
def test_wide_bands_fp8_walks_the_small_tile_lists(D):
    """Band groups that the bf16 kernels run on the large query tile (wide bands): the FP8 path takes the small-tile
    lists the plan keeps beside them.  Grouped launches asked for explicitly, so that the bf16 lists stay large."""
    L = 2500
    table = np.asarray([W.DIAG, W.MULTIDIAG, W.DENSE, W.DIAG], dtype=np.int32)
    params = [{"half_width": 1100, "offsets": (0,), "cols": ()}, {"half_width": 380, "offsets": (-900, 0, 900), "cols": ()},
              {"half_width": 0, "offsets": (), "cols": ()}, {"half_width": 1100, "offsets": (0,), "cols": ()}]
    wl = W.Workload("wide-bands", -1, 1, 4, L, D, 500, 5, 0, table, params, 77)
    q, k, v = _cuda(W.make_qkv(wl))
    desc = svd.desc_of(q)
    ws = torch.empty(svd.svd_plan_workspace_bytes(desc, table, params, single_launch=2), dtype=torch.uint8, device=DEV)
    plan = svd.svd_plan_create(desc, table, params, workspace=ws, single_launch=2)
    bq, _ = svd.svd_default_blocks(D)
    assert all(g["block_q"] == bq for g in plan.groups())
    assert plan.work_fp8()["computed_tiles"] != plan.work()["computed_tiles"]
    ws8 = torch.full((svd.svd_fp8_workspace_bytes(desc),), 0x7f, dtype=torch.uint8, device=DEV)
    out = torch.full_like(q, float("nan"))
    svd.svd_attn_forward_fp8(plan, q, k, v, out, ws8)
    torch.cuda.synchronize()
    check_layer_fp8(wl, q, k, v, out)
    out16 = torch.full_like(q, float("nan"))
    svd.svd_attn_forward_planned(plan, q, k, v, out16)
    torch.cuda.synchronize()
    from parity_util import check_layer
    check_layer(wl, q, k, v, out16)
    plan.close()
