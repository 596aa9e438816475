#!/usr/bin/env python3
"""Benchmark of the sparse attention layer on one MI355X.

A step is one forward pass of the whole layer: the fused launch of every mode
group of the per-head strategy table plus the zero fill of skipped heads, on
Q/K/V already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
                    [--workload all|cogvideox1.5|hunyuanvideo|hunyuanvideo+text|wan2.1|stack|search|rearranged]
                    [--precision bf16|fp8]

The default, --workload all, times the HunyuanVideo-shaped layer (the largest
single-GPU configuration) as the headline and, in the same run, the
CogVideoX1.5- and Wan2.1-shaped layers and the 40-layer stack as sub-records
under "other_workloads", each with its own roofline, CPU-oracle leg and check
against the oracle; a calibration leg measures what the chip sustains on a loop
of bf16 matrix instructions and on a streaming copy.

--precision fp8 times the FP8 (E4M3) variant of the same layer: a step then also
contains the quantisation pre-pass of K and V (the inputs stay bf16).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
FP8_MFMA_PEAK_TFLOPS = 5000.0    # MI355X dense fp8 matrix peak
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")
KERNEL_SOURCES = ("attn_kernels.hip", "attn_kernels.h", "fp8_kernels.hip", "api.cpp")


def kernel_source_stamp():
    """Short hash of the kernel and launch sources: a traffic record is only valid for the sources it was measured on."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2506_03065_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def recorded_traffic(precision, workload, group):
    """HBM bytes per launch of a group's kernels from profiles/traffic.json (written by
    `python -m paper_2506_03065_amd.traffic_record` from two rocprofv3 --pmc runs, FETCH_SIZE and
    WRITE_SIZE, scaled by what the same counters read for the library's copy probe).  Counters cannot be
    read from inside this process.  None when there is no record or it was taken on other kernel sources."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None, "no record"
    entry = rec.get("records", {}).get(precision, {}).get(workload, {}).get(group)
    if entry is None:
        return None, "no record"
    if entry.get("kernel_source_stamp") != kernel_source_stamp():
        return None, "record is stale (kernel sources changed since the counter run)"
    return entry.get("bytes"), entry.get("source")


MODE_NAMES = {0: "dense", 1: "skip", 2: "diagonal", 3: "multi-diagonal", 4: "vertical-stripe"}


def gpu_time_ms(fn, reps, warmup, torch):
    """Average milliseconds of fn() over reps, HIP events on the current stream."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(reps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / reps


def cpu_baseline(wl, q, k, v, out, budget_s, torch, np, fp8=False):
    """The oracle on a bounded row sample of every head, on the host cores; the
    same rows are used to check the GPU output."""
    from oracle import sparse_attention as O
    from oracle import fp8_attention as F8
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    gen = np.random.default_rng(wl.seed)
    n_rows = 512
    rows = np.sort(gen.choice(wl.L, size=n_rows, replace=False))
    spent, heads_done, max_err, sum_err, n_err = 0.0, 0, 0.0, 0.0, 0
    f64 = lambda t: t.cpu().to(torch.float64).numpy()
    b = wl.B - 1      # the last batch element
    for h in range(wl.H):
        mode, p = int(wl.strategy_table[h]), wl.pattern_params[h]
        qh, kh, vh = f64(q[b, h][torch.as_tensor(rows)]), f64(k[b, h]), f64(v[b, h])
        full_q = np.zeros((wl.L, wl.D))
        full_q[rows] = qh
        t0 = time.perf_counter()
        if fp8:
            want = F8.attention_head_fp8(full_q, kh, vh, mode, p, rows=rows)
        else:
            want = O.attention_head(full_q, kh, vh, mode, p, rows=rows)
        spent += time.perf_counter() - t0
        heads_done += 1
        got = f64(out[b, h][torch.as_tensor(rows)])
        err = np.abs(got - want)
        max_err, sum_err, n_err = max(max_err, float(err.max())), sum_err + float(err.sum()), n_err + err.size
        if spent > budget_s:
            break
    layer_s = spent / heads_done * wl.H * (wl.L / n_rows) * wl.B
    return {"value": layer_s * 1e3, "unit": "ms per layer (extrapolated from the sample)", "cores": int(threads),
            "kind": "oracle", "measured_s": round(spent, 3),
            "sample": f"{n_rows} seeded query rows x {heads_done} of {wl.H} heads, float64 numpy, inputs "
                      f"already widened; scaled by L/rows and H/heads"}, max_err, sum_err / max(n_err, 1)


def run_stack(args, torch, np, svd, W, cpu_seconds=None, calib=None, dense_reps=1):
    """The 40-layer stack at the Wan2.1-like shape: one plan per layer, built once;
    a step is one forward pass of all 40 attention layers (the same Q/K/V serve
    every layer: kernel time does not depend on the values)."""
    dev = "cuda:0"
    n_layers = 40
    fp8 = args.precision == "fp8"
    layers = [W.stack_layer(i, n_layers) for i in range(n_layers)]
    wl0 = layers[0]
    q, k, v = (t.to(dev) for t in W.make_qkv(wl0))
    out = torch.empty_like(q)
    desc = svd.desc_of(q)
    t0 = time.perf_counter()
    plans, spaces = [], []
    for wl in layers:
        ws = torch.empty(svd.svd_plan_workspace_bytes(desc, wl.strategy_table, wl.pattern_params,
                                                      single_launch=args.single_launch),
                         dtype=torch.uint8, device=dev)
        plans.append(svd.svd_plan_create(desc, wl.strategy_table, wl.pattern_params, workspace=ws,
                                         single_launch=args.single_launch))
        spaces.append(ws)
    plan_ms = (time.perf_counter() - t0) * 1e3

    if fp8:
        ws8 = torch.empty(svd.svd_fp8_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        layer_fwd = lambda plan: svd.svd_attn_forward_fp8(plan, q, k, v, out, ws8)
    else:
        layer_fwd = lambda plan: svd.svd_attn_forward_planned(plan, q, k, v, out)

    def step():
        for plan in plans:
            layer_fwd(plan)
    t_warm = time.perf_counter()
    while time.perf_counter() - t_warm < 1.5:
        layer_fwd(plans[-1])
        torch.cuda.synchronize()
    steps, warmup = max(1, min(args.steps, 3)), max(1, min(args.warmup, 1))
    ms_per_step = gpu_time_ms(step, steps, warmup, torch)
    per_layer = [gpu_time_ms(lambda p=p: layer_fwd(p), 1, 0, torch) for p in plans]
    dense_out = torch.empty_like(q)
    dense_ms = gpu_time_ms(lambda: svd.svd_dense_attn_forward(q, k, v, dense_out), max(1, dense_reps), 1, torch)
    del dense_out
    work = [p.work() for p in plans]
    computed = sum(w["computed_flops"] for w in work)
    # dominant kernel of the stack: the dense group of the first layer (most dense heads)
    g0 = [gi for gi, g in enumerate(plans[0].groups()) if g["mode"] == 0]
    roofline = None
    if g0:
        run0 = ((lambda: svd.svd_attn_forward_fp8_group(plans[0], g0[0], q, k, v, out, ws8)) if fp8 else
                (lambda: svd.svd_attn_forward_group(plans[0], g0[0], q, k, v, out)))
        ms0 = gpu_time_ms(run0, 3, 1, torch)
        tf0 = plans[0].work(g0[0])["computed_flops"] / 1e9 / ms0
        peak = FP8_MFMA_PEAK_TFLOPS if fp8 else BF16_MFMA_PEAK_TFLOPS
        roofline = {"bound": "mfma", "kernel": f"{'attn_fwd_fp8_kernel' if fp8 else 'attn_fwd_kernel'}[dense group of layer 0]",
                    "achieved": round(tf0, 1), "peak": peak, "unit": "TFLOP/s", "frac": round(tf0 / peak, 4), "traffic": None}
        if plans[0].single_launch() and not fp8:
            # every layer is one launch of the layer kernel: the step is the dominant kernel, 40 times over
            tf = computed / 1e9 / ms_per_step
            roofline = {"bound": "mfma", "kernel": "attn_layer_kernel (one launch per layer, the whole step)",
                        "achieved": round(tf, 1), "peak": peak, "unit": "TFLOP/s", "frac": round(tf / peak, 4), "traffic": None}
        add_measured_peak(roofline, calib, fp8)
    dense_flops = wl0.dense_flops * n_layers
    cpu, max_err, mean_err = None, None, None
    cpu_seconds = args.cpu_seconds if cpu_seconds is None else cpu_seconds
    if cpu_seconds > 0:
        mid = layers[n_layers // 2]
        layer_fwd(plans[n_layers // 2])
        torch.cuda.synchronize()
        cpu, max_err, mean_err = cpu_baseline(mid, q, k, v, out, cpu_seconds, torch, np, fp8=fp8)
        cpu["value"] *= n_layers
        cpu["sample"] += f"; layer {n_layers // 2} of the stack, times {n_layers} layers"
    dense_heads = [int((wl.strategy_table == 0).sum()) for wl in layers]
    result = {
        "metric": "sparse-attn layer latency" + (" (FP8 variant, pre-pass included)" if fp8 else ""), "value": round(ms_per_step, 3), "unit": "ms", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "fp8-e4m3 (fp32 accumulation)" if fp8 else "bf16",
        "data": "synthetic",
        "config": {"workload": "layer-stack (40 layers, Wan2.1-like shape)", "precision": args.precision, "B": wl0.B, "H": wl0.H, "L": wl0.L,
                   "D": wl0.D, "dense_heads_first_last": [dense_heads[0], dense_heads[-1]],
                   "launch_form": "layer kernel" if plans[0].single_launch() else "grouped launches"},
        "computed_tile_tflops": round(computed / 1e9 / ms_per_step, 1),
        "computed_tile_frac_of_bf16_peak": round(computed / 1e9 / ms_per_step / BF16_MFMA_PEAK_TFLOPS, 4),
        "computed_tile_frac_of_measured_mfma_peak": round(computed / 1e9 / ms_per_step / calib["measured_mfma_peak_tflops"], 4) if calib and not fp8 else None,
        "dense_all_heads_ms": round(dense_ms * n_layers, 1),
        "speedup_vs_dense_kernel": round(dense_ms * n_layers / ms_per_step, 3),
        "flop_reduction_block_level": round(dense_flops / computed, 3),
        "per_layer_ms": [round(x, 2) for x in per_layer],
        "plan_create_ms": round(plan_ms, 1),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "check_vs_oracle": {"max_abs_err": max_err, "mean_abs_err": mean_err, "layer": n_layers // 2},
    }
    for plan in plans:
        plan.close()
    return result


def run_search(args, torch, np, svd, W):
    """One layer of the offline search at the CogVideoX1.5-like shape: all five
    modes on the same Q/K/V, four per-head MSE reductions, selection, assembly."""
    dev = "cuda:0"
    wl = W.BY_NAME["cogvideox1.5"]()
    q, k, v = (t.to(dev) for t in W.make_qkv(wl))
    out = torch.empty_like(q)
    desc = svd.desc_of(q)
    by_mode = {m: [None] * wl.H for m in (2, 3, 4)}
    first = {m: next(p for h, p in enumerate(wl.pattern_params) if wl.strategy_table[h] == m) for m in (2, 3)}
    vert = [p for h, p in enumerate(wl.pattern_params) if wl.strategy_table[h] == 4]
    for h in range(wl.H):
        by_mode[2][h], by_mode[3][h], by_mode[4][h] = first[2], first[3], vert[h % len(vert)]
    ws = torch.empty(svd.svd_search_layer_workspace_bytes(desc, by_mode), dtype=torch.uint8, device=dev)
    lam, eps = 0.5, 1.0
    table, loss = svd.svd_search_layer(q, k, v, by_mode, lam, eps, out, ws)      # warm-up
    steps = max(1, min(args.steps, 3))
    t0 = time.perf_counter()
    for _ in range(steps):
        table, loss = svd.svd_search_layer(q, k, v, by_mode, lam, eps, out, ws)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps       # the call synchronises: wall clock is the time
    # the reduction kernel on its own: reads two tensors once
    mse = torch.empty(wl.H, dtype=torch.float32, device=dev)
    mws = torch.empty(max(svd.svd_head_mse_workspace_bytes(desc), 4), dtype=torch.uint8, device=dev)
    other = torch.empty_like(q).copy_(q)
    mse_ms = gpu_time_ms(lambda: svd.svd_head_mse(out, other, mse, mws), 20, 3, torch)
    nbytes = 2.0 * q.numel() * 2
    sel_ms = gpu_time_ms(lambda: svd.svd_select_heads([q, k, v, other, out], table, out), 20, 3, torch)
    result = {
        "metric": "search-step latency (five modes + four reductions + selection, one layer)",
        "value": round(ms_per_step, 3), "unit": "ms", "n_gpus": 1, "steps": steps, "warmup": 1,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "search step, " + wl.name, "B": wl.B, "H": wl.H, "L": wl.L, "D": wl.D,
                   "lambda": lam, "epsilon": eps},
        "table_counts": {MODE_NAMES[m]: int((table == m).sum()) for m in range(5)},
        "head_mse_ms": round(mse_ms, 4), "select_heads_ms": round(sel_ms, 4),
        "roofline": {"bound": "hbm", "kernel": "head_mse_partial_kernel", "achieved": round(nbytes / 1e6 / mse_ms, 1),
                     "peak": 8000.0, "unit": "GB/s", "frac": round(nbytes / 1e6 / mse_ms / 8000.0, 4), "traffic": None},
        "cpu_baseline": None,
    }
    print(json.dumps(result))


def run_rearranged(args, torch, np, svd, W):
    """Section 4.1.2: attention between nearby positions of all frames, computed (a)
    as the multi-diagonal mode with every frame offset on the frame-major order and
    (b) as the diagonal mode on rearranged (position-major) tokens: three
    rearrangements in, one out, and (c) as multi-diagonal heads in rearranged form,
    whose kernel reaches the rows through a row map (the timed step).  Wan2.1-like
    shape, 8 heads."""
    dev = "cuda:0"
    H, D, N, F, w = 8, 128, 3600, 21, 40
    L = N * F
    gen = torch.Generator().manual_seed(20250603)
    q, k, v = (torch.randn(1, H, L, D, generator=gen).to(torch.bfloat16).to(dev) for _ in range(3))
    out = torch.empty_like(q)
    desc = svd.desc_of(q)

    def planned(table, params):
        ws = torch.empty(svd.svd_plan_workspace_bytes(desc, table, params, single_launch=args.single_launch),
                         dtype=torch.uint8, device=dev)
        return svd.svd_plan_create(desc, table, params, workspace=ws, single_launch=args.single_launch), ws
    multi, ws_a = planned(np.full(H, W.MULTIDIAG, dtype=np.int32),
                          [{"half_width": w, "offsets": tuple(kk * N for kk in range(-(F - 1), F))}] * H)
    Wd = w * F + F - 1
    diag, ws_b = planned(np.full(H, W.DIAG, dtype=np.int32), [{"half_width": Wd}] * H)
    # (c) the same kept set as multi-diagonal heads in rearranged form: rows reached through a row map, no copies
    fused, ws_c = planned(np.full(H, W.MULTIDIAG, dtype=np.int32), [{"half_width": Wd, "rearranged": (0, N, F)}] * H)
    qp, kp, vp, op = (torch.empty_like(q) for _ in range(4))

    def step():
        for src, dst in ((q, qp), (k, kp), (v, vp)):
            svd.svd_rearrange_tokens(src, dst, 0, N, F)
        svd.svd_attn_forward_planned(diag, qp, kp, vp, op)
        svd.svd_rearrange_tokens(op, out, 0, N, F, inverse=True)
    t_warm = time.perf_counter()
    while time.perf_counter() - t_warm < 1.5:
        step()
        torch.cuda.synchronize()
    ms = gpu_time_ms(step, args.steps, args.warmup, torch)
    ms_move = gpu_time_ms(lambda: svd.svd_rearrange_tokens(q, qp, 0, N, F), args.steps, 1, torch)
    ms_back = gpu_time_ms(lambda: svd.svd_rearrange_tokens(op, out, 0, N, F, inverse=True), args.steps, 1, torch)
    ms_diag = gpu_time_ms(lambda: svd.svd_attn_forward_planned(diag, qp, kp, vp, op), args.steps, 1, torch)
    ms_multi = gpu_time_ms(lambda: svd.svd_attn_forward_planned(multi, q, k, v, out), max(2, args.steps // 2), 1, torch)
    out_copy = out.clone()
    step()
    torch.cuda.synchronize()
    out_copy.copy_(out)
    ms_fused = gpu_time_ms(lambda: svd.svd_attn_forward_planned(fused, q, k, v, out), args.steps, args.warmup, torch)
    torch.cuda.synchronize()
    max_diff = float((out.float() - out_copy.float()).abs().max())
    ws8 = torch.empty(svd.svd_fp8_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    ms_fused8 = gpu_time_ms(lambda: svd.svd_attn_forward_fp8(fused, q, k, v, out, ws8), args.steps, args.warmup, torch)
    tensor_bytes = q.numel() * 2
    wd, wm = diag.work(), multi.work()
    result = {
        "metric": "position-window attention latency (multi-diagonal heads in rearranged form, rows through a row map)",
        "value": round(ms_fused, 4), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_fused, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "rearranged window, Wan2.1-like shape", "B": 1, "H": H, "L": L, "D": D,
                   "frame_tokens": N, "frames": F, "position_half_width": w, "band_half_width": Wd},
        "fp8_row_map_ms": round(ms_fused8, 4),
        "copy_path_ms": round(ms, 4),
        "max_abs_diff_row_map_vs_copy_path": max_diff,
        "row_map_tflops": round(wd["computed_flops"] / 1e9 / ms_fused, 1),
        "rearrange_one_tensor_ms": round(ms_move, 4), "rearrange_back_ms": round(ms_back, 4),
        "diagonal_on_rearranged_ms": round(ms_diag, 4),
        "diagonal_tflops": round(wd["computed_flops"] / 1e9 / ms_diag, 1),
        "computed_tiles": wd["computed_tiles"],
        "multi_diagonal_all_offsets_ms": round(ms_multi, 4),
        "multi_diagonal_all_offsets_tiles": wm["computed_tiles"],
        "speedup_vs_multi_diagonal_lists": round(ms_multi / ms_fused, 3),
        "roofline": {"bound": "hbm", "kernel": "rearrange_tokens_kernel", "achieved": round(2 * tensor_bytes / 1e6 / ms_move, 1),
                     "peak": 8000.0, "unit": "GB/s", "frac": round(2 * tensor_bytes / 1e6 / ms_move / 8000.0, 4),
                     "traffic": None},
        "cpu_baseline": None,
        "note": "the two paths keep different pairs at frame edges: diagonals on the frame-major index wrap from "
                "the end of a frame into the next one, the window in position-major order does not",
    }
    print(json.dumps(result))
    multi.close()
    diag.close()
    fused.close()



def add_measured_peak(roofline, calib, fp8):
    """frac_of_measured_peak beside frac: the same rate against what a loop of nothing but bf16 matrix
    instructions sustained in this run (the FP8 kernels are not put against a bf16 loop)."""
    if roofline is None or not calib or fp8 or roofline.get("unit") != "TFLOP/s":
        return
    roofline["measured_peak"] = calib["measured_mfma_peak_tflops"]
    roofline["frac_of_measured_peak"] = round(roofline["achieved"] / calib["measured_mfma_peak_tflops"], 4)


def calibrate(torch, svd):
    """Measured ceilings: the matrix-instruction loop (two work-groups of eight waves per compute unit and
    round, about 60 ms) and the library's streaming copy of 1 GiB, HIP events on the launch stream."""
    dev = "cuda:0"
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    wgs, iters = 2 * n_cu, 20000
    scratch = torch.empty(wgs * 512, dtype=torch.float32, device=dev)
    flops = svd.svd_probe_mfma(scratch, iters, wgs)
    t_warm = time.perf_counter()
    while time.perf_counter() - t_warm < 1.0:      # the sustained rate, not the first launch's boost clock
        svd.svd_probe_mfma(scratch, iters, wgs)
        torch.cuda.synchronize()
    ms = gpu_time_ms(lambda: svd.svd_probe_mfma(scratch, iters, wgs), 5, 1, torch)
    src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    ms_copy = gpu_time_ms(lambda: svd.svd_probe_copy(src, dst), 5, 2, torch)
    nbytes = 2.0 * src.numel() * 4
    del src, dst, scratch
    torch.cuda.empty_cache()
    return {"measured_mfma_peak_tflops": round(flops / 1e9 / ms, 1),
            "mfma_probe": f"v_mfma_f32_32x32x16_bf16 loop, {wgs} work-groups x 512 threads, {iters} x 8 per wave, {ms:.2f} ms",
            "measured_hbm_gbs": round(nbytes / 1e6 / ms_copy, 1),
            "copy_probe": f"1 GiB read + 1 GiB written, {ms_copy:.3f} ms",
            "compute_units": n_cu}


def measure_layer(wl, args, torch, np, svd, cpu_seconds, dense_reps, calib=None):
    """One layer workload: the timed steps, the per-group launches, the dense baseline, the CPU-oracle leg."""
    dev = "cuda:0"
    fp8 = args.precision == "fp8"
    from paper_2506_03065_amd import workloads as W
    t0 = time.perf_counter()
    q, k, v = (t.to(dev) for t in W.make_qkv(wl))
    if args.layout == "blhd":      # token-major storage, seen through a [B,H,L,D] view
        q, k, v = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (q, k, v))
    gen_s = time.perf_counter() - t0
    out = torch.empty_like(q)
    desc = svd.desc_of(q)

    t0 = time.perf_counter()
    ws = torch.empty(svd.svd_plan_workspace_bytes(desc, wl.strategy_table, wl.pattern_params,
                                                  single_launch=args.single_launch),
                     dtype=torch.uint8, device=dev)
    plan = svd.svd_plan_create(desc, wl.strategy_table, wl.pattern_params, workspace=ws,
                               single_launch=args.single_launch)
    plan_ms = (time.perf_counter() - t0) * 1e3
    work = plan.work()
    if fp8:      # the FP8 path walks small-tile lists in every band group
        work = dict(work, **plan.work_fp8())

    # ---- the timed region: K full-layer steps ----
    step16 = lambda: svd.svd_attn_forward_planned(plan, q, k, v, out)
    step = step16
    if fp8:
        ws8 = torch.empty(svd.svd_fp8_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        step = lambda: svd.svd_attn_forward_fp8(plan, q, k, v, out, ws8)
    t_warm = time.perf_counter()          # bring the clocks to their sustained level before the W warm-up steps
    while time.perf_counter() - t_warm < 1.5:
        step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(args.steps):
        step()
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_per_step = start.elapsed_time(stop) / args.steps

    # ---- the same layer through the other launch form (single launch <-> grouped launches) ----
    other = None
    if not fp8:
        alt_form = 2 if plan.single_launch() else 1      # grouped launches <-> the layer kernel
        ws_alt = torch.empty(svd.svd_plan_workspace_bytes(desc, wl.strategy_table, wl.pattern_params,
                                                          single_launch=alt_form),
                             dtype=torch.uint8, device=dev)
        plan_alt = svd.svd_plan_create(desc, wl.strategy_table, wl.pattern_params, workspace=ws_alt,
                                       single_launch=alt_form)
        alt_ms = gpu_time_ms(lambda: svd.svd_attn_forward_planned(plan_alt, q, k, v, out), args.steps, args.warmup, torch)
        other = {"form": "layer kernel" if plan_alt.single_launch() else "grouped launches",
                 "ms": round(alt_ms, 4),
                 "computed_tile_frac_of_bf16_peak": round(plan_alt.work()["computed_flops"] / 1e9 / alt_ms / BF16_MFMA_PEAK_TFLOPS, 4),
                 "dense_split": plan_alt.dense_split()}
        plan_alt.close()
        del ws_alt

    # ---- per-group kernels (one launch each), HIP events on the launch stream ----
    groups = []
    for gi, g in enumerate(plan.groups()):
        gw = plan.work_fp8(gi) if fp8 else plan.work(gi)
        run_group = ((lambda: svd.svd_attn_forward_fp8_group(plan, gi, q, k, v, out, ws8)) if fp8 else
                     (lambda: svd.svd_attn_forward_group(plan, gi, q, k, v, out)))
        ms = gpu_time_ms(run_group, max(3, args.steps // 2), 1, torch)
        groups.append({"mode": MODE_NAMES[g["mode"]], "heads": len(g["heads"]), "ms": round(ms, 4),
                       "computed_tflop": round(gw["computed_flops"] / 1e12, 4),
                       "tflops": round(gw["computed_flops"] / 1e9 / ms, 1) if ms > 0 else None,
                       "tiles": gw["computed_tiles"]})
    compute_groups = [g for g in groups if g["mode"] != "skip"]
    dom = max(compute_groups, key=lambda g: g["ms"])
    peak = FP8_MFMA_PEAK_TFLOPS if fp8 else BF16_MFMA_PEAK_TFLOPS
    traffic, traffic_source = recorded_traffic(args.precision, wl.name, dom["mode"])
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    kname = "attn_fwd_fp8_kernel" if fp8 else "attn_fwd_kernel"
    dom_g = next(g for g in plan.groups() if MODE_NAMES[g["mode"]] == dom["mode"])
    dom_threads = 64 * (8 if dom_g["block_q"] == svd.svd_default_blocks(wl.D)[0] else 4)
    dom_items = -(-wl.L // dom_g["block_q"]) * len(dom_g["heads"]) * wl.B * (plan.dense_split() if dom["mode"] == "dense" else 1)
    dispatches = [{"kernel": kname, "grid_size": -(-dom_items // 8) * 8 * dom_threads}]
    if dom["mode"] == "dense" and plan.dense_split() > 1:
        dispatches.append({"kernel": "combine_partials_kernel"})
    if fp8:
        dispatches.append({"kernel": "quantise_kv_kernel", "grid_size": (-(-wl.L // 128) * 128 // 64) * len(dom_g["heads"]) * wl.B * 256})
    roofline = {"bound": "mfma", "kernel": f"{kname}[{dom['mode']} group]",
                "achieved": dom["tflops"], "peak": peak, "unit": "TFLOP/s", "frac": round(dom["tflops"] / peak, 4),
                "traffic": traffic, "traffic_source": traffic_source, "traffic_key": dom["mode"], "dispatches": dispatches}
    if plan.single_launch() and not fp8:
        # the step IS the dominant kernel: the layer kernel (with the dense kernel's head start ahead of it, and
        # the 5 us fill of the queue positions); algorithmic FLOPs = the plan's listed tiles
        tf = work["computed_flops"] / 1e9 / ms_per_step
        traffic, traffic_source = recorded_traffic(args.precision, wl.name, "layer")
        dispatches = [{"kernel": "attn_layer_kernel"}]
        n_dense = int((wl.strategy_table == 0).sum())
        bq = svd.svd_default_blocks(wl.D)[0]
        head_start = (-(-wl.L // bq) * n_dense * wl.B) // n_cu * n_cu      # whole rounds of one dense item per compute unit
        if head_start and plan.launch_form() == 3:
            dispatches.append({"kernel": f"attn_fwd_kernel<{wl.D}, 8, 1, {svd.svd_default_blocks(wl.D)[1]}, 2, 0>",
                               "grid_size": -(-head_start // 8) * 8 * 512})
        roofline = {"bound": "mfma", "kernel": "attn_layer_kernel" + (" + attn_fwd_kernel[dense head start]" if plan.launch_form() == 3 else "") + " (the whole step)",
                    "achieved": round(tf, 1), "peak": peak, "unit": "TFLOP/s", "frac": round(tf / peak, 4),
                    "traffic": traffic, "traffic_source": traffic_source, "traffic_key": "layer", "dispatches": dispatches}
    add_measured_peak(roofline, calib, fp8)
    bf16_ms = gpu_time_ms(step16, max(3, args.steps // 2), 1, torch) if fp8 else None

    # ---- in-house dense kernel on all heads: the speed-up baseline ----
    dense_ms = None
    if dense_reps > 0:
        dense_out = torch.empty_like(q)
        dense_ms = gpu_time_ms(lambda: svd.svd_dense_attn_forward(q, k, v, dense_out), dense_reps, 1 if dense_reps > 1 else 0, torch)
        del dense_out
    step()
    torch.cuda.synchronize()

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        svd.svd_probe_copy(src, dst)      # the library's streaming copy: reads 2^30 B, writes 2^30 B
        torch.cuda.synchronize()
        del src, dst

    cpu, max_err, mean_err = (None, None, None)
    if cpu_seconds > 0:
        cpu, max_err, mean_err = cpu_baseline(wl, q, k, v, out, cpu_seconds, torch, np, fp8=fp8)

    dense_flops = wl.dense_flops
    computed_tflops = work["computed_flops"] / 1e9 / ms_per_step
    text = int(wl.pattern_params[int((wl.strategy_table >= 2).argmax())].get("text_tokens", 0)) if (wl.strategy_table >= 2).any() else 0
    result = {
        "metric": "sparse-attn layer latency" + (" (FP8 variant, pre-pass included)" if fp8 else ""),
        "value": round(ms_per_step, 4),
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp8-e4m3 (fp32 accumulation)" if fp8 else "bf16",
        "data": "synthetic",
        "config": {"workload": wl.name, "precision": args.precision, "layout": args.layout,
                   "text_tokens_with_dense_borders": text, "B": wl.B, "H": wl.H, "L": wl.L, "D": wl.D,
                   "block_q": svd.svd_default_blocks(wl.D)[0], "block_k": svd.svd_default_blocks(wl.D)[1],
                   "dense_split": plan.dense_split(),
                   "launch_form": {0: "grouped launches", 1: "layer kernel (the whole layer in one launch)",
                                   3: "layer kernel after a dense head start"}[plan.launch_form()],
                   "heads_by_mode": {MODE_NAMES[m]: int((wl.strategy_table == m).sum()) for m in range(5)}},
        "wall_ms_per_step": round(wall_ms, 4),
        "dense_equiv_tflops": round(dense_flops / 1e9 / ms_per_step, 1),
        "computed_tile_tflops": round(computed_tflops, 1),
        "computed_tile_frac_of_bf16_peak": round(computed_tflops / BF16_MFMA_PEAK_TFLOPS, 4),
        "computed_tile_frac_of_measured_mfma_peak": round(computed_tflops / calib["measured_mfma_peak_tflops"], 4) if calib and not fp8 else None,
        "computed_tile_frac_of_fp8_peak": round(computed_tflops / FP8_MFMA_PEAK_TFLOPS, 4) if fp8 else None,
        "bf16_same_plan_ms": round(bf16_ms, 4) if bf16_ms else None,
        "speedup_vs_bf16_sparse": round(bf16_ms / ms_per_step, 3) if bf16_ms else None,
        "computed_tflop_per_layer": round(work["computed_flops"] / 1e12, 3),
        "dense_tflop_per_layer": round(dense_flops / 1e12, 3),
        "flop_reduction_block_level": round(dense_flops / work["computed_flops"], 3),
        "flop_reduction_element_level": round(float(wl.B * wl.H) * wl.L ** 2 / work["kept_pairs"], 3),
        "dense_all_heads_ms": round(dense_ms, 3) if dense_ms else None,
        "dense_all_heads_tflops": round(dense_flops / 1e9 / dense_ms, 1) if dense_ms else None,
        "speedup_vs_dense_kernel": round(dense_ms / ms_per_step, 3) if dense_ms else None,
        "plan_create_ms": round(plan_ms, 2),
        "input_gen_s": round(gen_s, 1),
        "other_launch_form": other,
        "groups": groups,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "check_vs_oracle": {"max_abs_err": max_err, "mean_abs_err": mean_err},
    }
    plan.close()
    del q, k, v, out, ws
    torch.cuda.empty_cache()
    return result


def brief(rec):
    """The sub-record of a workload that is not the headline."""
    keys = ("config", "ms_per_step", "steps", "computed_tile_tflops", "computed_tile_frac_of_bf16_peak",
            "computed_tile_frac_of_measured_mfma_peak", "dense_all_heads_ms", "speedup_vs_dense_kernel",
            "flop_reduction_block_level", "flop_reduction_element_level", "other_launch_form", "groups", "roofline", "cpu_baseline",
            "check_vs_oracle", "plan_create_ms")
    out = {"ms": rec["ms_per_step"]}
    out.update({k: rec[k] for k in keys if k in rec})
    return out


PAPER_CONTEXT = ("end-to-end speedups 1.76x/1.85x (A800) and 1.58x (H800) in the paper's Table 2; "
                 "no kernel-level numbers are published")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="all",
                    help="all (default): the HunyuanVideo-shaped layer as the headline plus the CogVideoX1.5- and "
                         "Wan2.1-shaped layers and the 40-layer stack as sub-records; or one workload by name")
    ap.add_argument("--precision", default="bf16", choices=["bf16", "fp8"],
                    help="bf16 (the headline metric) or the FP8 E4M3 variant of the same layer")
    ap.add_argument("--layout", default="bhld", choices=["bhld", "blhd"],
                    help="storage order of q, k, v, out: head-major [B,H,L,D] (default) or the model's token-major "
                         "[B,L,H,D] (Eq. 1's head concatenation then needs no copy); the kernels take either through strides")
    ap.add_argument("--batch", type=int, default=None, help="batch size B (default: the workload's, 1); 2 = a CFG pair")
    ap.add_argument("--dense-reps", type=int, default=None,
                    help="timed passes of the all-heads dense baseline (0 = skip; default 2, 1 per layer with --workload all)")
    ap.add_argument("--cpu-seconds", type=float, default=None,
                    help="budget of the CPU-oracle leg (0 = skip; default 25, with --workload all 20 for the headline "
                         "and 8 for each other workload)")
    ap.add_argument("--single-launch", type=int, default=0, choices=[0, 1, 2, 3],
                    help="plan option single_launch: 0 = the library's choice, 1 = the whole layer as one launch, "
                         "2 = one launch per mode group, 3 = one launch with a dense head start")
    ap.add_argument("--no-calibrate", action="store_true",
                    help="skip the calibration leg (matrix-instruction loop and streaming copy)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run the library's streaming copy once (1 GiB read, 1 GiB written) so that a rocprofv3 "
                         "--pmc run of this command holds a dispatch of known HBM traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2506_03065_amd import binding as svd
    from paper_2506_03065_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    svd.lib()   # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    fp8 = args.precision == "fp8"
    if fp8 and args.workload in ("search", "rearranged"):
        print("--precision fp8: this workload is built in bf16 only", file=sys.stderr)
        sys.exit(2)
    if args.batch is not None and args.batch < 1:
        print("--batch must be at least 1", file=sys.stderr)
        sys.exit(2)
    everything = args.workload == "all"
    if args.workload == "search":
        run_search(args, torch, np, svd, W)
        return
    if args.workload == "rearranged":
        run_rearranged(args, torch, np, svd, W)
        return
    calib = None if args.no_calibrate else calibrate(torch, svd)
    cpu_head = args.cpu_seconds if args.cpu_seconds is not None else (20.0 if everything else 25.0)
    cpu_other = args.cpu_seconds if args.cpu_seconds is not None else 8.0
    dense_reps = args.dense_reps if args.dense_reps is not None else (1 if everything else 2)
    if args.workload == "stack":
        result = run_stack(args, torch, np, svd, W, cpu_head, calib, dense_reps)
    else:
        wl = W.BY_NAME["hunyuanvideo" if everything else args.workload]()
        if args.batch is not None:
            wl.B = args.batch
        result = measure_layer(wl, args, torch, np, svd, cpu_head, dense_reps, calib)
    if everything:
        others = {}
        for name in ("cogvideox1.5", "wan2.1"):
            wl = W.BY_NAME[name]()
            if args.batch is not None:
                wl.B = args.batch
            others[name] = brief(measure_layer(wl, args, torch, np, svd, cpu_other, dense_reps, calib))
        others["stack"] = brief(run_stack(args, torch, np, svd, W, cpu_other, calib, dense_reps))
        result["other_workloads"] = others
    result["calibration"] = calib
    result["paper_context"] = PAPER_CONTEXT
    print(json.dumps(result))


if __name__ == "__main__":
    main()
