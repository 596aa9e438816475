"""The tool that turns two rocprofv3 counter runs into profiles/traffic.json, on hand-written counter output:
scaling by the copy probe's dispatch, averaging over dispatches, matching by kernel name part and grid size,
the source stamp that lets bench.py drop a stale record."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = "Kernel_Name,Grid_Size,Counter_Name,Counter_Value\n"


def test_record_from_hand_written_counter_output(tmp_path):
    layer = "void svd::(anonymous namespace)::attn_layer_kernel<128, 64>(svd::LayerLaunch)"
    dense = "void svd::(anonymous namespace)::attn_fwd_kernel<128, 8, 1, 64, 2, 0>(svd::AttnLaunch)"
    copy = "svd::(anonymous namespace)::copy_probe_kernel(HIP_vector_type<unsigned int, 4u> const*, HIP_vector_type<unsigned int, 4u>*, unsigned long)"
    fetch = (HEADER + f'"{layer}",131072,FETCH_SIZE,1000\n"{layer}",131072,FETCH_SIZE,3000\n'
             f'"{dense}",131072,FETCH_SIZE,500\n"{dense}",233472,FETCH_SIZE,99999\n'        # another grid: not matched
             f'"{copy}",2097152,FETCH_SIZE,524288\n')
    write = (HEADER + f'"{layer}",131072,WRITE_SIZE,400\n"{layer}",131072,WRITE_SIZE,600\n'
             f'"{dense}",131072,WRITE_SIZE,100\n"{copy}",2097152,WRITE_SIZE,1048576\n')
    (tmp_path / "fetch.csv").write_text(fetch)
    (tmp_path / "write.csv").write_text(write)
    run = {"config": {"workload": "hunyuanvideo", "precision": "bf16"},
           "roofline": {"traffic_key": "layer",
                        "dispatches": [{"kernel": "attn_layer_kernel"},
                                       {"kernel": "attn_fwd_kernel<128, 8, 1, 64, 2, 0>", "grid_size": 131072}]}}
    (tmp_path / "run.json").write_text("some log line\n" + json.dumps(run) + "\n")
    out = tmp_path / "traffic.json"
    res = subprocess.run([sys.executable, "-m", "paper_2506_03065_amd.traffic_record", "--bench-json", str(tmp_path / "run.json"),
                          "--fetch-csv", str(tmp_path / "fetch.csv"), "--write-csv", str(tmp_path / "write.csv"),
                          "--out", str(out)], capture_output=True, text=True, cwd=ROOT)
    assert res.returncode == 0, res.stderr
    rec = json.loads(out.read_text())["records"]["bf16"]["hunyuanvideo"]["layer"]
    # the copy moved 2^20 KiB each way: FETCH_SIZE reads half of it (factor 2), WRITE_SIZE all of it (factor 1)
    assert rec["scale"]["FETCH_SIZE"] == 2.0 and rec["scale"]["WRITE_SIZE"] == 1.0
    want = ((2000 * 2 + 500) + (500 * 2 + 100)) * 1024        # layer kernel averaged over two dispatches, dense head start
    assert rec["bytes"] == want
    assert [k["dispatches_averaged"] for k in rec["kernels"]] == [2, 1]
    sys.path.insert(0, ROOT)
    import bench
    assert rec["kernel_source_stamp"] == bench.kernel_source_stamp()
    # bench.py reads it back, and drops it when the sources it was measured on have changed
    bench.TRAFFIC_FILE = str(out)
    assert bench.recorded_traffic("bf16", "hunyuanvideo", "layer")[0] == want
    assert bench.recorded_traffic("bf16", "wan2.1", "layer") == (None, "no record")
    data = json.loads(out.read_text())
    data["records"]["bf16"]["hunyuanvideo"]["layer"]["kernel_source_stamp"] = "0" * 16
    out.write_text(json.dumps(data))
    got, why = bench.recorded_traffic("bf16", "hunyuanvideo", "layer")
    assert got is None and "stale" in why


def test_a_missing_dispatch_is_an_error(tmp_path):
    (tmp_path / "fetch.csv").write_text(HEADER + '"copy_probe_kernel",1,FETCH_SIZE,524288\n')
    (tmp_path / "write.csv").write_text(HEADER + '"copy_probe_kernel",1,WRITE_SIZE,1048576\n')
    run = {"config": {"workload": "w", "precision": "bf16"},
           "roofline": {"traffic_key": "dense", "dispatches": [{"kernel": "attn_fwd_kernel"}]}}
    (tmp_path / "run.json").write_text(json.dumps(run))
    res = subprocess.run([sys.executable, "-m", "paper_2506_03065_amd.traffic_record", "--bench-json", str(tmp_path / "run.json"),
                          "--fetch-csv", str(tmp_path / "fetch.csv"), "--write-csv", str(tmp_path / "write.csv"),
                          "--out", str(tmp_path / "t.json")], capture_output=True, text=True, cwd=ROOT)
    assert res.returncode != 0 and "no dispatch" in res.stderr
    assert not (tmp_path / "t.json").exists()
