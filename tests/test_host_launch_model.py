"""The library's host code under AddressSanitizer + UBSan on a host model of the HIP runtime.

tests/hip_stub/ holds a stand-in <hip/hip_runtime.h> (streams, events, stream
capture with its fork/join rules, "device" memory that is exact-size host
memory) and host models of every kernel launch that walk the kernels' index
arithmetic and touch each byte a launch would address.  The harness replays,
per layer: workspace sizing, plan creation, the bf16 and FP8 forward passes
eagerly, on a caller stream and under a modelled capture, the per-group entry
points, plan destruction.  It reports 256 compute units (or the count given),
so the key-range splits, the text-row launches and the fork onto plan-owned
streams all run - none of which a box without a GPU reaches otherwise."""
import os
import subprocess
import sys

import pytest

from paper_2506_03065_amd import workloads as W
from test_gpu_random_layers import random_layer

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
STUB = os.path.join(ROOT, "tests", "hip_stub")
CSRC = os.path.join(ROOT, "paper_2506_03065_amd", "csrc")


@pytest.fixture(scope="module")
def replay(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("hip_stub") / "replay")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
           "-fno-sanitize-recover=undefined", "-I", STUB, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(CSRC, "api.cpp"), os.path.join(CSRC, "pattern_compiler.cpp"),
           os.path.join(STUB, "hip_stub.cpp"), os.path.join(STUB, "launch_models.cpp"),
           os.path.join(STUB, "replay.cpp"), "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-4000:]
    return exe


def layer_text(wl, split, rounds, tensors=1, cu=256):
    text = wl.text_tokens if any("text_tokens" in (p or {}) for p in wl.pattern_params) else 0
    lines = [f"layer {wl.name} {wl.B} {wl.H} {wl.L} {wl.D} {text} {split} {rounds} {tensors} {cu}",
             "table " + " ".join(str(int(m)) for m in wl.strategy_table)]
    for p in wl.pattern_params:
        p = p or {}
        offs = [int(o) for o in p.get("offsets", ())]
        cols = [int(c) for c in p.get("cols", ())]
        first, n, f = p.get("rearranged") or (0, 0, 0)
        lines.append(" ".join(map(str, ["head", int(p.get("half_width", 0)), len(offs), *offs, len(cols), *cols,
                                        first, n, f])))
    return "\n".join(lines) + "\n"


def run(replay, tmp_path, layers, shortfall=None):
    path = tmp_path / "layers.txt"
    path.write_text("".join(layers))
    cmd = [replay, str(path)] + ([str(shortfall)] if shortfall else [])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    return subprocess.run(cmd, capture_output=True, text=True, env=env, timeout=600)


def test_capture_and_replay_sequence_of_the_layer_that_aborted(replay, tmp_path):
    """Three random layers, 25 plans each, both precisions eagerly, on a caller stream and under capture.
    The third (L 998, D 128, 7 heads, 256 text tokens, five-way dense split, table [3,3,3,3,1,0,2]) is the
    first that splits the key range of its text-row launches."""
    layers = []
    for seed in (0, 1, 2):
        wl, split = random_layer(seed)
        layers.append(layer_text(wl, split, rounds=25))
    wl, split = random_layer(2)
    assert (wl.L, wl.D, wl.H, wl.text_tokens, split) == (998, 128, 7, 256, 5)
    assert wl.strategy_table.tolist() == [3, 3, 3, 3, 1, 0, 2]
    res = run(replay, tmp_path, layers)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert "3 layers replayed" in res.stdout


def test_random_layers_stay_inside_their_workspace(replay, tmp_path):
    layers = [layer_text(*random_layer(seed), rounds=2) for seed in range(40)]
    res = run(replay, tmp_path, layers)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]


@pytest.mark.parametrize("cu", [1, 8, 80, 304])
def test_other_compute_unit_counts(replay, tmp_path, cu):
    """The splits are sized from the compute-unit count: the workspace must cover whatever they come to."""
    layers = [layer_text(*random_layer(seed), rounds=1, cu=cu) for seed in range(12)]
    res = run(replay, tmp_path, layers)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]


def test_benchmark_layers_index_arithmetic(replay, tmp_path):
    """The full-size layers: tensors are not allocated, every workspace word and partial-result row is checked."""
    names = ["cogvideox1.5", "hunyuanvideo", "wan2.1", "hunyuanvideo+text"]
    layers = [layer_text(W.BY_NAME[n](), 0, rounds=1, tensors=0) for n in names]
    layers.append(layer_text(W.stack_layer(0), 0, rounds=1, tensors=0))
    res = run(replay, tmp_path, layers)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    # the library's own choice of the launch form with 256 compute units: the whole layer in one launch at D = 128
    # (long items), a launch per group at D = 64
    forms = {line.split()[1].rstrip(":"): int(line.split()[-1]) for line in res.stdout.splitlines() if "launch form is" in line}
    assert forms == {"cogvideox1.5": 0, "hunyuanvideo": 1, "wan2.1": 1, "hunyuanvideo+text256": 1, "stack-layer0": 1}, forms


def test_short_items_keep_the_grouped_launches(replay, tmp_path):
    """Small layers (few key tiles per item) stay on grouped launches whatever the head size."""
    layers = [layer_text(*random_layer(seed), rounds=1) for seed in range(6)]
    res = run(replay, tmp_path, layers)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    forms = [int(line.split()[-1]) for line in res.stdout.splitlines() if "launch form is" in line]
    assert forms == [0] * 6, forms


def test_the_harness_sees_a_planted_shortfall(replay, tmp_path):
    """The checker has teeth: with the plan workspace allocated 64 bytes short of what the library is told,
    the launch models report the accesses that leave it."""
    wl, split = random_layer(2)
    res = run(replay, tmp_path, [layer_text(wl, split, rounds=1)], shortfall=64)
    assert res.returncode != 0
    assert "outside every device allocation" in res.stderr or "AddressSanitizer" in res.stderr
