"""Pins of the oracle's masks, pair counts, block lists and head grouping."""
import json
import os

import numpy as np
import pytest

from oracle import sparse_attention as O
from paper_2506_03065_amd import workloads as W

GOLDEN = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "pattern_counts.json")))


def band_pairs_closed_form(L, w, offsets):
    """Kept pairs of non-overlapping bands: diagonal delta has L - |delta| cells."""
    total = 0
    for o in offsets:
        for delta in range(o - w, o + w + 1):
            total += max(0, L - abs(delta))
    return total


def test_pair_counts_closed_form_vs_explicit_mask():
    for L, w, offs in [(1024, 128, (0,)), (1024, 32, (-256, 0, 256)), (1500, 40, (-700, 0, 700, 1490)),
                       (777, 0, (0,)), (300, 400, (0,))]:
        mode = O.MODE_DIAG if offs == (0,) else O.MODE_MULTIDIAG
        got = O.mask_popcount(mode, {"half_width": w, "offsets": offs}, L)
        assert got == band_pairs_closed_form(L, w, offs)
    assert O.mask_popcount(O.MODE_VSTRIPE, {"cols": (1, 5, 9)}, 100) == 300
    assert O.mask_popcount(O.MODE_DENSE, {}, 100) == 10000


def test_golden_pair_counts():
    """The stored counts follow from the closed form at every benchmark shape and
    from the explicit mask at the tiny one."""
    for name, g in GOLDEN.items():
        if name.startswith("_"):
            continue
        L = g["L"]
        assert L * (2 * g["diag"]["w"] + 1) - g["diag"]["w"] * (g["diag"]["w"] + 1) == g["diag"]["pairs"]
        assert band_pairs_closed_form(L, g["multi"]["w"], g["multi"]["offsets"]) == g["multi"]["pairs"]
        assert g["vertical"]["n_cols"] * L == g["vertical"]["pairs"]
    g = GOLDEN["tiny"]
    wl = W.tiny()
    assert O.mask_popcount(O.MODE_DIAG, wl.pattern_params[1], wl.L) == g["diag"]["pairs"]
    assert O.mask_popcount(O.MODE_MULTIDIAG, wl.pattern_params[2], wl.L) == g["multi"]["pairs"]
    assert O.mask_popcount(O.MODE_VSTRIPE, wl.pattern_params[3], wl.L) == g["vertical"]["pairs"]


def test_workloads_match_the_golden_parameters():
    for name, make in W.BY_NAME.items():
        wl, g = make(), GOLDEN[name.split("+")[0]]   # a "+text" variant shares the parameters of its base
        assert wl.L == g["L"]
        for h in range(wl.H):
            mode, p = int(wl.strategy_table[h]), wl.pattern_params[h]
            if mode == W.DIAG:
                assert p["half_width"] == g["diag"]["w"] and p["offsets"] == (0,)
            if mode == W.MULTIDIAG:
                assert p["half_width"] == g["multi"]["w"] and list(p["offsets"]) == g["multi"]["offsets"]
            if mode == W.VSTRIPE:
                assert len(p["cols"]) == g["vertical"]["n_cols"] == len(set(p["cols"]))
                assert list(p["cols"][:wl.text_tokens]) == list(range(wl.text_tokens))


def test_tiny_block_counts_match_golden():
    wl = W.tiny()
    for bs, key in ((128, "tiles128"), (64, "tiles64")):
        d = O.block_lists(O.MODE_DIAG, wl.pattern_params[1], wl.L, bs, bs)
        m = O.block_lists(O.MODE_MULTIDIAG, wl.pattern_params[2], wl.L, bs, bs)
        assert d["kv_block_idx"].size == GOLDEN["tiny"][key]["diag"]
        assert m["kv_block_idx"].size == GOLDEN["tiny"][key]["multi"]


def diag_tiles_closed_form(L, w, T):
    """Square T x T tiles, L a multiple of T.  Tile (qb, kb) spans the diagonals
    (kb-qb)T - (T-1) .. (kb-qb)T + (T-1); it holds a kept cell iff the nearest of
    them is within w, and is wholly kept iff the farthest is."""
    n = L // T
    listed = sum(n - abs(d) for d in range(-n + 1, n) if abs(d) * T - (T - 1) <= w)
    full = sum(n - abs(d) for d in range(-n + 1, n) if abs(d) * T + (T - 1) <= w)
    return listed, full


@pytest.mark.parametrize("L,w,T", [(1024, 128, 128), (1024, 128, 64), (2048, 300, 64), (512, 31, 32), (512, 0, 32)])
def test_diagonal_block_counts_closed_form(L, w, T):
    bl = O.block_lists(O.MODE_DIAG, {"half_width": w}, L, T, T)
    listed, full = diag_tiles_closed_form(L, w, T)
    assert bl["kv_block_idx"].size == listed
    assert int(bl["flags"].sum()) == full
    assert bl["row_ptr"][-1] == listed and bl["row_ptr"].size == L // T + 1


def _loop_block_lists(mode, p, L, bq, bk):
    """Tile lists by plain loops over every (i, j) - no array reshapes."""
    offs = (0,) if mode == O.MODE_DIAG else tuple(p["offsets"])
    w = p["half_width"]
    kept_delta = lambda d: any(abs(d - o) <= w for o in offs)
    runs, d = [], -(L - 1)
    while d <= L - 1:
        if kept_delta(d):
            s = d
            while d + 1 <= L - 1 and kept_delta(d + 1):
                d += 1
            runs.append((s, d))
        d += 1
    row_ptr, idx, flags, first, count = [0], [], [], [], []
    for qb in range(-(-L // bq)):
        for kb in range(-(-L // bk)):
            seen, complete, hit = False, True, set()
            for i in range(qb * bq, min(L, (qb + 1) * bq)):
                for j in range(kb * bk, (kb + 1) * bk):
                    ok = j < L and kept_delta(j - i)
                    seen |= ok
                    complete &= ok
                    if ok:
                        hit.add([t for t, (a, b) in enumerate(runs) if a <= j - i <= b][0])
            if seen:
                idx.append(kb)
                flags.append(int(complete))
                first.append(min(hit))
                count.append(max(hit) - min(hit) + 1)
        row_ptr.append(len(idx))
    return runs, row_ptr, idx, flags, first, count


@pytest.mark.parametrize("mode,p,L,bq,bk", [
    (O.MODE_DIAG, {"half_width": 5}, 50, 8, 4),
    (O.MODE_DIAG, {"half_width": 70}, 50, 8, 8),
    (O.MODE_MULTIDIAG, {"half_width": 2, "offsets": (-20, 0, 20)}, 53, 8, 8),
    (O.MODE_MULTIDIAG, {"half_width": 3, "offsets": (0, 7, -7, 30)}, 47, 16, 4),   # touching bands merge
    (O.MODE_MULTIDIAG, {"half_width": 1, "offsets": (0, 4, 9)}, 40, 8, 16),        # several runs in one tile
    (O.MODE_MULTIDIAG, {"half_width": 0, "offsets": (0, -100, 100)}, 33, 4, 8),    # bands off the map
])
def test_block_lists_against_plain_loops(mode, p, L, bq, bk):
    runs, row_ptr, idx, flags, first, count = _loop_block_lists(mode, p, L, bq, bk)
    bl = O.block_lists(mode, p, L, bq, bk)
    assert bl["runs"].tolist() == [list(r) for r in runs]
    assert bl["row_ptr"].tolist() == row_ptr
    assert bl["kv_block_idx"].tolist() == idx
    assert bl["flags"].tolist() == flags
    assert bl["run_first"].tolist() == first
    assert bl["run_count"].tolist() == count
    assert all(a.dtype == np.int32 for a in bl.values())


def test_runs_merge_touching_bands_and_clip():
    runs = O.delta_runs(O.MODE_MULTIDIAG, {"half_width": 3, "offsets": (0, 7, -7, 30)}, 47)
    assert runs.tolist() == [[-10, 10], [27, 33]]
    runs = O.delta_runs(O.MODE_DIAG, {"half_width": 100}, 20)
    assert runs.tolist() == [[-19, 19]]
    runs = O.delta_runs(O.MODE_MULTIDIAG, {"half_width": 2, "offsets": (0, 22, 25)}, 20)
    assert runs.tolist() == [[-2, 2]]            # the other bands lie outside the map


def test_column_list_padding():
    got = O.column_list({"cols": (9, 2, 7)}, 10, 4)
    assert got.dtype == np.int32 and got.tolist() == [2, 7, 9, -1]
    assert O.column_list({"cols": tuple(range(8))}, 8, 4).tolist() == list(range(8))
    with pytest.raises(ValueError):
        O.column_list({"cols": (1, 1)}, 8, 4)


def test_head_groups_fuse_by_mode_and_share_lists():
    table = [2, 0, 2, 4, 1, 3, 2, 4, 4]
    p_d1, p_d2 = {"half_width": 8}, {"half_width": 9}
    p_m = {"half_width": 2, "offsets": (0, 10, -10)}
    c1, c2 = {"cols": (1, 2, 3)}, {"cols": (3, 2, 1)}
    params = [p_d1, {}, p_d2, c1, {}, p_m, p_d1, c2, {"cols": (4,)}]
    groups = O.head_groups(table, params)
    assert [g["mode"] for g in groups] == [0, 1, 2, 3, 4]
    by_mode = {g["mode"]: g for g in groups}
    assert by_mode[2]["heads"] == [0, 2, 6] and by_mode[2]["list_id"] == [0, 1, 0] and by_mode[2]["n_lists"] == 2
    assert by_mode[4]["heads"] == [3, 7, 8] and by_mode[4]["list_id"] == [0, 0, 1]
    assert by_mode[0]["heads"] == [1] and by_mode[1]["heads"] == [4]
    with pytest.raises(ValueError):
        O.head_groups([0, 5], [{}, {}])
