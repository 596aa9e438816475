"""CPU oracle for pattern-specific sparse 3D attention (Sparse-vDiT, arxiv 2506.03065).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition the HIP
path is checked against.  It may be imported by the tests, by the smoke check
and by the benchmark's CPU-baseline leg, and by nothing else; it shares no code
with the HIP library and never imports it.

What it follows in the paper
----------------------------
* Section 3, Eq. 1: per head, O_h = softmax(Q_h K_h^T / sqrt(d)) V_h.
* Section 3 ("Sparse Attention") and Section 4.2 ("Sparse Computation
  Pre-definition"): a sparse mode evaluates Eq. 1 only over the kept region of
  the attention map; mode M_1 skips the head and writes zeros.
* Section 4.1.2: the three kept regions - a band around the main diagonal
  (diagonal pattern), several evenly spaced bands (multi-diagonal pattern) and
  a set of key columns seen by every query (vertical-stripe pattern).
* Section 4.2: the sparsity of a kernel is counted in blocks of the attention
  map, which is why block lists are derived here as well.

* Section 4.1.1: with text tokens in the sequence the attention map has four
  regions, T-T, T-V, V-T and V-V, and the patterns are described for V-V.  A
  head whose parameters carry text_tokens = T > 0 (text first) keeps the three
  border regions whole: key j < T for every query, every key for query i < T.

* Section 4.1.2 (multi-diagonal pattern): "by rearranging tokens" the evenly
  spaced diagonals become one diagonal band.  A multi-diagonal head whose
  parameters carry rearranged = (first, frame_tokens, frames) is that form: with
  pi the move from frame-major to position-major order of the video block, it
  keeps (i, j) iff |pi(i) - pi(j)| <= half_width; its offsets are not used and
  its block lists live in the rearranged order.

Readings where the paper is silent:
the band is inclusive (|delta| <= w), several bands form a union, the softmax is
renormalised over the kept keys, a row without any kept key is an error, modes
are numbered 0 dense, 1 skip, 2 diagonal, 3 multi-diagonal, 4 vertical-stripe.

All floating point is numpy float64.  Everything is written as the definition:
an explicit boolean mask is materialised for the rows at hand, masked scores are
set to -inf, and a plain softmax follows.  There is no blocking or fusion.

Pins (tests/test_oracle_*.py): library softmax attention with an explicit mask,
a pure-Python triple loop, full-width patterns == dense, constant-V and zero-Q
closed forms, closed-form mask popcounts, and block counts fixed by counting
arguments.  No function here is "parity unpinned".
"""
from __future__ import annotations

import math

import numpy as np

MODE_DENSE = 0      # M_0, Eq. 1 as is
MODE_SKIP = 1       # M_1, output zeros (Section 4.2)
MODE_DIAG = 2       # M_2, diagonal pattern (Section 4.1.2)
MODE_MULTIDIAG = 3  # M_3, multi-diagonal pattern (Section 4.1.2)
MODE_VSTRIPE = 4    # M_4, vertical-stripe pattern (Section 4.1.2)

BAND_MODES = (MODE_DIAG, MODE_MULTIDIAG)


def _offsets_of(mode, params):
    if mode == MODE_DIAG:
        return (0,)
    offs = tuple(int(o) for o in params["offsets"])
    if len(offs) < 1:
        raise ValueError("multi-diagonal head without offsets")
    return offs


def rearranged_of(params):
    """(first, frame_tokens, frames) of a multi-diagonal head that is computed as a
    window in position-major order, or None."""
    r = params.get("rearranged") if params else None
    return tuple(int(x) for x in r) if r else None


def position_major_index(L, first, frame_tokens, frames):
    """pi: int64 [L].  Section 4.1.1 orders video tokens frame by frame: frame f,
    position p sits at first + f*N + p.  pi moves it to first + p*F + f
    (position-major); tokens outside the video block keep their index."""
    N, F = int(frame_tokens), int(frames)
    if first < 0 or N < 1 or F < 1 or first + N * F > L:
        raise ValueError("the video block does not fit the sequence")
    pi = np.arange(L, dtype=np.int64)
    v = np.arange(N * F, dtype=np.int64)
    pi[first:first + N * F] = first + (v % N) * F + v // N
    return pi


def text_tokens_of(params):
    """Length T of the text prefix whose borders the head keeps whole (0: none)."""
    return int(params.get("text_tokens", 0)) if params else 0


def allowed_mask(mode, params, L, rows):
    """Explicit boolean mask [len(rows), L]: True where key j is kept for query i.

    Section 4.1.2 patterns, element level:
      dense          every j
      diagonal       |i - j| <= w
      multi-diagonal exists o in offsets with |j - i - o| <= w
      vertical       j in the head's column set
    and, for the sparse modes with text_tokens = T > 0 (Section 4.1.1), also every
    j < T and every j when i < T.
    """
    rows = np.asarray(rows, dtype=np.int64)
    if mode == MODE_DENSE:
        return np.ones((rows.size, L), dtype=bool)
    T = text_tokens_of(params)
    if T:
        if not 0 < T < L:
            raise ValueError("text prefix must be shorter than the sequence")
        mask = _pattern_mask(mode, params, L, rows)
        mask[:, :T] = True
        mask[rows < T, :] = True
        return mask
    return _pattern_mask(mode, params, L, rows)


def _pattern_mask(mode, params, L, rows):
    """The V-V pattern of Section 4.1.2 on the global token index, without borders."""
    if mode in BAND_MODES:
        w = int(params["half_width"])
        if w < 0:
            raise ValueError("negative half width")
        if mode == MODE_MULTIDIAG and rearranged_of(params):
            if text_tokens_of(params):
                raise ValueError("a rearranged head takes no text prefix")
            pi = position_major_index(L, *rearranged_of(params))
            return np.abs(pi[None, :] - pi[rows][:, None]) <= w
        delta = np.arange(L, dtype=np.int64)[None, :] - rows[:, None]
        mask = np.zeros((rows.size, L), dtype=bool)
        for o in _offsets_of(mode, params):
            mask |= np.abs(delta - o) <= w
        return mask
    if mode == MODE_VSTRIPE:
        cols = np.asarray(params["cols"], dtype=np.int64)
        if cols.size < 1:
            raise ValueError("vertical-stripe head without columns")
        if cols.min() < 0 or cols.max() >= L:
            raise ValueError("column out of range")
        if np.unique(cols).size != cols.size:
            raise ValueError("duplicate column")
        mask = np.zeros((rows.size, L), dtype=bool)
        mask[:, cols] = True
        return mask
    raise ValueError(f"mode {mode} has no mask")


def attention_rows(q_rows, k, v, mask):
    """Eq. 1 for a set of query rows of one head, restricted to mask.

    q_rows [R, D], k [L, D], v [L, D] (any float dtype, widened to float64),
    mask [R, L] bool.  Returns float64 [R, D].
    """
    q_rows = np.asarray(q_rows, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    d = q_rows.shape[-1]
    if not mask.any(axis=1).all():
        raise ValueError("a query row keeps no key")
    scores = (q_rows @ k.T) / math.sqrt(d)
    scores[~mask] = -np.inf
    scores -= scores.max(axis=1, keepdims=True)
    p = np.exp(scores)
    p /= p.sum(axis=1, keepdims=True)
    return p @ v


def attention_head(q, k, v, mode, params, rows=None, chunk=128):
    """One head, all rows or the given rows.  q, k, v are [L, D]."""
    L, d = q.shape
    rows = np.arange(L, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.zeros((rows.size, d), dtype=np.float64)
    if mode == MODE_SKIP:
        return out
    for s in range(0, rows.size, chunk):
        r = rows[s:s + chunk]
        out[s:s + chunk] = attention_rows(q[r], k, v, allowed_mask(mode, params, L, r))
    return out


def attention_layer(q, k, v, strategy_table, pattern_params, rows=None, chunk=128):
    """The layer of Section 4.2: every head runs the mode the table assigns to it.

    q, k, v: [B, H, L, D].  strategy_table: H mode ids.  pattern_params: H dicts
    with the keys each mode needs (half_width, offsets, cols).  Returns float64
    [B, H, R, D] with R = L or len(rows).
    """
    B, H, L, d = q.shape
    n_rows = L if rows is None else len(rows)
    out = np.zeros((B, H, n_rows, d), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            out[b, h] = attention_head(q[b, h], k[b, h], v[b, h], int(strategy_table[h]),
                                       pattern_params[h], rows=rows, chunk=chunk)
    return out


# --------------------------------------------------------------------------
# Block-level view of the patterns (Section 4.2: sparsity counted in blocks).
# --------------------------------------------------------------------------

def delta_runs(mode, params, L):
    """Maximal runs of kept diagonals of a band pattern.

    A band pattern keeps (i, j) depending on delta = j - i only.  Returns an
    int64 array [n, 2] of inclusive [lo, hi] runs of consecutive kept deltas
    inside [-(L-1), L-1], ascending.  Found by marking every delta.
    """
    if mode == MODE_MULTIDIAG and rearranged_of(params):   # one band, in the rearranged order
        mode, params = MODE_DIAG, {"half_width": int(params["half_width"])}
    w = int(params["half_width"])
    deltas = np.arange(-(L - 1), L, dtype=np.int64)
    kept = np.zeros(deltas.size, dtype=bool)
    for o in _offsets_of(mode, params):
        kept |= np.abs(deltas - o) <= w
    runs = []
    start = None
    for t in range(deltas.size):
        if kept[t] and start is None:
            start = deltas[t]
        if start is not None and (t + 1 == deltas.size or not kept[t + 1]):
            runs.append((start, deltas[t]))
            start = None
    return np.asarray(runs, dtype=np.int64).reshape(-1, 2)


def _run_lookup(runs, L):
    run_of_delta = np.full(2 * L - 1, -1, dtype=np.int32)
    for t, (lo, hi) in enumerate(runs):
        run_of_delta[lo + L - 1: hi + L] = t
    return run_of_delta


def query_block_entries(mode, params, L, block_q, block_k, qb, runs=None):
    """List entries of one query block of a band pattern, read off the explicit
    mask of its in-range rows.  Returns (kv_block_idx, flags, run_first,
    run_count) as int32 arrays; see block_lists for their meaning."""
    if mode not in BAND_MODES:
        raise ValueError("block lists exist for the band modes only")
    if mode == MODE_MULTIDIAG and rearranged_of(params):
        # rows and keys of the list are positions in the rearranged order, where the head is a plain band
        position_major_index(L, *rearranged_of(params))   # validates the geometry
        mode, params = MODE_DIAG, {"half_width": int(params["half_width"])}
    T = text_tokens_of(params)
    if T and (T % block_q or T % block_k):
        raise ValueError("the text prefix must be a multiple of both block sizes")
    runs = delta_runs(mode, params, L) if runs is None else runs
    run_of_delta = _run_lookup(runs, L)
    n_kb = -(-L // block_k)
    rows = np.arange(qb * block_q, min(L, (qb + 1) * block_q), dtype=np.int64)
    as32 = lambda a: np.asarray(a, dtype=np.int32)
    if T and rows[0] < T:
        # text queries see every key: their rows are computed densely, not from a list
        return (as32([]), as32([]), as32([]), as32([]))
    mask = allowed_mask(mode, params, L, rows)
    band = _pattern_mask(mode, params, L, rows)
    delta = np.arange(L, dtype=np.int64)[None, :] - rows[:, None]
    rid = run_of_delta[delta + (L - 1)]
    pad = n_kb * block_k - L
    tile = lambda a, fill: np.pad(a, ((0, 0), (0, pad)), constant_values=fill).reshape(rows.size, n_kb, block_k)
    tiles, btiles, rtiles = tile(mask, False), tile(band, False), tile(rid, -1)
    any_ = tiles.any(axis=(0, 2))
    all_ = tiles.all(axis=(0, 2))
    rmin = np.where(btiles, rtiles, np.iinfo(np.int32).max).min(axis=(0, 2))
    rmax = np.where(btiles, rtiles, -1).max(axis=(0, 2))
    has_band = btiles.any(axis=(0, 2))
    rmin = np.where(has_band, rmin, 0)
    count = np.where(has_band, rmax - rmin + 1, 0)
    kbs = np.nonzero(any_)[0]
    return (as32(kbs), as32(all_[kbs]), as32(rmin[kbs]), as32(count[kbs]))


def block_lists(mode, params, L, block_q, block_k):
    """Key-block lists of a band pattern, read off the explicit mask.

    For every query block (block_q rows, the last one may be short):
      kv_block_idx  ascending ids of the key blocks that hold a kept element
      flags         1 if every element of the tile is kept for every in-range
                    row and the tile lies wholly inside [0, L), else 0
      run_first,    the kept-diagonal runs (see delta_runs) that have a kept
      run_count     element in the tile are consecutive; their first id and
                    their number (0, 0 for a tile kept for its text keys only)
    row_ptr is the CSR pointer over query blocks.  All int32.
    With a text prefix T (a multiple of both block sizes) the query blocks of the
    text rows have no entries (those rows are dense) and every other query block
    lists the T / block_k text tiles, kept whole.
    For a rearranged multi-diagonal head the lists are those of the plain band in
    the rearranged order, and row_map gives the original row of every position.
    """
    runs = delta_runs(mode, params, L)
    n_qb = -(-L // block_q)
    row_ptr = [0]
    parts = [[], [], [], []]
    for qb in range(n_qb):
        ent = query_block_entries(mode, params, L, block_q, block_k, qb, runs)
        for dst, src in zip(parts, ent):
            dst.append(src)
        row_ptr.append(row_ptr[-1] + ent[0].size)
    cat = lambda a: np.concatenate(a).astype(np.int32)
    out = {"row_ptr": np.asarray(row_ptr, dtype=np.int32), "kv_block_idx": cat(parts[0]),
           "flags": cat(parts[1]), "run_first": cat(parts[2]), "run_count": cat(parts[3]),
           "runs": runs.astype(np.int32)}
    if mode == MODE_MULTIDIAG and rearranged_of(params):
        out["row_map"] = row_map(L, *rearranged_of(params), block_k)
    return out


def row_map(L, first, frame_tokens, frames, block_k):
    """Original row of every position of the rearranged order (the inverse of
    position_major_index), padded with -1 to a multiple of block_k (int32)."""
    pi = position_major_index(L, first, frame_tokens, frames)
    padded = -(-L // block_k) * block_k
    out = np.full(padded, -1, dtype=np.int32)
    out[pi] = np.arange(L, dtype=np.int32)
    return out


def column_list(params, L, block_k):
    """Sorted unique key columns of a vertical-stripe head (with the text columns
    0..T-1 when the head has a text prefix), padded with -1 to a multiple of
    block_k (int32)."""
    cols = np.asarray(params["cols"], dtype=np.int64)
    if cols.size < 1 or cols.min() < 0 or cols.max() >= L or np.unique(cols).size != cols.size:
        raise ValueError("bad column set")
    cols = np.union1d(cols, np.arange(text_tokens_of(params), dtype=np.int64))   # sorted, text columns included
    padded = -(-cols.size // block_k) * block_k
    out = np.full(padded, -1, dtype=np.int32)
    out[:cols.size] = cols
    return out


def mask_popcount(mode, params, L, chunk=256):
    """Number of kept (i, j) pairs, counted on the explicit mask."""
    total = 0
    for s in range(0, L, chunk):
        rows = np.arange(s, min(L, s + chunk))
        total += int(allowed_mask(mode, params, L, rows).sum())
    return total


def _params_key(mode, params):
    if mode in BAND_MODES:
        if mode == MODE_MULTIDIAG and rearranged_of(params):
            return (int(params["half_width"]), rearranged_of(params))
        return (int(params["half_width"]), tuple(sorted(set(_offsets_of(mode, params)))), text_tokens_of(params))
    if mode == MODE_VSTRIPE:
        return (tuple(sorted(int(c) for c in params["cols"])), text_tokens_of(params))
    return ()


def head_groups(strategy_table, pattern_params):
    """Head fusion of Section 4.2: heads of one layer that share a mode form a
    group (one launch).  Inside a group, heads whose parameters describe the
    same kept region share one list.

    Returns a list of groups in ascending mode order (rearranged multi-diagonal
    heads after the plain ones); a group is a dict with mode, heads (ascending
    head ids), list_id (per head, ids numbered in order of first appearance),
    n_lists and rearranged.
    """
    groups = []
    # rearranged multi-diagonal heads run another loop shape and form a group of their own, after the plain ones
    for mode, rearranged in ((MODE_DENSE, False), (MODE_SKIP, False), (MODE_DIAG, False), (MODE_MULTIDIAG, False),
                             (MODE_MULTIDIAG, True), (MODE_VSTRIPE, False)):
        heads = [h for h in range(len(strategy_table)) if int(strategy_table[h]) == mode
                 and (mode != MODE_MULTIDIAG or bool(rearranged_of(pattern_params[h])) == rearranged)]
        if not heads:
            continue
        seen = {}
        list_id = []
        for h in heads:
            key = _params_key(mode, pattern_params[h])
            if key not in seen:
                seen[key] = len(seen)
            list_id.append(seen[key])
        groups.append({"mode": mode, "heads": heads, "list_id": list_id, "n_lists": len(seen), "rearranged": rearranged})
    for m in strategy_table:
        if int(m) not in (0, 1, 2, 3, 4):
            raise ValueError("mode id outside 0..4")
    return groups
