"""CPU oracle of the token rearrangement that turns the multi-diagonal pattern
into one diagonal band.

TEST INFRASTRUCTURE ONLY.  Imported by the tests and by nothing in the product
path; it shares no code with the HIP library and never imports it.

What it follows in the paper
----------------------------
Section 4.1.1: video tokens are ordered frame by frame, so the diagonal blocks of
the V-V region are self-frame interactions and the off-diagonal blocks cross-frame
ones.  Section 4.1.2 (multi-diagonal pattern): the evenly spaced diagonals are
attention between tokens at nearby spatial positions of different frames, and
"by rearranging tokens" the pattern becomes a diagonal structure that window
attention can compute.

Written out: with F frames of N tokens after T0 leading tokens, the token at
frame f, position p has index T0 + f*N + p (frame-major).  The rearrangement
moves it to T0 + p*F + f (position-major); tokens outside the video block stay
where they are.  A window of half width W in the rearranged order keeps (i, j)
iff |pi(i) - pi(j)| <= W.  For W = w*F + F - 1 this contains every pair of video
tokens whose positions differ by at most w, in any two frames (the reading of
"nearby spatial positions across different frames"), plus part of the pairs at
distance w + 1; unlike diagonals on the frame-major index it does not wrap from
the end of one frame into the start of the next.

The oracle states the kept set in the ORIGINAL order through an explicit mask
and evaluates Eq. 1 on it with the attention oracle; that the same result is a
diagonal-band attention on rearranged tensors, rearranged back, is a theorem
the tests check, not something this module assumes.

Pins (tests/test_oracle_rearrange.py): the index map against explicit (frame,
position) loops, bijectivity, identity cases, a closed-form pair count, the
containment claims above, and the equivalence with the diagonal oracle applied
to rearranged inputs.  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

from . import sparse_attention as SA


position_major_index = SA.position_major_index   # the index map, stated once in the attention oracle


def rearrange(x, first, frame_tokens, frames, inverse=False):
    """Rows of x ([L, ...]) moved to position-major order (or back)."""
    pi = position_major_index(x.shape[0], first, frame_tokens, frames)
    out = np.empty_like(x)
    if inverse:
        out[...] = x[pi]          # the token at original index i sits at pi[i]
    else:
        out[pi] = x
    return out


def window_mask(L, first, frame_tokens, frames, half_width, rows):
    """Explicit mask [len(rows), L] in the original order: |pi(i) - pi(j)| <= W."""
    pi = position_major_index(L, first, frame_tokens, frames)
    rows = np.asarray(rows, dtype=np.int64)
    return np.abs(pi[None, :] - pi[rows][:, None]) <= int(half_width)


def attention_head_rearranged(q, k, v, first, frame_tokens, frames, half_width, rows=None, chunk=128):
    """Eq. 1 restricted to the window in position-major order; q, k, v: [L, D] in
    the original order, result rows in the original order."""
    L, d = q.shape
    rows = np.arange(L, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.zeros((rows.size, d), dtype=np.float64)
    for s in range(0, rows.size, chunk):
        r = rows[s:s + chunk]
        out[s:s + chunk] = SA.attention_rows(q[r], k, v, window_mask(L, first, frame_tokens, frames, half_width, r))
    return out
