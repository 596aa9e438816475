"""Seeded synthetic workloads with the shapes of the paper's models.

This module only draws inputs (Q/K/V tensors, per-head strategy tables and the
pattern parameters that go with them).  It holds none of the method's
arithmetic and is the one module that both the tests of the CPU oracle and the
callers of the HIP library use.

Shapes follow Section 5.1 (tokens per frame, frame counts, text prefix) and the
frame-major token order of Section 4.1.1; the widths, column counts and the mix
of modes per layer are this build's stand-ins for the constants the paper only
shows in a figure.  The tensors stand in for the post-RoPE/Norm Q, K, V of
CogVideoX1.5, HunyuanVideo and Wan2.1 on VBench / Penguin prompts, which are
not available here.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

DENSE, SKIP, DIAG, MULTIDIAG, VSTRIPE = 0, 1, 2, 3, 4
BASE_SEED = 20250603 * 10


@dataclass
class Workload:
    name: str
    index: int                 # position in the list of configurations
    B: int
    H: int
    L: int
    D: int
    frame_tokens: int
    n_frames: int
    text_tokens: int
    strategy_table: np.ndarray  # int32 [H], mode id per head
    pattern_params: list        # H dicts: half_width, offsets, cols
    seed: int
    notes: dict = field(default_factory=dict)

    @property
    def dense_flops(self) -> float:
        return 4.0 * self.B * self.H * float(self.L) ** 2 * self.D


def _head_params(mode, diag_w, multi_w, multi_offsets, cols):
    if mode == DIAG:
        return {"half_width": int(diag_w), "offsets": (0,), "cols": ()}
    if mode == MULTIDIAG:
        return {"half_width": int(multi_w), "offsets": tuple(int(o) for o in multi_offsets), "cols": ()}
    if mode == VSTRIPE:
        return {"half_width": 0, "offsets": (), "cols": tuple(int(c) for c in cols)}
    return {"half_width": 0, "offsets": (), "cols": ()}


def _seeded_table(counts, H, gen):
    """Seeded permutation of the multiset of modes given by counts[mode]."""
    modes = []
    for mode in (DIAG, MULTIDIAG, VSTRIPE, SKIP, DENSE):
        modes += [mode] * counts.get(mode, 0)
    assert len(modes) == H, (len(modes), H)
    perm = torch.randperm(H, generator=gen).numpy()
    return np.asarray(modes, dtype=np.int32)[perm]


def _seeded_columns(n, video_tokens, text_tokens, gen):
    """text columns 0..text-1 plus n seeded video columns (sorted)."""
    video = torch.randperm(video_tokens, generator=gen)[:n].numpy() + text_tokens
    return np.sort(np.concatenate([np.arange(text_tokens), video])).astype(np.int64)


def _build(name, index, H, D, frame_tokens, n_frames, text_tokens, counts, diag_w, multi_w,
           multi_k, n_cols, table_seed_offset=0):
    L = text_tokens + frame_tokens * n_frames
    seed = BASE_SEED + index
    gen = torch.Generator(device="cpu").manual_seed(seed + 1000 + table_seed_offset)
    table = _seeded_table(counts, H, gen)
    offsets = [k * frame_tokens for k in range(-multi_k, multi_k + 1)]
    params = []
    for h in range(H):
        cols = ()
        if table[h] == VSTRIPE:
            cols = _seeded_columns(n_cols, frame_tokens * n_frames, text_tokens, gen)
        params.append(_head_params(int(table[h]), diag_w, multi_w, offsets, cols))
    return Workload(name, index, 1, H, L, D, frame_tokens, n_frames, text_tokens, table, params, seed)


def tiny() -> Workload:
    """4 heads, D=64, 4 frames of 16x16 tokens; one head per non-skip mode."""
    table = np.asarray([DENSE, DIAG, MULTIDIAG, VSTRIPE], dtype=np.int32)
    cols = [256 * f + t for f in range(4) for t in range(16)]
    params = [_head_params(DENSE, 0, 0, (), ()),
              _head_params(DIAG, 128, 0, (), ()),
              _head_params(MULTIDIAG, 0, 32, (-256, 0, 256), ()),
              _head_params(VSTRIPE, 0, 0, (), cols)]
    return Workload("tiny", 0, 1, 4, 1024, 64, 256, 4, 0, table, params, BASE_SEED + 0)


def cogvideox15() -> Workload:
    """CogVideoX1.5-shaped layer: 48 heads, D=64, 20 frames of 60x72 tokens."""
    return _build("cogvideox1.5", 1, 48, 64, 4320, 20, 0,
                  {DIAG: 20, MULTIDIAG: 12, VSTRIPE: 12, SKIP: 2, DENSE: 2},
                  diag_w=2048, multi_w=512, multi_k=2, n_cols=2048)


def hunyuanvideo() -> Workload:
    """HunyuanVideo-shaped layer: 24 heads, D=128, 256 text + 32 frames of 45x80."""
    return _build("hunyuanvideo", 2, 24, 128, 3600, 32, 256,
                  {DIAG: 10, MULTIDIAG: 6, VSTRIPE: 6, SKIP: 1, DENSE: 1},
                  diag_w=3600, multi_w=900, multi_k=2, n_cols=2048)


def wan21() -> Workload:
    """Wan2.1-shaped layer: 40 heads, D=128, 21 frames of 45x80 tokens."""
    return _build("wan2.1", 3, 40, 128, 3600, 21, 0,
                  {DIAG: 16, MULTIDIAG: 10, VSTRIPE: 10, SKIP: 2, DENSE: 2},
                  diag_w=3600, multi_w=900, multi_k=2, n_cols=2048)


def stack_layer_counts(layer: int, n_layers: int = 40, H: int = 40) -> dict:
    """Mode counts of one layer of the stack: the dense share falls linearly
    from 80 % (first layer) to 10 % (last); the other heads are split
    diag : multi-diag : vertical : skip = 16 : 10 : 10 : 2 by largest remainder."""
    n_dense = int(round(H * (0.8 - 0.7 * layer / (n_layers - 1))))
    rest = H - n_dense
    weights = {DIAG: 16, MULTIDIAG: 10, VSTRIPE: 10, SKIP: 2}
    total = sum(weights.values())
    exact = {m: rest * w / total for m, w in weights.items()}
    counts = {m: int(np.floor(x)) for m, x in exact.items()}
    left = rest - sum(counts.values())
    for m in sorted(weights, key=lambda m: (-(exact[m] - counts[m]), m))[:left]:
        counts[m] += 1
    counts[DENSE] = n_dense
    return counts


def stack_layer(layer: int, n_layers: int = 40) -> Workload:
    """Layer `layer` of the 40-layer stack at the Wan2.1 shape."""
    wl = _build(f"stack-layer{layer}", 4, 40, 128, 3600, 21, 0, stack_layer_counts(layer, n_layers),
                diag_w=3600, multi_w=900, multi_k=2, n_cols=2048, table_seed_offset=layer)
    wl.notes["layer"] = layer
    return wl


def with_text_borders(wl: Workload, text_tokens=None) -> Workload:
    """The same layer with the borders of the text prefix kept whole by every
    sparse head (Section 4.1.1: T-T, T-V and V-T around the V-V pattern): the
    parameter dicts of the sparse heads gain the key "text_tokens".  Default
    prefix: the workload's own text tokens."""
    import copy
    T = wl.text_tokens if text_tokens is None else int(text_tokens)
    out = copy.copy(wl)
    out.name = f"{wl.name}+text{T}"
    out.text_tokens = T
    out.notes = dict(wl.notes)
    out.pattern_params = [dict(p, text_tokens=T) if int(m) >= DIAG else dict(p)
                          for m, p in zip(wl.strategy_table, wl.pattern_params)]
    return out


def hunyuanvideo_text() -> Workload:
    """The HunyuanVideo-shaped layer with the borders of its 256 text tokens kept whole."""
    return with_text_borders(hunyuanvideo())


BY_NAME = {"tiny": tiny, "cogvideox1.5": cogvideox15, "hunyuanvideo": hunyuanvideo, "wan2.1": wan21,
           "hunyuanvideo+text": hunyuanvideo_text}


def small(L=333, H=5, D=64, seed=7, B=1) -> Workload:
    """A ragged little layer for parity tests: one head per mode, lengths that
    are no multiple of any tile size."""
    gen = torch.Generator(device="cpu").manual_seed(seed)
    table = np.asarray(([DENSE, DIAG, MULTIDIAG, VSTRIPE, SKIP] * H)[:H], dtype=np.int32)
    frame = max(8, L // 5)
    params = []
    for h in range(H):
        cols = ()
        if table[h] == VSTRIPE:
            cols = np.sort(torch.randperm(L, generator=gen)[:max(1, L // 7)].numpy())
        params.append(_head_params(int(table[h]), max(1, L // 9), max(1, L // 40),
                                   (-2 * frame, -frame, 0, frame, 2 * frame), cols))
    return Workload(f"small-L{L}-D{D}", -1, B, H, L, D, frame, 5, 0, table, params, seed)


def make_qkv(wl: Workload, device="cpu", heads=None):
    """bf16 N(0,1) Q, K, V of shape [B, H, L, D] drawn head by head from the
    workload's seed (float32 normal, rounded to bf16).  With `heads`, only those
    heads are drawn (others stay zero) - the values of a head do not depend on
    which other heads are drawn."""
    shape = (wl.B, wl.H, wl.L, wl.D)
    out = [torch.zeros(shape, dtype=torch.bfloat16, device=device) for _ in range(3)]
    for b in range(wl.B):
        for h in range(wl.H):
            if heads is not None and h not in heads:
                continue
            gen = torch.Generator(device="cpu").manual_seed(wl.seed * 1000 + b * wl.H + h)
            for t in out:
                x = torch.randn(wl.L, wl.D, generator=gen, dtype=torch.float32).to(torch.bfloat16)
                t[b, h].copy_(x)
    return out


def sample_rows(wl: Workload, n_random=64, seed=0):
    """Query rows for sampled checks at full size: the first and last rows, rows
    around every frame boundary and the text/video boundary, and seeded random
    rows (sorted, unique)."""
    gen = torch.Generator(device="cpu").manual_seed(wl.seed + 77 + seed)
    rows = set(range(0, 4)) | set(range(wl.L - 4, wl.L))
    for f in range(wl.n_frames + 1):
        edge = wl.text_tokens + f * wl.frame_tokens
        rows |= {r for r in (edge - 1, edge) if 0 <= r < wl.L}
    rows |= set(torch.randint(0, wl.L, (n_random,), generator=gen).tolist())
    return np.asarray(sorted(rows), dtype=np.int64)
