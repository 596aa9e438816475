"""Where the per-head relative gate of the bf16 parity tests comes from (parity_util.MAX_OVER_RMS).

The precision reading of this build (the paper states none): bf16 inputs, Q multiplied by log2(e)/sqrt(D) and
rounded back to bf16, scores and softmax in fp32, P rounded to bf16 before PV, fp32 accumulation, bf16 output.
This test carries that arithmetic out on the CPU (numpy float64 between the roundings, no blocking, exact row
maximum) for the narrow-band heads that gave the largest deviations in a sweep of random layers, and compares it
with the exact definition (the oracle).  The deviation of the SPECIFIED arithmetic alone, before any kernel, reaches
6.6 % of a head's rms on a single element: a gate of 5 % would reject the reading itself, the gate of 8 % sits
1.2 times above it.  No GPU, no library."""
import numpy as np
import torch

from oracle import sparse_attention as O
from paper_2506_03065_amd import workloads as W
from parity_util import MAX_ABS, MAX_OVER_RMS, MEAN_ABS, REL_L2
from test_gpu_random_layers import random_layer


def bf16(x):
    return torch.tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16).to(torch.float64).numpy()


def specified_arithmetic(q, k, v, mode, p):
    """One head in the precision the build specifies, row by row over explicit masks."""
    L, D = q.shape
    c = np.float32(1.4426950408889634 / np.sqrt(D))
    qs = bf16(q.astype(np.float32) * c)                       # pre-scaled Q, rounded to bf16
    out = np.zeros((L, D))
    for r0 in range(0, L, 256):
        rows = np.arange(r0, min(L, r0 + 256))
        mask = O.allowed_mask(mode, p, L, rows)
        s = qs[rows] @ k.T
        s[~mask] = -np.inf
        pr = bf16(np.exp2(s - s.max(axis=1, keepdims=True)))  # P rounded to bf16, numerator and denominator alike
        out[rows] = bf16((pr @ v) / pr.sum(axis=1, keepdims=True))
    return out


def test_the_relative_gate_sits_just_above_the_specified_arithmetic():
    worst = 0.0
    for seed, heads in ((23, (5, 2)), (45, (3, 0)), (3, (5,))):
        wl, _ = random_layer(seed)
        q, k, v = W.make_qkv(wl)
        for h in heads:
            mode, p = int(wl.strategy_table[h]), wl.pattern_params[h]
            assert mode in (W.DIAG, W.MULTIDIAG)
            qh, kh, vh = (t[0, h].to(torch.float64).numpy() for t in (q, k, v))
            want = O.attention_head(qh, kh, vh, mode, p)
            got = specified_arithmetic(qh, kh, vh, mode, p)
            diff = np.abs(got - want)
            rms = float(np.sqrt((want ** 2).mean()))
            # the contract bars and the relative-L2 gate hold with a wide margin for the arithmetic itself
            assert diff.max() <= MAX_ABS / 2 and diff.mean() <= MEAN_ABS / 2
            assert np.sqrt((diff ** 2).sum() / (want ** 2).sum()) <= REL_L2 / 2
            worst = max(worst, float(diff.max()) / rms)
    assert 0.05 < worst <= MAX_OVER_RMS - 0.01, worst      # above the 5 % first tried, inside the gate with room for the kernel's blocking
    assert MAX_OVER_RMS <= 1.5 * worst                     # and the gate is not loose against it
