"""Oracle of the per-layer step of the offline sparse diffusion search.

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke test and the CPU leg of
the benchmark; the product path never calls it.  Plain numpy float64, no
blocking, written from the paper's text.

What it computes (Section 4.2, "Offline Sparse Diffusion Search", Eq. 2 and 3,
and the per-layer part of Algorithm 1): the layer's Q, K, V are passed through
all five modes M_0..M_4; for every head h and every sparse mode i = 1..4

    L_i[h] = MSE(O_i[h] - O_0[h]) + lambda * (1 - S_i[h])              (Eq. 2)

with S_i[h] the share of the attention map that mode i leaves out for that head
(1 for the skip mode).  Section 4.2 words S_i as a ratio of blocks of the authors'
kernels, whose block size is not given; this oracle counts elements (head_sparsity),
which no block size enters, and states the block count as well (head_block_sparsity).  The head keeps full attention (mode 0) when all four
losses exceed epsilon, otherwise it takes the mode with the smallest loss
(Eq. 3).  The layer's output x^o carries, per head, the output of the chosen
mode (Algorithm 1, "Per-Head Optimization").

Reading taken where the paper is at odds with itself: the listing of
Algorithm 1 adds `lambda * S_i`, Eq. 2 and the sentence after it ("the sparsity
penalty is added") add `lambda * (1 - S_i)`; a penalty must grow with the work a
mode keeps, so Eq. 2 is followed.  MSE is the mean over batch, tokens and
channels of the head.  Ties between losses go to the lower mode id.
"""
import numpy as np

from . import sparse_attention as A

SPARSE_MODES = (A.MODE_SKIP, A.MODE_DIAG, A.MODE_MULTIDIAG, A.MODE_VSTRIPE)   # i = 1..4 of Eq. 2


def head_sparsity(mode, params, L):
    """S_i of one head: share of the L x L attention map that the mode leaves out."""
    if mode == A.MODE_SKIP:
        return 1.0
    if mode == A.MODE_DENSE:
        return 0.0
    return 1.0 - A.mask_popcount(mode, params, L) / float(L * L)


def head_block_sparsity(mode, params, L, block_q, block_k):
    """The block-level count of S_i in the wording of Section 4.2 ("the ratio of actual computation blocks to the
    total number of blocks"): 1 - computed tiles / all tiles of the map for tiles of block_q x block_k.  A tile is
    computed when the explicit mask keeps at least one pair in it (band modes), a vertical-stripe head computes
    ceil(|C| / block_k) column tiles for every query tile, and the rows of a text prefix are computed as dense
    tiles on top of the pattern's own tiles."""
    if mode == A.MODE_SKIP:
        return 1.0
    if mode == A.MODE_DENSE:
        return 0.0
    n_qb, n_kb = -(-L // block_q), -(-L // block_k)
    text_tiles = (A.text_tokens_of(params) // block_q) * n_kb
    if mode == A.MODE_VSTRIPE:
        computed = n_qb * (A.column_list(params, L, block_k).size // block_k) + text_tiles
    else:
        computed = A.block_lists(mode, params, L, block_q, block_k)["kv_block_idx"].size + text_tiles
    return 1.0 - computed / float(n_qb * n_kb)


def head_mse(o, o_ref):
    """MSE(O_i - O_0) per head.  o, o_ref: [B, H, L, D] -> [H]."""
    diff = np.asarray(o, dtype=np.float64) - np.asarray(o_ref, dtype=np.float64)
    return (diff ** 2).mean(axis=(0, 2, 3))


def losses(mse, sparsity, lam):
    """Eq. 2 for arrays of shape [4, H] (row i - 1 = mode i)."""
    return np.asarray(mse, dtype=np.float64) + lam * (1.0 - np.asarray(sparsity, dtype=np.float64))


def select_modes(loss, eps):
    """Eq. 3: per head, mode 0 if every loss exceeds eps, else the arg-min sparse mode.
    loss: [4, H] (row i - 1 = mode i).  Returns int32 [H]."""
    loss = np.asarray(loss, dtype=np.float64)
    table = np.zeros(loss.shape[1], dtype=np.int32)
    for h in range(loss.shape[1]):
        column = loss[:, h]
        if (column > eps).sum() >= 4:
            table[h] = A.MODE_DENSE
        else:
            table[h] = SPARSE_MODES[int(np.argmin(column))]   # first minimum: lower mode id on ties
    return table


def search_layer(q, k, v, params_by_mode, lam, eps):
    """One layer of the search.  q, k, v: [B, H, L, D]; params_by_mode: dict
    mode id (2, 3, 4) -> list of H parameter dicts for that mode.

    Returns (table [H], loss [4, H], mse [4, H], sparsity [4, H], x_o [B, H, L, D]).
    """
    B, H, L, D = q.shape
    none = [dict() for _ in range(H)]
    outs = {}
    for mode in (A.MODE_DENSE,) + SPARSE_MODES:
        table = np.full(H, mode, dtype=np.int32)
        outs[mode] = A.attention_layer(q, k, v, table, params_by_mode.get(mode, none))
    mse = np.stack([head_mse(outs[m], outs[A.MODE_DENSE]) for m in SPARSE_MODES])
    sparsity = np.array([[head_sparsity(m, params_by_mode.get(m, none)[h], L) for h in range(H)]
                         for m in SPARSE_MODES])
    loss = losses(mse, sparsity, lam)
    table = select_modes(loss, eps)
    x_o = np.stack([outs[int(table[h])][:, h] for h in range(H)], axis=1)
    return table, loss, mse, sparsity, x_o
