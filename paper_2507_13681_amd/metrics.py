"""Host-side bookkeeping for reports: how many attention cells a selection allows.

Not part of the compute path.  The count is exact and follows from the index sets alone:
column b is crossed by min(n_hat, n - b) new-turn rows, diagonal o by min(n_hat, n - o), and a
column and a diagonal share the one cell (row position b + o, key b) when that row belongs to
the newest turn, i.e. n - n_hat <= b + o <= n - 1.
"""
from __future__ import annotations

import numpy as np


def allowed_cells(n: int, n_hat: int, v_idx, s_idx) -> int:
    """Cells of the n_hat x n causal block covered by the union of the given lines."""
    v = np.unique(np.asarray(v_idx, dtype=np.int64))
    s = np.unique(np.asarray(s_idx, dtype=np.int64))
    cells = int(np.minimum(n_hat, n - v).sum() + np.minimum(n_hat, n - s).sum())
    if len(v) and len(s):
        lo = np.searchsorted(v, n - n_hat - s, side="left")
        hi = np.searchsorted(v, n - 1 - s, side="right")
        cells -= int((hi - lo).sum())
    return cells


def selection_cells(n: int, n_hat: int, sel: dict) -> np.ndarray:
    """allowed_cells for every (batch, head) of a selection dict (numpy arrays)."""
    B, Hq = sel["v_cnt"].shape
    out = np.zeros((B, Hq), np.int64)
    for b in range(B):
        for h in range(Hq):
            nv = min(int(sel["v_cnt"][b, h]), sel["v_idx"].shape[-1])
            ns = min(int(sel["s_cnt"][b, h]), sel["s_idx"].shape[-1])
            out[b, h] = allowed_cells(n, n_hat, sel["v_idx"][b, h, :nv], sel["s_idx"][b, h, :ns])
    return out


def visited_tiles(n: int, n_hat: int, v_idx, s_idx, rows: int = 128, keys: int = 64) -> int:
    """Number of (rows x keys) tiles the sparse attention kernel visits for one head: per block of `rows` query rows
    (aligned to absolute positions that are multiples of `rows`), the key blocks of `keys` keys that hold a cell on a
    selected diagonal, plus the packed tiles of `keys` gathered columns each (none when every diagonal is selected).
    Reports split the kernel's time between heads in proportion to this count."""
    v = np.unique(np.asarray(v_idx, dtype=np.int64))
    s = np.unique(np.asarray(s_idx, dtype=np.int64))
    bm = np.zeros(n + 1, np.int64)
    bm[s[(s >= 0) & (s < n)]] = 1
    cs = np.concatenate(([0], np.cumsum(bm[:n])))           # cs[i] = selected diagonals below i
    pos0 = (n - n_hat) // rows * rows
    every = len(s) >= n
    tiles = 0
    for bp in range(pos0, n, rows):
        posmax = min(bp + rows - 1, n - 1)
        kb = np.arange(posmax // keys + 1)
        lo = np.clip(bp - (kb * keys + keys - 1), 0, n)      # diagonals of the tile: (first row - last key) .. (last row - first key)
        hi = np.clip(bp + rows - 1 - kb * keys + 1, 0, n)
        tiles += int(((cs[np.maximum(hi, lo)] - cs[lo]) > 0).sum())
        if not every:
            tiles += -(-int(np.searchsorted(v, posmax, side="right")) // keys)
    return tiles


def causal_cells(n: int, n_hat: int) -> int:
    return n_hat * (n - n_hat) + n_hat * (n_hat + 1) // 2


def coverage_from_lse(lse_selected, lse_dense) -> np.ndarray:
    """Share of each row's attention mass that a selection keeps (the left side of Eq. 1, per row).

    Both arguments are natural-log softmax denominators of the same rows: over the allowed cells
    (ls_sparse_prefill with the selection) and over all visible cells (ls_sparse_prefill with every
    diagonal selected).  Their ratio is the sum of the dense attention weights over the allowed
    cells.  A row without any allowed cell (lse = -inf) keeps 0."""
    a = np.asarray(lse_selected, np.float64)
    b = np.asarray(lse_dense, np.float64)
    with np.errstate(invalid="ignore"):
        c = np.exp(a - b)
    return np.where(np.isfinite(a), c, 0.0)
