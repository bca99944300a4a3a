"""TEST INFRASTRUCTURE: host-side checks of an arrow decomposition.

A decomposition of a square sparse A with block width b is a list of levels
``(perm_i, rows_i, cols_i, vals_i)``: ``perm_i`` maps a position p of level i
to an original vertex id, and ``(rows_i, cols_i, vals_i)`` are the stored
entries of the arrow matrix ``B_i`` in position coordinates, so that
``A = sum_i P_i^T B_i P_i`` with ``(P_i X)[p, :] = X[perm_i[p], :]``.

The three properties the method promises:

* reassembly -- the multiset ``(perm_i[p], perm_i[q], bits(v))`` over all
  levels equals the multiset ``(row, col, bits(val))`` of A, bit for bit
  (so every nonzero lives in exactly one level, never split or summed);
* arrow shape -- every stored (p, q) has ``p // b == q // b`` (diagonal
  block) or ``p < b`` (first block row) or ``q < b`` (first block column);
* every ``perm_i`` is injective into ``[0, n)``.

:func:`arrow_product` evaluates ``sum_i P_i^T B_i P_i X`` slowly in fp64 from
such levels; tests compare it with the CSR product of A to validate what the
library exports, without a GPU.  None of this is used by the product.
"""
from __future__ import annotations

import numpy as np


def check_perm_injective(perm: np.ndarray, n: int) -> None:
    perm = np.asarray(perm)
    assert perm.ndim == 1
    if perm.size == 0:
        return
    assert perm.min() >= 0 and perm.max() < n, "perm entry out of range"
    assert np.unique(perm).size == perm.size, "perm is not injective"


def check_arrow_shape(rows: np.ndarray, cols: np.ndarray, b: int, n_i: int) -> None:
    rows = np.asarray(rows, dtype=np.int64)
    cols = np.asarray(cols, dtype=np.int64)
    if rows.size == 0:
        return
    assert rows.min() >= 0 and rows.max() < n_i and cols.min() >= 0 and cols.max() < n_i, \
        "position outside the level"
    ok = (rows // b == cols // b) | (rows < b) | (cols < b)
    bad = np.flatnonzero(~ok)
    assert bad.size == 0, f"{bad.size} entries outside the arrow of width {b}, first at " \
                          f"({rows[bad[0]]}, {cols[bad[0]]})"


def check_reassembly(n: int, rowptr: np.ndarray, colidx: np.ndarray, vals: np.ndarray,
                     levels) -> None:
    """Bit-exact multiset equality between A and the union of the mapped level entries."""
    a_rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    a_key = a_rows * n + colidx.astype(np.int64)
    a_bits = np.ascontiguousarray(vals, dtype=np.float32).view(np.uint32)
    keys, bits = [], []
    for perm, r, c, v in levels:
        perm = np.asarray(perm, dtype=np.int64)
        keys.append(perm[np.asarray(r, dtype=np.int64)] * n + perm[np.asarray(c, dtype=np.int64)])
        bits.append(np.ascontiguousarray(v, dtype=np.float32).view(np.uint32))
    d_key = np.concatenate(keys) if keys else np.zeros(0, np.int64)
    d_bits = np.concatenate(bits) if bits else np.zeros(0, np.uint32)
    assert d_key.size == a_key.size, f"entry count differs: {d_key.size} vs {a_key.size}"
    oa = np.lexsort((a_bits, a_key))
    od = np.lexsort((d_bits, d_key))
    assert np.array_equal(a_key[oa], d_key[od]), "coordinates differ"
    assert np.array_equal(a_bits[oa], d_bits[od]), "value bits differ"


def check_decomposition(n, rowptr, colidx, vals, b, levels) -> None:
    for perm, r, c, v in levels:
        check_perm_injective(perm, n)
        check_arrow_shape(r, c, b, len(perm))
    check_reassembly(n, rowptr, colidx, vals, levels)


def arrow_product(n: int, levels, X: np.ndarray) -> np.ndarray:
    """``sum_i P_i^T B_i (P_i X)`` in fp64, one stored entry at a time (vectorised over k)."""
    Y = np.zeros((n, X.shape[1]), dtype=np.float64)
    Xd = X.astype(np.float64)
    for perm, r, c, v in levels:
        perm = np.asarray(perm, dtype=np.int64)
        Xp = Xd[perm]                                   # gather  P_i X
        Z = np.zeros_like(Xp)
        np.add.at(Z, np.asarray(r, dtype=np.int64),     # Z = B_i Xp
                  np.asarray(v, dtype=np.float64)[:, None] * Xp[np.asarray(c, dtype=np.int64)])
        np.add.at(Y, perm, Z)                           # scatter-add  P_i^T Z
    return Y
