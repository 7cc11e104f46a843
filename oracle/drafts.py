"""Oracle: negligible-cost approximation models (section 3.6).

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

An n-gram model is a table lookup: the next-token logits depend on the last
token only (bigram) or on nothing (unigram).  As a "scorer" (see
oracle.decode) it plugs into Algorithm 1 in place of Mq unchanged: the
algorithm never looks inside the approximation model (section 2.1).
"""
from __future__ import annotations

import numpy as np


class TableDraft:
    """score(prefix, k) -> logits rows [k, V] for the last k positions of prefix:
    row j is table[row_of[token at that position]] (row 0 for every context when
    row_of is None)."""

    def __init__(self, table, row_of=None):
        self.table = np.asarray(table, dtype=np.float64)
        if self.table.ndim != 2:
            raise ValueError("table must be [rows, vocab]")
        self.row_of = None if row_of is None else np.asarray(row_of, dtype=np.int64)
        if self.row_of is not None and (self.row_of.min() < 0 or self.row_of.max() >= self.table.shape[0]):
            raise ValueError("row_of points outside the table")

    def score(self, prefix, k: int) -> np.ndarray:
        if k < 1 or k > len(prefix):
            raise ValueError("need 1 <= k <= len(prefix)")
        rows = []
        for tok in prefix[len(prefix) - k:]:
            rows.append(self.table[0 if self.row_of is None else self.row_of[int(tok)]])
        return np.stack(rows)
