"""Oracle: negligible-cost approximation models (section 3.6).

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

An n-gram model is a table lookup: the next-token logits depend on the last
token only (bigram) or on nothing (unigram).  A copying model guesses that
the context repeats itself.  As a "scorer" (see oracle.decode) each plugs
into Algorithm 1 in place of Mq unchanged: the algorithm never looks inside
the approximation model (section 2.1).
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


class CopyDraft:
    """The parameter-less model of section 3.6 that copies from the context.

    Reading taken here (the paper gives the idea, not the rule): the context s
    is everything before the position to fill, guesses of the running
    iteration included.  Its last `match` tokens are looked up in s itself; of
    all earlier occurrences that are followed by a token, the most recent one
    wins and the model puts all its mass on the token that followed it (logit
    0 there, -inf elsewhere).  Without such an occurrence the model is the
    `fallback` scorer, or, with none, the uniform distribution: the random
    model that closes section 3.6.
    """

    def __init__(self, vocab: int, match: int, fallback=None):
        if vocab < 1 or match < 1:
            raise ValueError("vocab and match must be positive")
        self.vocab, self.match, self.fallback = int(vocab), int(match), fallback

    def copied_token(self, s):
        """Token after the most recent earlier occurrence of s[-match:], or None."""
        s = [int(t) for t in s]
        k, n = self.match, len(s)
        tail = s[n - k:]
        for j in range(n - k - 1, -1, -1):      # occurrence s[j:j+k], followed by s[j+k]
            if s[j:j + k] == tail:
                return s[j + k]
        return None

    def score(self, prefix, k: int) -> np.ndarray:
        if k < 1 or k > len(prefix):
            raise ValueError("need 1 <= k <= len(prefix)")
        rows = []
        for end in range(len(prefix) - k + 1, len(prefix) + 1):
            ctx = list(prefix[:end])
            tok = self.copied_token(ctx)
            if tok is not None:
                row = np.full(self.vocab, -np.inf)
                row[tok] = 0.0
            elif self.fallback is not None:
                row = np.asarray(self.fallback.score(ctx, 1)[0], dtype=np.float64)
            else:
                row = np.zeros(self.vocab)
            rows.append(row)
        return np.stack(rows)
