"""Second oracle: attention, importance and eviction with the normalisation deferred.

Test infrastructure only.  ``longflow_oracle.c`` writes out the plain definitions
(eq. 1, eq. 6, argmin) with a max-subtracted softmax over the valid rows.  The
paper's fused operator (Sec. 3.4 "Fused Attention and Eviction Kernel", Alg. 1)
reaches the same values by another route, and this module states that route as a
property of the definitions:

  * exponentials are taken WITHOUT subtracting a maximum (wide floating point,
    float64 here) and nothing is divided by the softmax denominator until every
    row has been seen;
  * an invalid row (mask 0) has logit -inf, hence weight exactly 0, whatever the
    row holds;
  * the cache may be cut into any number of consecutive pieces: per piece one
    takes the sum of the weights, the weighted sum of the value rows, and per
    row the L1 norm of the contribution vector (weight times value row); pieces
    combine by plain addition;
  * at the end the output and the per-row norms are divided by the total weight
    and the row with the smallest normalised norm is the one to evict.

The cut is done in one reshape (rows padded with invalid ones up to a whole
number of pieces), the per-piece sums are array reductions.  Results must not
depend on the piece length.  The loop bounds printed in Alg. 1 are garbled; the
reading taken is "every row, in consecutive pieces, the last one ragged".
"""
from __future__ import annotations

import numpy as np


def attend_in_pieces(query, keys, values, valid, piece):
    """One query head.  query [d]; keys, values [rows, d]; valid [rows] (nonzero = live);
    piece = rows per piece.  Returns (output [d], normalised norms [rows], row to evict)."""
    query = np.asarray(query, dtype=np.float64)
    keys = np.asarray(keys, dtype=np.float64)
    values = np.asarray(values, dtype=np.float64)
    live = np.asarray(valid).astype(bool)
    rows, d = keys.shape
    pieces = -(-rows // piece)
    pad = pieces * piece - rows
    # dead rows may hold anything, NaN included: they are replaced before any arithmetic
    keys = np.concatenate([np.where(live[:, None], keys, 0.0), np.zeros((pad, d))])
    values = np.concatenate([np.where(live[:, None], values, 0.0), np.zeros((pad, d))])
    live = np.concatenate([live, np.zeros(pad, dtype=bool)])
    keys, values, live = keys.reshape(pieces, piece, d), values.reshape(pieces, piece, d), live.reshape(pieces, piece)

    logits = np.where(live, keys @ query / np.sqrt(d), -np.inf)          # [pieces, piece]
    weights = np.exp(logits)                                             # no maximum subtracted; exp(-inf) = 0
    contributions = weights[..., None] * values                          # weight times value row
    piece_weight = weights.sum(axis=1)                                   # per piece ...
    piece_output = contributions.sum(axis=1)
    row_norms = np.abs(contributions).sum(axis=2)
    total = piece_weight.sum()                                           # ... combined by addition
    output = piece_output.sum(axis=0) / total
    norms = (row_norms / total).reshape(-1)[:rows]
    return output, norms, int(np.argmin(norms))


def attend_in_pieces_group(queries, keys, values, valid, piece):
    """Group form used by this build: queries [G, d]; the norms of the G heads that share the
    KV head are added (the paper leaves heads out, Sec. 2.1)."""
    queries = np.asarray(queries, dtype=np.float64)
    per_head = [attend_in_pieces(qh, keys, values, valid, piece) for qh in queries]
    return np.stack([o for o, _, _ in per_head]), sum(s for _, s, _ in per_head)
