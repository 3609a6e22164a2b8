"""Oracle for greedy sampling with a confidence gap (test infrastructure, never used by the product
path): the token a greedy sampler picks from a row of logits, the runner-up, and the gap between
their logits.

Sec. 3.8 (on-device greedy sampling: argmax over the ~128k-entry logit row instead of copying it
to the host); Sec. 3.9.2 (confidence gamma = top-1 logit minus top-2 logit of a cached answer);
Sec. 3.9.4 (Delta_ready = l(1) - l(2), compared with a threshold).

The paper does not say how equal logits are ordered: the lowest index wins, for both places.
Selection only compares the given fp32 values, so indices and values are exact; the gap is the
fp32 difference of the two selected values.
"""
import numpy as np


def top2(logits):
    """logits [rows, vocab] float32 -> (idx1 int32, idx2 int32, val1 f32, val2 f32, gap f32), each [rows].
    idx1 = lowest index of the maximum; idx2 = lowest index of the maximum of the row without
    entry idx1 (vocab >= 2)."""
    x = np.asarray(logits, dtype=np.float32)
    if x.ndim != 2 or x.shape[1] < 2:
        raise ValueError("logits must be [rows, vocab >= 2]")
    rows = x.shape[0]
    idx1 = np.empty(rows, np.int32); idx2 = np.empty(rows, np.int32)
    val1 = np.empty(rows, np.float32); val2 = np.empty(rows, np.float32)
    for r in range(rows):
        row = x[r]
        i1 = int(np.argmax(row))                     # first occurrence of the maximum
        rest = row.copy()
        rest[i1] = -np.inf
        i2 = int(np.argmax(rest))
        if i2 == i1:                                 # every other entry is -inf as well: next index
            i2 = 1 if i1 == 0 else 0
            if not np.all(np.isneginf(np.delete(row, i1))):
                raise AssertionError
        idx1[r], idx2[r], val1[r], val2[r] = i1, i2, row[i1], row[i2]
    with np.errstate(invalid="ignore"):              # a row of nothing but -inf: the gap is NaN on both sides
        gap = (val1 - val2).astype(np.float32)
    return idx1, idx2, val1, val2, gap
