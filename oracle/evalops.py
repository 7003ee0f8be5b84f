"""A six-output evaluation function over rows of class scores, each output
with its own reduce/gather op (Sec. 3.1), evaluated in slices and aggregated
(Sec. 5.1).  Outputs on a row set R (logits [|R| x C], labels y):

  ce_sum      sum_i ( logsumexp(logits_i) - logits_i[y_i] )        op sum
  counts[c]   #{ i : a_i = c },  a_i = argmax_c logits[i,c]        op sum (int)
  max_logit   max_{i,c} logits[i,c]                                op max
  min_logit   min_{i,c} logits[i,c]                                op min
  n_correct   #{ i : a_i = y_i }                                   op sum (int)
  argmax[i]   a_i, ties -> lowest class index                      op concat
"""
import numpy as np

from . import split
from .mlp import row_losses
from .reduce import reduce_buffers


def function(logits, y):
    logits = np.asarray(logits, dtype=np.float64)
    y = np.asarray(y).astype(np.int64)
    rows, C = logits.shape
    if rows == 0:
        return dict(ce_sum=np.zeros(1), counts=np.zeros(C, np.int64),
                    max_logit=np.full(1, -np.inf), min_logit=np.full(1, np.inf),
                    n_correct=np.zeros(1, np.int64), argmax=np.zeros(0, np.int64))
    a = np.empty(rows, dtype=np.int64)
    for i in range(rows):
        best = 0
        for c in range(1, C):
            if logits[i, c] > logits[i, best]:
                best = c
        a[i] = best
    counts = np.zeros(C, dtype=np.int64)
    for i in range(rows):
        counts[a[i]] += 1
    return dict(ce_sum=np.array([row_losses(logits, y).sum()]),
                counts=counts,
                max_logit=np.array([logits.max()]),
                min_logit=np.array([logits.min()]),
                n_correct=np.array([int((a == y).sum())], dtype=np.int64),
                argmax=a)


OUTPUT_OPS = dict(ce_sum="sum", counts="sum", max_logit="max", min_logit="min",
                  n_correct="sum", argmax="concat")


def sliced(logits, y, n_slices):
    """Run `function` on each of n_slices contiguous subsets and aggregate
    every output with its op, in slice order."""
    logits = np.asarray(logits)
    parts = [function(logits[a:b], y[a:b]) for (a, b) in split.share_bounds(logits.shape[0], n_slices)]
    return {k: reduce_buffers([p[k] for p in parts], op) for k, op in OUTPUT_OPS.items()}
