"""Reduce / gather ops applied to per-worker (or per-slice) results.

Sec. 3.1 "Build Functions": each output of a function carries a reduce or
gather operation; Sec. 3.2 step 3: worker results are reduced or gathered back;
Sec. 3.3 step 2: the flat gradient array is all-reduced (read as an average).
"""
import numpy as np

OPS = ("sum", "mean", "max", "min", "prod", "concat")


def reduce_buffers(bufs, op, weights=None):
    """bufs: list of equally long 1-D arrays (concat: any lengths).
    sum/prod fold in list order; mean = sum_w omega_w * buf_w with omega = 1/N
    unless weights are given; integer inputs stay integer (mean is refused for
    them); floats are combined in float64."""
    if op not in OPS:
        raise ValueError(op)
    bufs = [np.asarray(b) for b in bufs]
    if not bufs:
        raise ValueError("nothing to reduce")
    if op == "concat":
        return np.concatenate(bufs)
    is_int = np.issubdtype(bufs[0].dtype, np.integer)
    work = [b.astype(np.int64 if is_int else np.float64) for b in bufs]
    if op == "mean":
        if is_int:
            raise TypeError("mean of integer buffers is not defined here")
        n = len(work)
        omega = [1.0 / n] * n if weights is None else [float(x) for x in weights]
        acc = np.zeros_like(work[0])
        for w, b in zip(omega, work):
            acc = acc + w * b
        return acc
    acc = work[0].copy()
    for b in work[1:]:
        if op == "sum":
            acc = acc + b
        elif op == "prod":
            acc = acc * b
        elif op == "max":
            acc = np.maximum(acc, b)
        else:
            acc = np.minimum(acc, b)
    return acc
