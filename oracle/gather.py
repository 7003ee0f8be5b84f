"""Input indexing (Sec. 5.2): the minibatch is data[idx] for a list of row
indexes, duplicates allowed, or for a slice start:stop:step; worker w receives
the rows named by its contiguous share of the list.  For data that already
lives on the workers (Sec. 5.2 last part, Sec. 4.2 "scatter": an array is
divided over the workers by its first dimension), every worker indexes its own
share with its own list, or all of them with the same one."""
import numpy as np

from . import split


def gather_rows(data, idx):
    data = np.asarray(data)
    idx = np.asarray(idx)
    if idx.size and (idx.min() < 0 or idx.max() >= data.shape[0]):
        raise IndexError("index out of range")
    out = np.empty((idx.shape[0],) + data.shape[1:], dtype=data.dtype)
    for j in range(idx.shape[0]):
        out[j] = data[int(idx[j])]
    return out


def gather_shares(data, idx, n_workers):
    """List of per-worker arrays, in worker order."""
    return [gather_rows(data, idx[a:b]) for (a, b) in split.share_bounds(len(idx), n_workers)]


def slice_indexes(start, stop, step):
    """The index list a slice start:stop:step (step >= 1, 0 <= start <= stop)
    stands for: start, start+step, ... below stop."""
    if step < 1 or start < 0 or stop < start:
        raise ValueError("slice out of the supported form")
    out = []
    j = start
    while j < stop:
        out.append(j)
        j += step
    return np.asarray(out, dtype=np.int64)


def scatter(data, n_workers):
    """Sec. 4.2: the array divided over the workers by its first dimension,
    shares as equal as possible, in order."""
    data = np.asarray(data)
    return [data[a:b].copy() for (a, b) in split.share_bounds(data.shape[0], n_workers)]


def gather_resident(shares, idx_lists):
    """Every worker w excerpts rows idx_lists[w] from its own resident share."""
    if len(shares) != len(idx_lists):
        raise ValueError("one index list per worker")
    return [gather_rows(s, i) for s, i in zip(shares, idx_lists)]


def normalise_u8(rows_u8, mean, std):
    """rows_u8: [n, C, ...] uint8; mean/std: [C] on the 0..255 scale.
    out = float32( (float64(x) - mean_c) / std_c ): the correctly rounded
    float32 of the float64 quotient."""
    x = np.asarray(rows_u8)
    if x.dtype != np.uint8:
        raise TypeError("expects uint8")
    mean = np.asarray(mean, dtype=np.float64)
    std = np.asarray(std, dtype=np.float64)
    shape = (1, x.shape[1]) + (1,) * (x.ndim - 2)
    return ((x.astype(np.float64) - mean.reshape(shape)) / std.reshape(shape)).astype(np.float32)


def round_to_bf16(x):
    """Round-to-nearest-even of float32-valued numbers to bfloat16 (8 exponent
    bits, 7 stored mantissa bits), returned as float32.  Finite inputs only."""
    a = np.asarray(x, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    keep = bits >> np.uint64(16)
    rest = bits & np.uint64(0xFFFF)
    half = np.uint64(0x8000)
    up = (rest > half) | ((rest == half) & ((keep & np.uint64(1)) == np.uint64(1)))
    keep = keep + up.astype(np.uint64)
    out = (keep << np.uint64(16)).astype(np.uint32)
    return out.view(np.float32).reshape(a.shape)
