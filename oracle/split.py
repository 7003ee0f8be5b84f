"""Contiguous near-equal split of a run of data points.

Sec. 3.2 step 1: a call's inputs are scattered over the workers as equally as
possible along the first dimension (Sec. 4.1); Sec. 5.1: each worker cuts its
share into `num_slices` subsets; Sec. 5.2: with input indexing the thing being
split is the index list, each worker taking its own share of it.

Reading where the paper is silent: the remainder goes to the first shares
(count % parts shares get one extra element); shares may be empty.
"""


def share_sizes(count, parts):
    if parts <= 0 or count < 0:
        raise ValueError("need parts > 0 and count >= 0")
    base = count // parts
    extra = count % parts
    return [base + 1 if i < extra else base for i in range(parts)]


def share_bounds(count, parts):
    """[(start, stop)] of each share inside range(count)."""
    out = []
    start = 0
    for n in share_sizes(count, parts):
        out.append((start, start + n))
        start += n
    return out


def worker_slice_bounds(count, n_workers, n_slices):
    """bounds[w][s] = (start, stop) inside range(count): workers first, then
    each worker's share cut again by the same rule (Sec. 5.2, last sentence:
    slicing happens inside a worker after indexing fixed the assignment)."""
    out = []
    for (w0, w1) in share_bounds(count, n_workers):
        out.append([(w0 + a, w0 + b) for (a, b) in share_bounds(w1 - w0, n_slices)])
    return out
