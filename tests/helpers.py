"""Shared test plumbing: tolerances, the error metric, upload helpers and the
comparison that accepts either derivative of relu at a pre-activation that is
zero up to rounding."""
import numpy as np

# Tolerances fixed by the benchmark spec: bit-exact for integer/byte/index
# work; max relative error 1e-4 for fp32 arithmetic, 2e-2 for bf16-input /
# fp32-accumulate arithmetic.  "Relative" is per tensor and scale-normalised:
# max|got - ref| / max|ref| (element-wise ratios are undefined on the exact
# zeros a relu network produces).
TOL_F32 = 1e-4
TOL_BF16 = 2e-2

# How far the oracle with values rounded at the bf16 points may sit from the all-float64 oracle at
# the wide configuration's shape: per tensor (max-norm over the tensor's largest entry) and for a
# worker's whole gradient (Frobenius).  A property of bf16 inputs (relu decisions of near-zero units
# change, each moving a column by one of a worker's 128 row terms), pinned on the CPU for the oracle
# alone; GPU results are held to these bands plus the tolerance against the float64 oracle, and to
# the tolerance against the oracle rounded at the same points.
BF16_VS_F64_MAX = 0.25
BF16_VS_F64_FRO = 0.10


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    scale = max(np.abs(ref).max(), 1e-30)
    return float(np.abs(got - ref).max() / scale)


def mlp_tensors(flat, dims):
    """[(name, 2-D view)] of a flat array laid out like the parameters; biases
    come back as 1 x n so that 'column j' means unit j everywhere."""
    out = []
    at = 0
    for l in range(len(dims) - 1):
        k, n = dims[l], dims[l + 1]
        out.append(("W%d" % (l + 1), flat[at:at + k * n].reshape(k, n)))
        at += k * n
        out.append(("b%d" % (l + 1), flat[at:at + n].reshape(1, n)))
        at += n
    return out


# A column (= hidden unit) with two or more pre-activations that are zero up to rounding may have any
# subset of them on the other side of the relu kink, so neither oracle variant need match it to the
# tolerance; each such entry is one row's term of the column, so the column is still held to this
# looser bound instead of being skipped.
TIE_COLUMN_FACTOR = 5.0


def rel_err_either_tie(got, ref, alt, dims, loose_cols=None, report=None):
    """Worst per-tensor error of `got` against `ref`, where a column (= hidden unit) may instead
    match `alt`, the oracle evaluated with the other valid relu derivative at pre-activations that
    are zero up to rounding.  loose_cols: {tensor name: set(columns)} holding two or more such
    entries: their error is divided by TIE_COLUMN_FACTOR before it enters the maximum (so a caller
    that asserts `< tol` holds them to TIE_COLUMN_FACTOR * tol).  `report`, if a dict, collects the
    number of such columns and their worst raw error."""
    worst = 0.0
    for (name, g), (_, r), (_, a) in zip(mlp_tensors(np.asarray(got, np.float64), dims),
                                         mlp_tensors(np.asarray(ref, np.float64), dims),
                                         mlp_tensors(np.asarray(alt, np.float64), dims)):
        scale = max(np.abs(r).max(), 1e-30)
        e = np.minimum(np.abs(g - r).max(axis=0), np.abs(g - a).max(axis=0)) / scale
        if loose_cols and name in loose_cols:
            for j in loose_cols[name]:
                if report is not None:
                    report["loose_columns"] = report.get("loose_columns", 0) + 1
                    report["loose_worst"] = max(report.get("loose_worst", 0.0), float(e[j]))
                e[j] /= TIE_COLUMN_FACTOR
        worst = max(worst, float(e.max()))
    return worst


def tie_columns(trace, eps):
    """From the hidden pre-activations z_1.. of one row set: columns (units)
    per layer with two or more entries within eps of zero, as skip_cols, and
    the total number of such entries."""
    skip, total = {}, 0
    for l, z in enumerate(trace):
        cnt = (np.abs(z) <= eps).sum(axis=0)
        total += int(cnt.sum())
        cols = set(np.nonzero(cnt >= 2)[0].tolist())
        if cols:
            skip["W%d" % (l + 1)] = cols
            skip["b%d" % (l + 1)] = cols
    return skip, total


def lib_share_bounds(synk, count, parts):
    """[(start, stop)] of each share by the LIBRARY's split rule (synk_split): what the HIP leg of a
    test sizes its buffers with.  The oracle's split stays on the checker side."""
    off = synk.synk_split(int(count), int(parts))
    return list(zip(off[:-1], off[1:]))


def lib_share_sizes(synk, count, parts):
    return [b - a for a, b in lib_share_bounds(synk, count, parts)]
