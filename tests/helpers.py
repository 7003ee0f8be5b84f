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


def rel_err_either_tie(got, ref, alt, dims, skip_cols=None):
    """Worst per-tensor error of `got` against `ref`, where a column (= hidden
    unit) may instead match `alt`, the oracle evaluated with the other valid
    relu derivative at pre-activations that are zero up to rounding.
    skip_cols: {tensor name: set(columns)} holding two or more such entries,
    for which neither variant need match."""
    worst = 0.0
    for (name, g), (_, r), (_, a) in zip(mlp_tensors(np.asarray(got, np.float64), dims),
                                         mlp_tensors(np.asarray(ref, np.float64), dims),
                                         mlp_tensors(np.asarray(alt, np.float64), dims)):
        scale = max(np.abs(r).max(), 1e-30)
        e = np.minimum(np.abs(g - r).max(axis=0), np.abs(g - a).max(axis=0))
        if skip_cols and name in skip_cols:
            for j in skip_cols[name]:
                e[j] = 0.0
        worst = max(worst, float(e.max() / scale))
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
