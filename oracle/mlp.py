"""The gradient "function" of synchronous SGD (Sec. 3.3 step 1) for a ReLU MLP
with softmax cross-entropy, its evaluation in slices with aggregation
(Sec. 5.1), and the reduction of worker results (Sec. 3.2 step 3).

The paper names no model; the configurations fix: layers h_l = relu(h_{l-1} W_l
+ b_l), last layer affine (logits), per-row loss l_i = logsumexp(logits_i) -
logits_i[y_i]; one flat parameter array holding W_1, b_1, W_2, b_2, ... with
W_l stored [d_{l-1} x d_l] row-major (Sec. 3.3: all gradients live in one
flattened array, laid out like the parameters).

All arithmetic is float64.  `bf16_points=True` additionally rounds to bfloat16
the values a bf16-input GEMM would be fed: the input rows, every W_l, every
hidden activation, and every dZ_l; everything else stays float64.
"""
import numpy as np

from . import split
from .gather import gather_rows, round_to_bf16


def param_count(dims):
    return sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1))


def unpack(theta, dims):
    """[(W_l, b_l)] views into the flat array."""
    theta = np.asarray(theta)
    if theta.shape != (param_count(dims),):
        raise ValueError("flat parameter array has the wrong length")
    out = []
    at = 0
    for l in range(len(dims) - 1):
        k, n = dims[l], dims[l + 1]
        W = theta[at:at + k * n].reshape(k, n)
        at += k * n
        b = theta[at:at + n]
        at += n
        out.append((W, b))
    return out


def _q(a, on):
    return round_to_bf16(a).astype(np.float64) if on else a


def row_losses(logits, y):
    """l_i = log(sum_c exp(logits[i,c])) - logits[i, y_i], shifted by the row
    maximum (an exact identity) so nothing overflows."""
    m = logits.max(axis=1, keepdims=True)
    lse = np.log(np.exp(logits - m).sum(axis=1)) + m[:, 0]
    return lse - logits[np.arange(logits.shape[0]), y]


def function(theta, dims, X, y, bf16_points=False, tie_eps=0.0, flip_ties=False, trace=None):
    """Loss and gradient on one set of rows R: returns (mean_i l_i,
    d(mean_i l_i)/d theta as a flat array laid out like theta).
    Empty R returns (0, zeros): the identity of the aggregation.

    The derivative of relu at a pre-activation of exactly 0 is taken as 0.  A
    pre-activation that is 0 up to rounding (|z| <= tie_eps) has two valid
    derivatives; flip_ties=True takes the other one for every such entry, so
    that a caller can accept either (tie_eps: one bound, or one per hidden
    layer).  `trace`, if a list, receives the hidden
    pre-activations z_1 .. z_{L-1}."""
    theta = np.asarray(theta, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    y = np.asarray(y).astype(np.int64)
    rows = X.shape[0]
    grad = np.zeros_like(theta)
    if rows == 0:
        return 0.0, grad
    layers = unpack(theta, dims)
    L = len(layers)

    h = [_q(X, bf16_points)]           # h[l] = input of layer l+1 (as fed to its GEMM)
    pre_mask = []                      # relu masks of hidden layers
    for l, (W, b) in enumerate(layers):
        z = h[l] @ _q(W, bf16_points) + b
        if l < L - 1:
            a = np.maximum(z, 0.0)
            mask = a > 0.0             # derivative of relu at 0 taken as 0
            if flip_ties:
                eps = tie_eps[l] if isinstance(tie_eps, (list, tuple)) else tie_eps
                mask = mask ^ (np.abs(z) <= eps)
            pre_mask.append(mask)
            if trace is not None:
                trace.append(z)
            h.append(_q(a, bf16_points))
        else:
            logits = z

    loss = row_losses(logits, y).mean()

    m = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - m)
    soft = e / e.sum(axis=1, keepdims=True)
    onehot = np.zeros_like(soft)
    onehot[np.arange(rows), y] = 1.0
    dZ = _q((soft - onehot) / rows, bf16_points)

    gl = unpack(grad, dims)
    for l in range(L - 1, -1, -1):
        W, _ = layers[l]
        gW, gb = gl[l]
        gW[...] = h[l].T @ dZ
        gb[...] = dZ.sum(axis=0)
        if l > 0:
            dH = dZ @ _q(W, bf16_points).T
            dZ = _q(dH * pre_mask[l - 1], bf16_points)
    return float(loss), grad


def full(theta, dims, data, labels, idx, bf16_points=False):
    """The one full-batch call: rows data[idx], labels[idx]."""
    return function(theta, dims, gather_rows(data, idx), gather_rows(labels, idx), bf16_points)


def aggregate_slices(values, sizes, op):
    """Sec. 5.1: combine one output's slice results inside a worker.
    mean is weighted by slice row count (the only weighting for which the
    aggregate equals the unsliced call, Sec. 1.1); sum folds in slice order."""
    total = sum(sizes)
    if op == "mean":
        acc = 0.0 * values[0]
        for v, n in zip(values, sizes):
            if n:
                acc = acc + (n / total) * v
        return acc
    if op == "sum":
        acc = 0.0 * values[0]
        for v, n in zip(values, sizes):
            if n:
                acc = acc + v
        return acc
    raise ValueError(op)


def sliced(theta, dims, data, labels, idx, n_workers, n_slices, grad_op="mean",
           worker_weights=None, bf16_points=False):
    """The method, step by step: split idx over workers, then slices (Sec. 3.2,
    5.1, 5.2); run `function` on every slice with the same theta (Sec. 5.1:
    every slice sees the original values); aggregate a worker's slice outputs
    with grad_op; reduce worker outputs with weights omega_w.

    worker_weights: None -> 1/n_workers (plain average of Sec. 3.3 step 2);
    "rows" -> |R_w| / B (equals the full-batch call for any split).

    Returns dict(worker_grads [N x P], worker_losses [N], grad [P], loss).
    """
    idx = np.asarray(idx)
    B = idx.shape[0]
    bounds = split.worker_slice_bounds(B, n_workers, n_slices)
    P = param_count(dims)
    wg = np.zeros((n_workers, P))
    wl = np.zeros(n_workers)
    wrows = []
    for w, slices in enumerate(bounds):
        gs, ls, ns = [], [], []
        for (a, b) in slices:
            Xs = gather_rows(data, idx[a:b])
            ys = gather_rows(labels, idx[a:b])
            l_s, g_s = function(theta, dims, Xs, ys, bf16_points)
            gs.append(g_s)
            ls.append(l_s)
            ns.append(b - a)
        wrows.append(sum(ns))
        if sum(ns):
            wg[w] = aggregate_slices(gs, ns, grad_op)
            wl[w] = aggregate_slices(ls, ns, grad_op)
    if worker_weights is None:
        omega = np.full(n_workers, 1.0 / n_workers)
    elif isinstance(worker_weights, str) and worker_weights == "rows":
        omega = np.asarray(wrows, dtype=np.float64) / B
    else:
        omega = np.asarray(worker_weights, dtype=np.float64)
    G = np.zeros(P)
    loss = 0.0
    for w in range(n_workers):
        G = G + omega[w] * wg[w]
        loss = loss + omega[w] * wl[w]
    return dict(worker_grads=wg, worker_losses=wl, grad=G, loss=float(loss),
                worker_rows=wrows)
