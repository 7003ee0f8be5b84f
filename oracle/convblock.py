"""A second gradient "function" for the sliced call of Sec. 3.2 / 5.1: one
convolution + batch-normalisation block of the kind the scaling study's
network (Sec. 6: ResNet-50 on 3x224x224 images) is built from, closed by that
network's own ending (global average pool, one affine layer, softmax
cross-entropy).

On a set R of n images X_i [H x W x C_in] (channels last) with labels y_i:

  z      = conv3x3(X, Wc)            stride 1, zero padding 1, no bias
  mu_c   = mean of z[:, :, :, c] over all n*H*W positions of R
  var_c  = mean of (z - mu_c)^2 over the same positions (biased)
  xhat   = (z - mu) / sqrt(var + eps)
  a      = relu(gamma * xhat + beta)
  p_i    = mean of a_i over the H*W positions            [n x C_out]
  logits = p Wf + bf;   l_i = logsumexp(logits_i) - logits_i[y_i]
  loss_R = mean_i l_i;  g_R = d loss_R / d theta

The statistics are those of the rows the function is called on: a slice of a
worker's share is one call (Sec. 5.1), so every slice normalises with its own
mu and var, and the sliced result is the row-weighted mean of the slice
results, not the result of one call on the whole share.

theta is one flat array (Sec. 3.3): Wc [3 x 3 x C_in x C_out] (tap-major, i.e.
the [9 C_in x C_out] matrix of the convolution written as a product), gamma
[C_out], beta [C_out], Wf [C_out x classes], bf [classes].

All arithmetic is float64.  `bf16_points=True` additionally rounds to bfloat16
what a bf16 pipeline keeps in bfloat16: the operands of the two contractions
(X, Wc, dz) and the convolution's output z as stored (statistics,
normalisation and everything after it see the rounded z); the rest stays
float64.
"""
import numpy as np

from . import split
from .gather import gather_rows, round_to_bf16
from .mlp import aggregate_slices, row_losses


def param_count(shape):
    H, W, cin, cout, classes = shape
    return 9 * cin * cout + 2 * cout + cout * classes + classes


def unpack(theta, shape):
    """(Wc, gamma, beta, Wf, bf) as views into the flat array."""
    H, W, cin, cout, classes = shape
    theta = np.asarray(theta)
    if theta.shape != (param_count(shape),):
        raise ValueError("flat parameter array has the wrong length")
    at = 0
    Wc = theta[at:at + 9 * cin * cout].reshape(3, 3, cin, cout)
    at += 9 * cin * cout
    gamma = theta[at:at + cout]
    at += cout
    beta = theta[at:at + cout]
    at += cout
    Wf = theta[at:at + cout * classes].reshape(cout, classes)
    at += cout * classes
    bf = theta[at:at + classes]
    return Wc, gamma, beta, Wf, bf


def _q(a, on):
    return round_to_bf16(a).astype(np.float64) if on else a


def pad1(X):
    """Zero border of one pixel around every image: [n,H,W,C] -> [n,H+2,W+2,C]."""
    n, H, W, C = X.shape
    Xp = np.zeros((n, H + 2, W + 2, C), dtype=X.dtype)
    Xp[:, 1:H + 1, 1:W + 1, :] = X
    return Xp


def conv3x3(X, Wc):
    """z[i,h,w,o] = sum_{kh,kw,c} Xpad[i,h+kh,w+kw,c] Wc[kh,kw,c,o], where Xpad is
    X with a zero border (so tap (1,1) is the pixel itself)."""
    n, H, W, _ = X.shape
    Xp = pad1(X)
    z = np.zeros((n, H, W, Wc.shape[3]))
    for kh in range(3):
        for kw in range(3):
            z += Xp[:, kh:kh + H, kw:kw + W, :] @ Wc[kh, kw]
    return z


def conv3x3_weight_grad(X, dz):
    """g[kh,kw,c,o] = sum_{i,h,w} Xpad[i,h+kh,w+kw,c] dz[i,h,w,o]."""
    n, H, W, cin = X.shape
    Xp = pad1(X)
    g = np.zeros((3, 3, cin, dz.shape[3]))
    for kh in range(3):
        for kw in range(3):
            g[kh, kw] = np.einsum("ihwc,ihwo->co", Xp[:, kh:kh + H, kw:kw + W, :], dz)
    return g


def function(theta, shape, X, y, eps=1e-5, bf16_points=False, trace=None):
    """Loss and gradient on one set of images: returns (mean_i l_i, its gradient
    as a flat array laid out like theta).  X: [n, H*W*C_in] rows (channels
    last) or [n,H,W,C_in].  Empty R returns (0, zeros).  `trace`, if a dict,
    receives z, mu, var, p."""
    H, W, cin, cout, classes = shape
    theta = np.asarray(theta, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64).reshape(-1, H, W, cin)
    y = np.asarray(y).astype(np.int64)
    n = X.shape[0]
    grad = np.zeros_like(theta)
    if n == 0:
        return 0.0, grad
    Wc, gamma, beta, Wf, bf = unpack(theta, shape)
    gWc, ggamma, gbeta, gWf, gbf = unpack(grad, shape)

    Xq = _q(X, bf16_points)
    z = _q(conv3x3(Xq, _q(Wc, bf16_points)), bf16_points)
    mu = z.mean(axis=(0, 1, 2))
    var = ((z - mu) ** 2).mean(axis=(0, 1, 2))
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (z - mu) * rstd
    yb = gamma * xhat + beta
    a = np.maximum(yb, 0.0)
    p = a.mean(axis=(1, 2))
    logits = p @ Wf + bf
    loss = row_losses(logits, y).mean()
    if trace is not None:
        trace.update(z=z, mu=mu, var=var, p=p, logits=logits)

    m = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - m)
    soft = e / e.sum(axis=1, keepdims=True)
    onehot = np.zeros_like(soft)
    onehot[np.arange(n), y] = 1.0
    dlogits = (soft - onehot) / n

    gWf[...] = p.T @ dlogits
    gbf[...] = dlogits.sum(axis=0)
    dp = dlogits @ Wf.T
    da = np.broadcast_to(dp[:, None, None, :] / (H * W), z.shape)
    dy = da * (yb > 0.0)                   # derivative of relu at 0 taken as 0
    gbeta[...] = dy.sum(axis=(0, 1, 2))
    ggamma[...] = (dy * xhat).sum(axis=(0, 1, 2))
    cnt = n * H * W
    dz = gamma * rstd * (dy - gbeta / cnt - xhat * (ggamma / cnt))
    gWc[...] = conv3x3_weight_grad(Xq, _q(dz, bf16_points))
    return float(loss), grad


def sliced(theta, shape, data, labels, idx, n_workers, n_slices, grad_op="mean",
           worker_weights=None, eps=1e-5, bf16_points=False):
    """Split idx over workers, then slices (Sec. 3.2, 5.1, 5.2); one call of
    `function` per slice, all with the same theta; a worker's slice outputs
    are aggregated with grad_op; worker outputs are reduced with weights
    omega_w (None: 1/n_workers, Sec. 3.3 step 2; "rows": |R_w| / B).

    Returns dict(worker_grads [N x P], worker_losses [N], grad [P], loss,
    worker_rows)."""
    idx = np.asarray(idx)
    B = idx.shape[0]
    bounds = split.worker_slice_bounds(B, n_workers, n_slices)
    P = param_count(shape)
    wg = np.zeros((n_workers, P))
    wl = np.zeros(n_workers)
    wrows = []
    for w, slices in enumerate(bounds):
        gs, ls, ns = [], [], []
        for (a, b) in slices:
            l_s, g_s = function(theta, shape, gather_rows(data, idx[a:b]),
                                gather_rows(labels, idx[a:b]), eps, bf16_points)
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
    return dict(worker_grads=wg, worker_losses=wl, grad=G, loss=float(loss), worker_rows=wrows)
