"""Pins of the conv + BN block oracle (oracle/convblock.py) to things other
than itself: scalar-loop restatements of the definitions, torch's CPU
convolution / batch-norm / cross-entropy with autograd (float64), central
finite differences of the forward pass, the special cases that reduce to a
matrix product, and the invariants batch normalisation fixes."""
import numpy as np
import pytest
import torch

import workloads
from oracle import brute, convblock, mlp


def _tiny(shape, n, seed):
    rng = np.random.default_rng(seed)
    H, W, cin, cout, classes = shape
    theta = workloads.convblock_init(shape, rng).astype(np.float64)
    theta[-classes:] = rng.standard_normal(classes) * 0.1   # non-zero last bias
    X = rng.standard_normal((n, H, W, cin))
    y = rng.integers(0, classes, n)
    return theta, X, y


def test_conv_matches_scalar_loops_at_every_border_case():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((2, 3, 4, 2))
    Wc = rng.standard_normal((3, 3, 2, 3))
    z = convblock.conv3x3(X, Wc)
    for i in range(2):
        for h in range(3):
            for w in range(4):
                for o in range(3):
                    assert abs(z[i, h, w, o] - brute.conv3x3_point(X.tolist(), Wc.tolist(), i, h, w, o)) < 1e-12


def test_conv_and_weight_gradient_match_torch():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((3, 5, 6, 4))
    Wc = rng.standard_normal((3, 3, 4, 7))
    dz = rng.standard_normal((3, 5, 6, 7))
    xt = torch.from_numpy(X).permute(0, 3, 1, 2)
    wt = torch.from_numpy(Wc).permute(3, 2, 0, 1).clone().requires_grad_(True)
    zt = torch.nn.functional.conv2d(xt, wt, padding=1)
    np.testing.assert_allclose(convblock.conv3x3(X, Wc), zt.detach().permute(0, 2, 3, 1).numpy(), atol=1e-12)
    (zt * torch.from_numpy(dz).permute(0, 3, 1, 2)).sum().backward()
    np.testing.assert_allclose(convblock.conv3x3_weight_grad(X, dz), wt.grad.permute(2, 3, 1, 0).numpy(),
                               atol=1e-11)


def test_one_pixel_images_reduce_to_a_matrix_product():
    # H = W = 1: only the centre tap sees the pixel.
    rng = np.random.default_rng(3)
    X = rng.standard_normal((5, 1, 1, 6))
    Wc = rng.standard_normal((3, 3, 6, 4))
    np.testing.assert_allclose(convblock.conv3x3(X, Wc)[:, 0, 0, :], X[:, 0, 0, :] @ Wc[1, 1], atol=1e-13)


def test_loss_matches_scalar_loops():
    shape = (3, 2, 2, 3, 4)
    theta, X, y = _tiny(shape, 3, 4)
    loss, _ = convblock.function(theta, shape, X, y, eps=1e-3)
    assert abs(loss - brute.convblock_loss(theta, shape, X.tolist(), y, 1e-3)) < 1e-12


@pytest.mark.parametrize("shape,n", [((4, 5, 3, 6, 7), 4), ((1, 1, 2, 3, 2), 5), ((6, 3, 8, 8, 10), 2)])
def test_loss_and_gradient_match_cpu_autograd(shape, n):
    H, W, cin, cout, classes = shape
    theta, X, y = _tiny(shape, n, 5)
    eps = 1e-5
    loss, grad = convblock.function(theta, shape, X, y, eps=eps)
    t = torch.from_numpy(theta.copy()).requires_grad_(True)
    at = 0
    wc = t[at:at + 9 * cin * cout].reshape(3, 3, cin, cout).permute(3, 2, 0, 1)
    at += 9 * cin * cout
    gamma = t[at:at + cout]; at += cout
    beta = t[at:at + cout]; at += cout
    wf = t[at:at + cout * classes].reshape(cout, classes); at += cout * classes
    bf = t[at:]
    z = torch.nn.functional.conv2d(torch.from_numpy(X).permute(0, 3, 1, 2), wc, padding=1)
    a = torch.relu(torch.nn.functional.batch_norm(z, None, None, gamma, beta, training=True, eps=eps))
    logits = a.mean(dim=(2, 3)) @ wf + bf
    lt = torch.nn.functional.cross_entropy(logits, torch.from_numpy(y))
    lt.backward()
    assert abs(loss - lt.item()) < 1e-12
    np.testing.assert_allclose(grad, t.grad.numpy(), atol=1e-10, rtol=1e-9)


def test_gradient_finite_differences():
    shape = (4, 3, 3, 5, 6)
    theta, X, y = _tiny(shape, 3, 6)
    _, grad = convblock.function(theta, shape, X, y)
    rng = np.random.default_rng(7)
    P = theta.size
    bounds = np.cumsum([0, 9 * 3 * 5, 5, 5, 5 * 6, 6])
    picks = np.concatenate([rng.integers(bounds[j], bounds[j + 1], 6) for j in range(5)])
    h = 1e-6
    for j in picks:
        tp, tm = theta.copy(), theta.copy()
        tp[j] += h
        tm[j] -= h
        fd = (convblock.function(tp, shape, X, y)[0] - convblock.function(tm, shape, X, y)[0]) / (2 * h)
        assert abs(fd - grad[j]) < 1e-7 * max(1.0, abs(grad[j])), (j, fd, grad[j])
    assert picks.max() < P


def test_batch_norm_invariants():
    shape = (5, 4, 3, 6, 5)
    theta, X, y = _tiny(shape, 4, 8)
    tr = {}
    loss, grad = convblock.function(theta, shape, X, y, trace=tr)
    # the statistics are the plain mean and biased variance over images and positions
    zf = tr["z"].reshape(-1, 6)
    np.testing.assert_allclose(tr["mu"], zf.mean(axis=0), atol=1e-14)
    np.testing.assert_allclose(tr["var"], zf.var(axis=0), atol=1e-14)
    # normalisation removes scale and shift of z: scaling Wc by a constant changes
    # nothing but the eps term, so with eps = 0 the loss is unchanged and the
    # gradient wrt Wc shrinks by that constant
    l1, g1 = convblock.function(theta, shape, X, y, eps=0.0)
    t2 = theta.copy()
    t2[:9 * 3 * 6] *= 4.0
    l2, g2 = convblock.function(t2, shape, X, y, eps=0.0)
    assert abs(l1 - l2) < 1e-12
    np.testing.assert_allclose(g2[:9 * 3 * 6] * 4.0, g1[:9 * 3 * 6], atol=1e-12)
    np.testing.assert_allclose(g2[9 * 3 * 6:], g1[9 * 3 * 6:], atol=1e-12)
    # (Wc . dL/dWc) = 0 for a scale-invariant loss (Euler's relation, degree 0)
    assert abs(np.dot(theta[:9 * 3 * 6], g1[:9 * 3 * 6])) < 1e-12
    # softmax cross-entropy: the last bias gradient sums to zero
    assert abs(grad[-5:].sum()) < 1e-14


def test_sliced_call_is_the_row_weighted_mean_of_independent_slice_calls():
    shape = (3, 3, 2, 4, 3)
    rng = np.random.default_rng(9)
    data = rng.standard_normal((20, 3 * 3 * 2))
    labels = rng.integers(0, 3, 20)
    theta = workloads.convblock_init(shape, rng).astype(np.float64)
    idx = rng.integers(0, 20, 11)
    out = convblock.sliced(theta, shape, data, labels, idx, n_workers=2, n_slices=2)
    # worker 0 holds idx[0:6] as slices [0:3],[3:6]; worker 1 idx[6:11] as [6:9],[9:11]
    def call(a, b):
        return convblock.function(theta, shape, data[idx[a:b]], labels[idx[a:b]])
    l00, g00 = call(0, 3); l01, g01 = call(3, 6); l10, g10 = call(6, 9); l11, g11 = call(9, 11)
    np.testing.assert_allclose(out["worker_grads"][0], 0.5 * g00 + 0.5 * g01, atol=1e-14)
    np.testing.assert_allclose(out["worker_grads"][1], 0.6 * g10 + 0.4 * g11, atol=1e-14)
    np.testing.assert_allclose(out["worker_losses"], [0.5 * (l00 + l01), 0.6 * l10 + 0.4 * l11], atol=1e-14)
    np.testing.assert_allclose(out["grad"], 0.5 * (out["worker_grads"][0] + out["worker_grads"][1]), atol=1e-14)
    # with per-slice statistics the sliced call is NOT the unsliced one
    _, gfull = call(0, 6)
    assert np.abs(out["worker_grads"][0] - gfull).max() > 1e-4
    s = convblock.sliced(theta, shape, data, labels, idx, 2, 2, grad_op="sum")
    np.testing.assert_allclose(s["worker_grads"][1], g10 + g11, atol=1e-14)


def test_bf16_points_mode_stays_near_float64():
    shape = (6, 6, 8, 8, 10)
    theta, X, y = _tiny(shape, 4, 10)
    l0, g0 = convblock.function(theta, shape, X, y)
    l1, g1 = convblock.function(theta, shape, X, y, bf16_points=True)
    assert abs(l0 - l1) < 2e-2
    assert np.linalg.norm(g1 - g0) < 1e-1 * np.linalg.norm(g0)
    assert np.abs(g1 - g0).max() > 0.0


# ------------------------------------------------- the bf16 mode, pinned by autograd on the CPU
def _bf(t):
    """float64 tensor -> single precision -> bfloat16 (torch's casts, nearest-even) -> float64."""
    return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)


class _RoundOperand(torch.autograd.Function):
    """A contraction operand stored in bfloat16: the forward value is rounded, the gradient with
    respect to the unrounded value is passed through unchanged."""

    @staticmethod
    def forward(ctx, x):
        return _bf(x)

    @staticmethod
    def backward(ctx, g):
        return g


class _RoundStoredZ(torch.autograd.Function):
    """The convolution's output as a bf16 pipeline stores it.  Forward: everything after the
    convolution sees the rounded z.  Backward: the gradient arriving here IS dz, the operand of the
    weight-gradient contraction, so it is rounded on its way in.  `fwd` / `bwd` switch the two
    roundings so that a test can misplace one."""

    @staticmethod
    def forward(ctx, z, fwd, bwd):
        ctx.bwd = bwd
        return _bf(z) if fwd else z.clone()

    @staticmethod
    def backward(ctx, g):
        return (_bf(g) if ctx.bwd else g), None, None


def _autograd_bf16_twin(theta, shape, X, y, eps, round_x=True, round_w=True, round_z=True, round_dz=True):
    H, W, cin, cout, classes = shape
    t = torch.from_numpy(theta.copy()).requires_grad_(True)
    at = 0
    wc = t[at:at + 9 * cin * cout].reshape(3, 3, cin, cout).permute(3, 2, 0, 1)
    at += 9 * cin * cout
    gamma = t[at:at + cout]; at += cout
    beta = t[at:at + cout]; at += cout
    wf = t[at:at + cout * classes].reshape(cout, classes); at += cout * classes
    bf = t[at:]
    xt = torch.from_numpy(X).permute(0, 3, 1, 2)
    if round_x:
        xt = _bf(xt)
    if round_w:
        wc = _RoundOperand.apply(wc)
    z = torch.nn.functional.conv2d(xt, wc, padding=1)
    z = _RoundStoredZ.apply(z, round_z, round_dz)
    a = torch.relu(torch.nn.functional.batch_norm(z, None, None, gamma, beta, training=True, eps=eps))
    logits = a.mean(dim=(2, 3)) @ wf + bf
    lt = torch.nn.functional.cross_entropy(logits, torch.from_numpy(y))
    lt.backward()
    return lt.item(), t.grad.numpy()


@pytest.mark.parametrize("shape,n", [((4, 5, 3, 6, 7), 4), ((6, 3, 8, 8, 10), 2), ((3, 3, 2, 4, 3), 5)])
def test_bf16_points_mode_matches_autograd_with_rounded_operands(shape, n):
    """bf16 mode of the block = the float64 block with X, Wc rounded where they enter the forward
    contraction, z rounded as stored (statistics, normalisation and all later steps see the rounded
    z) and dz rounded where it enters the weight-gradient contraction; restated with torch's
    convolution, batch norm, cross-entropy, autograd and bfloat16 casts."""
    theta, X, y = _tiny(shape, n, 21)
    loss, grad = convblock.function(theta, shape, X, y, eps=1e-5, bf16_points=True)
    tl, tg = _autograd_bf16_twin(theta, shape, X, y, 1e-5)
    assert abs(loss - tl) < 1e-12
    np.testing.assert_allclose(grad, tg, atol=1e-10, rtol=1e-9)


@pytest.mark.parametrize("drop", ["round_x", "round_w", "round_z", "round_dz"])
def test_a_misplaced_rounding_point_of_the_block_is_detected(drop):
    shape, n = (4, 5, 3, 6, 7), 4
    theta, X, y = _tiny(shape, n, 21)
    loss, grad = convblock.function(theta, shape, X, y, eps=1e-5, bf16_points=True)
    tl, tg = _autograd_bf16_twin(theta, shape, X, y, 1e-5, **{drop: False})
    assert abs(loss - tl) + np.abs(grad - tg).max() > 1e-6


def test_cost_of_storing_z_in_bf16_against_float64():
    """What the bf16 mode costs against the all-float64 block, per tensor (max-norm, relative to the
    tensor's largest entry), and how much of that is the rounding of the stored z.  The distance is
    dominated by rounding X and Wc (relu decisions of near-zero normalised values change, and the
    weight gradient of a normalised layer is what is left after its mean terms cancel); storing z in
    bf16 as well does not add to it.  Bounded here so that the figures in the design notes stay true."""
    shape = (14, 14, 64, 64, 10)
    theta, X, y = _tiny(shape, 8, 22)
    l0, g0 = convblock.function(theta, shape, X, y)
    l1, g1 = convblock.function(theta, shape, X, y, bf16_points=True)
    _, g_noz = _autograd_bf16_twin(theta, shape, X, y, 1e-5, round_z=False)     # operands only, z kept exact
    names = ["Wc", "gamma", "beta", "Wf", "bf"]
    band = dict(Wc=1e-1, gamma=1e-2, beta=1e-2, Wf=1e-2, bf=1e-3)
    bounds = np.cumsum([0, 9 * 64 * 64, 64, 64, 64 * 10, 10])
    err = lambda a, b: float(np.abs(a - b).max() / np.abs(b).max())
    for k, name in enumerate(names):
        a, b = bounds[k], bounds[k + 1]
        with_z, without_z = err(g1[a:b], g0[a:b]), err(g_noz[a:b], g0[a:b])
        print("%-5s bf16 mode vs float64 %.2e; operands only (z exact) %.2e" % (name, with_z, without_z))
        assert with_z < band[name] and without_z < band[name]
        assert with_z < 1.5 * without_z + 1e-3          # the stored-z rounding adds nothing material
    assert abs(l1 - l0) < 1e-3 * abs(l0)
