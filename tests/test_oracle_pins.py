"""Pins of the CPU oracle to things other than itself: library routines,
closed forms, finite differences, brute-force loops, autograd on CPU, exact
rational arithmetic and the paper's defining invariant (Sec. 1.1: reducing the
results of independent calls over arbitrary subdivisions of the data gives the
result of the one call)."""
import math
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from oracle import brute, collectives, evalops, gather, mlp, reduce as oreduce, split, update


# ----------------------------------------------------------------- split
@pytest.mark.parametrize("count,parts", [(0, 3), (1, 4), (7, 3), (256, 2), (1024, 8), (13, 13), (5, 8), (100, 7)])
def test_split_matches_array_split(count, parts):
    ref = [len(a) for a in np.array_split(np.arange(count), parts)]
    assert split.share_sizes(count, parts) == ref
    b = split.share_bounds(count, parts)
    assert b[0][0] == 0 and b[-1][1] == count
    assert all(b[i][1] == b[i + 1][0] for i in range(parts - 1))


def test_worker_slice_bounds_tile_the_range():
    for count, n, s in [(256, 2, 4), (10, 3, 4), (3, 4, 2), (1000, 7, 5)]:
        flat = [ab for w in split.worker_slice_bounds(count, n, s) for ab in w]
        assert flat[0][0] == 0 and flat[-1][1] == count
        assert all(flat[i][1] == flat[i + 1][0] for i in range(len(flat) - 1))
        ref = [len(x) for part in np.array_split(np.arange(count), n) for x in np.array_split(part, s)]
        assert [b - a for a, b in flat] == ref


# ---------------------------------------------------------------- gather
def test_gather_matches_take_and_identity():
    rng = np.random.default_rng(0)
    data = rng.standard_normal((50, 7)).astype(np.float32)
    idx = rng.integers(0, 50, 33)
    assert np.array_equal(gather.gather_rows(data, idx), np.take(data, idx, axis=0))
    assert np.array_equal(gather.gather_rows(data, np.arange(50)), data)
    shares = gather.gather_shares(data, idx, 4)
    assert np.array_equal(np.concatenate(shares), np.take(data, idx, axis=0))
    assert [len(s) for s in shares] == [9, 8, 8, 8]
    with pytest.raises(IndexError):
        gather.gather_rows(data, np.array([50]))
    with pytest.raises(IndexError):
        gather.gather_rows(data, np.array([-1]))


def test_normalise_u8_exact_rational():
    mean = np.array([0.485 * 255, 0.456 * 255, 103.53], dtype=np.float32)
    std = np.array([0.229 * 255, 57.12, 0.225 * 255], dtype=np.float32)
    x = np.arange(256, dtype=np.uint8).reshape(1, 1, 256).repeat(3, axis=1)  # [1,3,256]
    got = gather.normalise_u8(x, mean, std)
    assert got.dtype == np.float32
    for c in range(3):
        for val in range(256):
            exact = (Fraction(val) - Fraction(float(mean[c]))) / Fraction(float(std[c]))
            assert got[0, c, val] == np.float32(float(exact))
    # special cases with obvious answers
    one = gather.normalise_u8(x, np.zeros(3, np.float32), np.ones(3, np.float32))
    assert np.array_equal(one[0, 0], np.arange(256, dtype=np.float32))
    pm = gather.normalise_u8(x, np.full(3, 127.5, np.float32), np.full(3, 127.5, np.float32))
    assert pm[0, 1, 0] == -1.0 and pm[0, 1, 255] == 1.0


def test_bf16_rounding_matches_torch_cast():
    rng = np.random.default_rng(1)
    a = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(3.0),
        (rng.standard_normal(2000).astype(np.float32) * np.float32(1e-20)),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 1.0078125, 3.3895314e38, 1e-40], np.float32),
        # exact ties: 1 + k/256 for odd k sit half-way between bf16 neighbours
        (1.0 + np.arange(1, 64, 2) / 256.0).astype(np.float32),
    ])
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    got = gather.round_to_bf16(a)
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    # every exponent, denormals and the overflow to infinity: random finite bit patterns and the edges
    bits = rng.integers(0, 1 << 32, 200000, dtype=np.uint64).astype(np.uint32)
    bits = bits[(bits & 0x7F800000) != 0x7F800000]
    bits = np.concatenate([bits, np.array([0x00000001, 0x00008000, 0x00018000, 0x007FFFFF, 0x7F7FFFFF, 0xFF7FFFFF,
                                           0x7F7F7FFF, 0x7F7F8000, 0x7F800000, 0xFF800000], np.uint32)])
    b = bits.view(np.float32)
    ref = torch.from_numpy(b).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(gather.round_to_bf16(b).view(np.uint32), ref.view(np.uint32))


# ------------------------------------------------------------------- mlp
def _tiny(dims, rows, seed):
    rng = np.random.default_rng(seed)
    P = mlp.param_count(dims)
    theta = rng.standard_normal(P) * 0.5
    X = rng.standard_normal((rows, dims[0]))
    y = rng.integers(0, dims[-1], rows)
    return theta, X, y


def test_hand_worked_example():
    # x=[1,2]; W1=[[1,-1],[.5,1]] -> z1=[2,1]; W2=I -> logits [2,1]; y=0
    dims = [2, 2, 2]
    theta = np.array([1, -1, .5, 1, 0, 0, 1, 0, 0, 1, 0, 0], dtype=np.float64)
    loss, g = mlp.function(theta, dims, np.array([[1.0, 2.0]]), np.array([0]))
    s = 1.0 / (1.0 + math.e)                      # softmax prob of class 1
    assert loss == pytest.approx(math.log1p(math.exp(-1.0)), abs=1e-15)
    exp = [-s, s, -2 * s, 2 * s, -s, s,           # dW1 = x^T dz1, db1
           -2 * s, 2 * s, -s, s, -s, s]           # dW2 = h^T dz2, db2
    assert np.allclose(g, exp, atol=1e-15)


def test_uniform_logits_give_ln_C():
    dims = [5, 4, 10]
    theta, X, y = _tiny(dims, 9, 2)
    (W1, b1), (W2, b2) = mlp.unpack(theta, dims)
    W2[...] = 0.0
    b2[...] = 0.25           # any constant row of logits
    loss, g = mlp.function(theta, dims, X, y)
    assert loss == pytest.approx(math.log(10.0), abs=1e-14)


def test_last_bias_gradient_sums_to_zero():
    dims = [6, 5, 4, 3]
    theta, X, y = _tiny(dims, 11, 3)
    _, g = mlp.function(theta, dims, X, y)
    gb_last = mlp.unpack(g, dims)[-1][1]
    assert abs(gb_last.sum()) < 1e-15


@pytest.mark.parametrize("dims", [[4, 3, 2], [5, 4, 3, 6], [3, 7]])
def test_gradient_finite_differences(dims):
    theta, X, y = _tiny(dims, 6, 4)
    _, g = mlp.function(theta, dims, X, y)
    h = 1e-5
    for k in range(theta.size):
        tp = theta.copy(); tp[k] += h
        tm = theta.copy(); tm[k] -= h
        fd = (mlp.function(tp, dims, X, y)[0] - mlp.function(tm, dims, X, y)[0]) / (2 * h)
        assert abs(fd - g[k]) < 1e-6 * max(1.0, abs(g[k])), (k, fd, g[k])


def test_loss_and_gradient_match_scalar_loops():
    dims = [4, 5, 3]
    theta, X, y = _tiny(dims, 7, 5)
    loss, g = mlp.function(theta, dims, X, y)
    assert loss == pytest.approx(brute.mlp_loss(theta, dims, X, y), abs=1e-13)
    assert np.allclose(g, brute.mlp_grad_two_layer(theta, dims, X, y), atol=1e-13)
    dims3 = [3, 4, 4, 2]
    theta, X, y = _tiny(dims3, 5, 6)
    assert mlp.function(theta, dims3, X, y)[0] == pytest.approx(brute.mlp_loss(theta, dims3, X, y), abs=1e-13)


def test_gradient_matches_cpu_autograd():
    dims = [12, 9, 8, 5]
    theta, X, y = _tiny(dims, 17, 7)
    t = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
    h = torch.tensor(X)
    at = 0
    for l in range(len(dims) - 1):
        k, n = dims[l], dims[l + 1]
        W = t[at:at + k * n].view(k, n); at += k * n
        b = t[at:at + n]; at += n
        h = h @ W + b
        if l < len(dims) - 2:
            h = torch.relu(h)
    loss = torch.nn.functional.cross_entropy(h, torch.tensor(y), reduction="mean")
    loss.backward()
    ol, og = mlp.function(theta, dims, X, y)
    assert ol == pytest.approx(loss.item(), abs=1e-13)
    assert np.allclose(og, t.grad.numpy(), atol=1e-13)


@pytest.mark.parametrize("B,N,S", [(24, 1, 1), (24, 2, 4), (25, 3, 4), (7, 4, 3), (5, 8, 2), (31, 5, 7), (16, 8, 4)])
def test_defining_invariant_sliced_equals_full(B, N, S):
    dims = [6, 5, 4]
    rng = np.random.default_rng(8)
    data = rng.standard_normal((40, 6)); labels = rng.integers(0, 4, 40)
    idx = rng.integers(0, 40, B)
    theta = rng.standard_normal(mlp.param_count(dims)) * 0.4
    fl, fg = mlp.full(theta, dims, data, labels, idx)
    r = mlp.sliced(theta, dims, data, labels, idx, N, S, "mean", worker_weights="rows")
    assert r["loss"] == pytest.approx(fl, abs=1e-13)
    assert np.allclose(r["grad"], fg, atol=1e-13)
    if B % N == 0:     # plain 1/N average is the same thing when shares are equal
        r2 = mlp.sliced(theta, dims, data, labels, idx, N, S, "mean")
        assert np.allclose(r2["grad"], fg, atol=1e-13)
    if N == 1 and S == 1:
        assert np.array_equal(r["grad"], fg)


def test_sum_aggregation_is_the_sum_of_slice_results():
    dims = [4, 3, 3]
    rng = np.random.default_rng(9)
    data = rng.standard_normal((20, 4)); labels = rng.integers(0, 3, 20)
    idx = rng.permutation(20)[:10]
    theta = rng.standard_normal(mlp.param_count(dims))
    r = mlp.sliced(theta, dims, data, labels, idx, 1, 3, "sum")
    tot_g = 0.0; tot_l = 0.0
    for (a, b) in split.share_bounds(10, 3):
        l, g = mlp.function(theta, dims, data[idx[a:b]], labels[idx[a:b]])
        tot_g = tot_g + g; tot_l += l
    assert np.allclose(r["worker_grads"][0], tot_g, atol=1e-14)
    assert r["worker_losses"][0] == pytest.approx(tot_l, abs=1e-14)


def test_index_permutation_invariance():
    dims = [5, 6, 3]
    rng = np.random.default_rng(10)
    data = rng.standard_normal((30, 5)); labels = rng.integers(0, 3, 30)
    idx = rng.integers(0, 30, 12)
    theta = rng.standard_normal(mlp.param_count(dims))
    a = mlp.sliced(theta, dims, data, labels, idx, 3, 2, worker_weights="rows")
    b = mlp.sliced(theta, dims, data, labels, rng.permutation(idx), 3, 2, worker_weights="rows")
    assert np.allclose(a["grad"], b["grad"], atol=1e-13) and a["loss"] == pytest.approx(b["loss"], abs=1e-13)


def test_bf16_points_mode_stays_near_float64():
    dims = [64, 48, 32, 10]
    rng = np.random.default_rng(11)
    theta = np.concatenate([np.r_[(rng.standard_normal(dims[l] * dims[l + 1]) * np.sqrt(2 / dims[l])),
                                  np.zeros(dims[l + 1])] for l in range(3)]).astype(np.float32)
    X = rng.random((32, 64)).astype(np.float32); y = rng.integers(0, 10, 32)
    l0, g0 = mlp.function(theta, dims, X, y)
    l1, g1 = mlp.function(theta, dims, X, y, bf16_points=True)
    assert abs(l1 - l0) < 2e-2 * abs(l0)
    # bf16 inputs move individual gradient entries by a few percent (relu
    # masks of near-zero units change); the band is on the whole array
    assert np.linalg.norm(g1 - g0) < 1e-1 * np.linalg.norm(g0)
    assert np.abs(g1 - g0).max() > 0      # the mode does something


def test_scalar_bf16_rounding_matches_torch_cast():
    rng = np.random.default_rng(31)
    a = np.concatenate([rng.standard_normal(3000) * 10.0 ** rng.uniform(-8, 8, 3000),
                        1.0 + np.arange(1, 512, 2) / 256.0,        # exact ties between bf16 neighbours
                        [0.0, -0.0, 1.0, -1.0, 255.0 / 256.0, 3.3895313892515355e38]])
    want = torch.from_numpy(a).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([brute.bf16_rne(v) for v in a])
    assert np.array_equal(got, want)


def _tiny_mlp(dims, rows, seed):
    rng = np.random.default_rng(seed)
    theta = rng.standard_normal(mlp.param_count(dims)) * 0.7     # biases non-zero on purpose
    X = rng.standard_normal((rows, dims[0]))
    y = rng.integers(0, dims[-1], rows)
    return theta, X, y


@pytest.mark.parametrize("dims,rows", [([5, 4, 3], 6), ([6, 5, 4, 3], 5), ([4, 3], 7), ([3, 4, 4, 4, 2], 4)])
def test_bf16_points_mode_matches_scalar_loop_twin(dims, rows):
    """The rounding points of the bf16 mode (input rows, every W_l, every hidden activation as fed
    forward, every dZ_l before all three of its uses), restated with scalar loops and an
    independent scalar rounding routine."""
    theta, X, y = _tiny_mlp(dims, rows, sum(dims))
    loss, grad = mlp.function(theta, dims, X, y, bf16_points=True)
    tl, tg = brute.mlp_loss_grad_bf16_points(theta, dims, X.tolist(), y)
    assert abs(loss - tl) < 1e-12
    assert np.abs(grad - np.array(tg)).max() < 1e-12
    # with no rounding point active the twin is the float64 function
    l0, g0 = mlp.function(theta, dims, X, y)
    ul, ug = brute.mlp_loss_grad_bf16_points(theta, dims, X.tolist(), y, points=())
    assert abs(l0 - ul) < 1e-12 and np.abs(g0 - np.array(ug)).max() < 1e-12


@pytest.mark.parametrize("points", [
    ("x", "w", "h"),                    # dZ_l not rounded
    ("x", "w", "dz"),                   # hidden activations not rounded
    ("x", "h", "dz"),                   # weights not rounded
    ("w", "h", "dz"),                   # inputs not rounded
    ("x", "w", "h", "dz", "b"),         # biases rounded as well
    ("x", "w", "h", "dz", "late_dz"),   # dZ_l rounded only on its way to dZ_{l-1}, not for dW_l / db_l
])
def test_a_misplaced_rounding_point_is_detected(points):
    """Negative cases: a copy of the twin with one rounding point dropped, added or moved must
    NOT agree with the oracle's bf16 mode (so the agreement above pins every point)."""
    dims, rows = [6, 5, 4, 3], 5
    theta, X, y = _tiny_mlp(dims, rows, sum(dims))
    loss, grad = mlp.function(theta, dims, X, y, bf16_points=True)
    tl, tg = brute.mlp_loss_grad_bf16_points(theta, dims, X.tolist(), y, points=points)
    assert abs(loss - tl) + np.abs(grad - np.array(tg)).max() > 1e-5


def test_bf16_tie_threshold_covers_single_precision_accumulation_noise():
    """Where the GPU tests' threshold for "a hidden pre-activation that is zero up to rounding"
    comes from, using the oracle only.  The kernels accumulate in single precision (the paper's
    precision, Sec. 6), the oracle in double.  A first-layer pre-activation that differs in its last
    single-precision bits can round to the neighbouring bfloat16 activation, which moves every
    second-layer pre-activation that unit feeds by |w| * one bf16 step of h.  Measured here at the
    wide configuration's layer widths: the largest such move is a few 1e-4, so 1e-3 covers it with
    room, and the fraction of pre-activations within 1e-3 of zero stays ~1e-3."""
    import workloads
    cfg = workloads.config2(n_data=256, batch=128)
    dims = cfg["dims"]
    idx = cfg["idx"][:64]
    X, y = gather.gather_rows(cfg["data"], idx), gather.gather_rows(cfg["labels"], idx)
    tr = []
    mlp.function(cfg["theta"], dims, X, y, bf16_points=True, trace=tr)
    (W1, b1), (W2, b2), _ = mlp.unpack(cfg["theta"].astype(np.float64), dims)
    q = lambda a: gather.round_to_bf16(a).astype(np.float64)
    # the oracle's own first layer, re-accumulated in single precision
    z1_single = (q(X).astype(np.float32) @ q(W1).astype(np.float32) + b1.astype(np.float32)).astype(np.float64)
    assert np.abs(z1_single - tr[0]).max() < 1e-4                      # same numbers up to accumulation rounding
    h1_double, h1_single = q(np.maximum(tr[0], 0.0)), q(np.maximum(z1_single, 0.0))
    moved = h1_double != h1_single
    assert 0 < moved.sum() < 0.01 * moved.size                         # a few activations take the other neighbour
    dz2 = np.abs((h1_single - h1_double) @ q(W2))
    assert 1e-5 < dz2.max() < 1e-3                                     # the threshold used on the GPU side
    near = (np.abs(tr[1]) <= 1e-3).mean()
    assert near < 5e-3


def test_bf16_points_mode_distance_to_float64_at_the_wide_configuration():
    """The band the GPU tests use for "bf16 result against the all-float64 oracle" (per tensor and
    whole gradient), measured for the oracle alone at the wide configuration's full model and
    per-worker row count."""
    import sys, os
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    from helpers import BF16_VS_F64_FRO, BF16_VS_F64_MAX, mlp_tensors, rel_err
    import workloads
    cfg = workloads.config2(n_data=2048)
    dims, idx = cfg["dims"], cfg["idx"]
    worst, fro = 0.0, 0.0
    for (a, b) in split.share_bounds(len(idx), cfg["n_workers"])[:3]:
        X, y = gather.gather_rows(cfg["data"], idx[a:b]), gather.gather_rows(cfg["labels"], idx[a:b])
        _, g0 = mlp.function(cfg["theta"], dims, X, y)
        _, g1 = mlp.function(cfg["theta"], dims, X, y, bf16_points=True)
        fro = max(fro, float(np.linalg.norm(g1 - g0) / np.linalg.norm(g0)))
        for (_, t1), (_, t0) in zip(mlp_tensors(g1, dims), mlp_tensors(g0, dims)):
            worst = max(worst, rel_err(t1, t0))
    assert 1e-3 < worst < BF16_VS_F64_MAX and 1e-3 < fro < BF16_VS_F64_FRO, (worst, fro)


def test_relu_tie_flag_changes_only_near_zero_units():
    dims = [3, 2, 2]
    theta = np.array([1, 1, -1, 1, 0, 0.5,   0, 0,   1, -1, 2, 1,   0, 0], dtype=np.float64)
    X = np.array([[1.0, 1.0, 0.0]])            # z1 = [0, 2]: unit 0 sits exactly on the kink
    y = np.array([1])
    tr = []
    _, g = mlp.function(theta, dims, X, y, trace=tr)
    assert np.array_equal(tr[0], [[0.0, 2.0]])
    _, gf = mlp.function(theta, dims, X, y, tie_eps=1e-12, flip_ties=True)
    gW1 = mlp.unpack(g, dims)[0][0]; gW1f = mlp.unpack(gf, dims)[0][0]
    assert np.all(gW1[:, 0] == 0) and np.any(gW1f[:, 0] != 0)      # column of the tied unit
    assert np.array_equal(gW1[:, 1], gW1f[:, 1])
    assert np.array_equal(mlp.unpack(g, dims)[1][0], mlp.unpack(gf, dims)[1][0])


# ---------------------------------------------------------------- reduce
def test_reduce_ops_against_numpy():
    rng = np.random.default_rng(12)
    f = [rng.uniform(0.5, 2.0, 100).astype(np.float32) for _ in range(5)]
    i = [rng.integers(-1000, 1000, 100).astype(np.int32) for _ in range(5)]
    st = np.stack(f).astype(np.float64)
    assert np.allclose(oreduce.reduce_buffers(f, "sum"), st.sum(0), rtol=1e-15)
    assert np.allclose(oreduce.reduce_buffers(f, "mean"), st.mean(0), rtol=1e-15)
    assert np.allclose(oreduce.reduce_buffers(f, "prod"), st.prod(0), rtol=1e-14)
    assert np.array_equal(oreduce.reduce_buffers(f, "max"), st.max(0))
    assert np.array_equal(oreduce.reduce_buffers(f, "min"), st.min(0))
    si = np.stack(i).astype(np.int64)
    assert np.array_equal(oreduce.reduce_buffers(i, "sum"), si.sum(0))
    assert np.array_equal(oreduce.reduce_buffers(i, "max"), si.max(0))
    assert np.array_equal(oreduce.reduce_buffers(i, "min"), si.min(0))
    assert np.array_equal(oreduce.reduce_buffers([f[0][:3], f[1][:5]], "concat"), np.r_[f[0][:3], f[1][:5]])
    with pytest.raises(TypeError):
        oreduce.reduce_buffers(i, "mean")


def test_mean_of_equal_buffers_is_bit_exact_and_pairs_cancel():
    rng = np.random.default_rng(13)
    x = rng.standard_normal(257).astype(np.float32)
    for n in (1, 2, 4, 8):
        out = oreduce.reduce_buffers([x] * n, "mean")
        assert np.array_equal(out.astype(np.float32), x)
    assert np.array_equal(oreduce.reduce_buffers([x, -x, x, -x], "mean"), np.zeros(257))
    x64 = x.astype(np.float64)
    w = oreduce.reduce_buffers([x64, 3 * x64], "mean", weights=[0.25, 0.75])
    assert np.allclose(w, 2.5 * x64, rtol=1e-15)


def test_slice_indexes_scatter_and_resident_gather_against_python_and_numpy():
    rng = np.random.default_rng(121)
    data = rng.standard_normal((29, 5))
    for start, stop, step in [(0, 29, 1), (3, 20, 4), (5, 5, 1), (0, 29, 30), (7, 28, 3)]:
        ix = gather.slice_indexes(start, stop, step)
        assert list(ix) == list(range(start, stop, step))
        assert np.array_equal(gather.gather_rows(data, ix), data[start:stop:step])
    for bad in [(0, 5, 0), (-1, 5, 1), (6, 5, 1)]:
        with pytest.raises(ValueError):
            gather.slice_indexes(*bad)
    for n in (1, 3, 4, 8, 40):
        sh = gather.scatter(data, n)
        ref = np.array_split(data, n)
        assert len(sh) == n and all(np.array_equal(a, b) for a, b in zip(sh, ref))
        assert np.array_equal(np.concatenate(sh), data)
        # scatter == indexing with the full slice, shares taken by the same split rule
        via = gather.gather_shares(data, gather.slice_indexes(0, 29, 1), n)
        assert all(np.array_equal(a, b) for a, b in zip(sh, via))
    shares = gather.scatter(data, 3)
    lists = [rng.integers(0, len(s), 6) for s in shares]
    out = gather.gather_resident(shares, lists)
    assert all(np.array_equal(o, np.take(s, i, axis=0)) for o, s, i in zip(out, shares, lists))
    same = gather.gather_resident(shares, [np.array([1, 0, 1])] * 3)
    assert all(np.array_equal(o, s[[1, 0, 1]]) for o, s in zip(same, shares))
    with pytest.raises(IndexError):
        gather.gather_resident(shares, [np.array([0]), np.array([len(shares[1])]), np.array([0])])
    with pytest.raises(ValueError):
        gather.gather_resident(shares, lists[:2])


# ----------------------------------------------------------- collectives
def test_collectives_against_library_routines_and_invariants():
    rng = np.random.default_rng(131)
    bufs = [rng.standard_normal(37) for _ in range(5)]
    stack = np.stack(bufs)
    for op, ref in (("sum", stack.sum(0)), ("max", stack.max(0)), ("min", stack.min(0)),
                    ("prod", stack.prod(0)), ("mean", stack.mean(0))):
        out = collectives.all_reduce(bufs, op)
        assert len(out) == 5 and all(np.allclose(o, ref, rtol=1e-13, atol=1e-15) for o in out)
        assert all(np.array_equal(o, out[0]) for o in out)          # every worker holds the same result
    # the parameter average (App. A): identical copies are a fixed point, and averaging is idempotent
    same = collectives.all_reduce([bufs[0]] * 4, "mean")
    assert all(np.allclose(o, bufs[0], rtol=1e-15) for o in same)
    once = collectives.all_reduce(bufs, "mean")
    twice = collectives.all_reduce(once, "mean")
    assert np.allclose(twice[0], once[0], rtol=1e-15)
    # results are copies, not views of one array
    once[0][0] = 123.0
    assert once[1][0] != 123.0
    ints = [rng.integers(-9, 9, 11).astype(np.int32) for _ in range(3)]
    assert np.array_equal(collectives.all_reduce(ints, "sum")[2], np.stack(ints).sum(0))
    with pytest.raises(ValueError):
        collectives.all_reduce(bufs, "concat")
    b = collectives.broadcast(bufs[2], 4)
    assert len(b) == 4 and all(np.array_equal(x, bufs[2]) for x in b) and b[0] is not b[1]
    ragged = [rng.standard_normal(k) for k in (3, 0, 7, 1)]
    g = collectives.all_gather(ragged)
    assert len(g) == 4 and all(np.array_equal(x, np.concatenate(ragged)) for x in g)
    # gathering a scattered array returns the array (Sec. 4.2: scatter by first dimension)
    whole = rng.standard_normal(23)
    parts = np.array_split(whole, 4)
    assert np.array_equal(collectives.all_gather(parts)[3], whole)


# ---------------------------------------------------------------- update
def test_sgd_zero_momentum_and_closed_form():
    rng = np.random.default_rng(14)
    p = rng.standard_normal(50); g = rng.standard_normal(50); v = np.zeros(50)
    p1, v1 = update.sgd_momentum(p, v, g, 0.1, 0.0)
    assert np.allclose(p1, p - 0.1 * g, rtol=0, atol=1e-16)
    pk, vk = p.copy(), v.copy()
    for k in range(1, 8):
        pk, vk = update.sgd_momentum(pk, vk, g, 0.05, 0.9)
        assert np.allclose(pk, brute.momentum_closed_form(p, g, 0.05, 0.9, k), atol=1e-13)


def test_sgd_trajectory_matches_torch_optim():
    rng = np.random.default_rng(15)
    p0 = rng.standard_normal(64)
    grads = [rng.standard_normal(64) for _ in range(6)]
    t = torch.nn.Parameter(torch.tensor(p0))
    opt = torch.optim.SGD([t], lr=0.1, momentum=0.9, dampening=0.0, weight_decay=1e-2)
    p, v = p0.copy(), np.zeros(64)
    for g in grads:
        t.grad = torch.tensor(g)
        opt.step()
        p, v = update.sgd_momentum(p, v, g, 0.1, 0.9, 1e-2)
        assert np.allclose(p, t.detach().numpy(), atol=1e-13)


def test_nesterov_trajectory_matches_torch_optim_and_differs_from_momentum():
    rng = np.random.default_rng(151)
    p0 = rng.standard_normal(64)
    grads = [rng.standard_normal(64) for _ in range(6)]
    t = torch.nn.Parameter(torch.tensor(p0))
    opt = torch.optim.SGD([t], lr=0.05, momentum=0.9, nesterov=True, weight_decay=1e-2)
    p, v = p0.copy(), np.zeros(64)
    pm, vm = p0.copy(), np.zeros(64)
    for g in grads:
        t.grad = torch.tensor(g)
        opt.step()
        p, v = update.nesterov_momentum(p, v, g, 0.05, 0.9, 1e-2)
        pm, vm = update.sgd_momentum(pm, vm, g, 0.05, 0.9, 1e-2)
        assert np.allclose(p, t.detach().numpy(), atol=1e-13)
    assert np.abs(p - pm).max() > 1e-3            # the look-ahead term is not a no-op
    # with zero momentum both rules are plain SGD
    a, _ = update.nesterov_momentum(p0, np.zeros(64), grads[0], 0.1, 0.0)
    assert np.allclose(a, p0 - 0.1 * grads[0], atol=1e-16)


def test_rmsprop_against_torch_closed_form_and_hand_numbers():
    rng = np.random.default_rng(152)
    p0 = rng.standard_normal(48)
    grads = [rng.standard_normal(48) for _ in range(5)]
    # eps = 0: eps inside or outside the square root makes no difference -> torch's routine applies
    t = torch.nn.Parameter(torch.tensor(p0))
    opt = torch.optim.RMSprop([t], lr=0.01, alpha=0.9, eps=0.0, weight_decay=1e-2)
    p, a = p0.copy(), np.zeros(48)
    for g in grads:
        t.grad = torch.tensor(g)
        opt.step()
        p, a = update.rmsprop(p, a, g, 0.01, 0.9, 0.0, 1e-2)
        assert np.allclose(p, t.detach().numpy(), atol=1e-12)
    # eps > 0 (inside the root): constant gradient, closed form
    g = rng.standard_normal(48)
    pk, ak = p0.copy(), np.zeros(48)
    for k in range(1, 7):
        pk, ak = update.rmsprop(pk, ak, g, 0.02, 0.9, 1e-6)
        assert np.allclose(pk, brute.rmsprop_constant_gradient(p0, g, 0.02, 0.9, 1e-6, k), atol=1e-13)
    # one element by hand: a = 0.1 * 4 = 0.4 ; p = 1 - 0.5 * 2 / sqrt(0.4 + 0.09) = 1 - 1/0.7
    p1, a1 = update.rmsprop([1.0], [0.0], [2.0], 0.5, 0.9, 0.09)
    assert a1[0] == pytest.approx(0.4, abs=1e-15) and p1[0] == pytest.approx(1.0 - 1.0 / 0.7, abs=1e-14)


def test_adam_against_torch_first_step_closed_form_and_hand_numbers():
    rng = np.random.default_rng(153)
    p0 = rng.standard_normal(48)
    grads = [rng.standard_normal(48) for _ in range(6)]
    # eps = 0: the two published placements of eps coincide -> torch's routine applies
    t = torch.nn.Parameter(torch.tensor(p0))
    opt = torch.optim.Adam([t], lr=0.01, betas=(0.9, 0.999), eps=0.0, weight_decay=1e-2)
    p, m, v = p0.copy(), np.zeros(48), np.zeros(48)
    for k, g in enumerate(grads, 1):
        t.grad = torch.tensor(g)
        opt.step()
        p, m, v = update.adam(p, m, v, g, 0.01, 0.9, 0.999, 0.0, k, 1e-2)
        assert np.allclose(p, t.detach().numpy(), atol=1e-12)
    # eps > 0: the first step from zero moments has a closed form without beta1
    p1, m1, v1 = update.adam(p0, np.zeros(48), np.zeros(48), grads[0], 0.01, 0.9, 0.999, 1e-8, 1)
    assert np.allclose(p1, brute.adam_first_step(p0, grads[0], 0.01, 0.999, 1e-8), atol=1e-14)
    p1b, _, _ = update.adam(p0, np.zeros(48), np.zeros(48), grads[0], 0.01, 0.5, 0.999, 1e-8, 1)
    assert np.allclose(p1, p1b, atol=1e-14)
    # second step, one element, by hand: g = 1 then g = 3, b1 = .5, b2 = .75, lr = 1, eps = 0.5
    #   t=1: m = .5, v = .25 ; t=2: m = .25 + 1.5 = 1.75, v = .1875 + 2.25 = 2.4375
    #   a_2 = sqrt(1 - .5625) / (1 - .25) = sqrt(.4375) / .75
    q, m_, v_ = update.adam([0.0], [0.0], [0.0], [1.0], 1.0, 0.5, 0.75, 0.5, 1)
    q, m_, v_ = update.adam(q, m_, v_, [3.0], 1.0, 0.5, 0.75, 0.5, 2)
    first = -(np.sqrt(0.25) / 0.5) * 0.5 / (np.sqrt(0.25) + 0.5)
    second = -(np.sqrt(0.4375) / 0.75) * 1.75 / (np.sqrt(2.4375) + 0.5)
    assert m_[0] == pytest.approx(1.75, abs=1e-15) and v_[0] == pytest.approx(2.4375, abs=1e-15)
    assert q[0] == pytest.approx(first + second, abs=1e-14)


def test_apply_rule_dispatch_matches_the_rule_functions():
    rng = np.random.default_rng(154)
    p = rng.standard_normal(16); s1 = rng.standard_normal(16) * 0.1; s2 = rng.random(16); g = rng.standard_normal(16)
    h = dict(lr=0.01, momentum=0.9, rho=0.9, beta1=0.9, beta2=0.999, eps=1e-6, t=3, weight_decay=1e-3)
    assert np.array_equal(update.apply_rule("momentum", p, s1, None, g, h)[0], update.sgd_momentum(p, s1, g, 0.01, 0.9, 1e-3)[0])
    assert np.array_equal(update.apply_rule("nesterov", p, s1, None, g, h)[0], update.nesterov_momentum(p, s1, g, 0.01, 0.9, 1e-3)[0])
    assert np.array_equal(update.apply_rule("rmsprop", p, s2, None, g, h)[1], update.rmsprop(p, s2, g, 0.01, 0.9, 1e-6, 1e-3)[1])
    assert np.array_equal(update.apply_rule("adam", p, s1, s2, g, h)[0], update.adam(p, s1, s2, g, 0.01, 0.9, 0.999, 1e-6, 3, 1e-3)[0])
    with pytest.raises(ValueError):
        update.apply_rule("adagrad", p, s1, s2, g, h)


def test_whole_step_independent_of_worker_count():
    # App. A: averaging over workers "preserves the algorithm" for plain SGD.
    dims = [6, 8, 3]
    rng = np.random.default_rng(16)
    data = rng.standard_normal((64, 6)); labels = rng.integers(0, 3, 64)
    idx = rng.permutation(64)[:24]
    theta = rng.standard_normal(mlp.param_count(dims)) * 0.3
    outs = []
    for n, s in [(1, 1), (2, 3), (4, 2), (8, 1)]:
        r = mlp.sliced(theta, dims, data, labels, idx, n, s)
        p2, v2, G, loss = update.reduce_and_update(theta, np.zeros_like(theta), r["worker_grads"],
                                                   0.01, 0.9, 0.0, None, r["worker_losses"])
        outs.append((p2, loss))
    for p2, loss in outs[1:]:
        assert np.allclose(p2, outs[0][0], atol=1e-14) and loss == pytest.approx(outs[0][1], abs=1e-14)


# --------------------------------------------------------------- evalops
def test_evalops_against_library_routines():
    rng = np.random.default_rng(17)
    logits = (rng.standard_normal((200, 37)) * 2).astype(np.float32)
    logits[5, 3] = logits[5, 9] = logits[5].max() + 1.0          # a tie: lowest index wins
    y = rng.integers(0, 37, 200).astype(np.int32)
    r = evalops.function(logits, y)
    am = np.argmax(logits, axis=1)
    assert r["argmax"][5] == 3
    assert np.array_equal(r["argmax"], am)
    assert np.array_equal(r["counts"], np.bincount(am, minlength=37)) and r["counts"].sum() == 200
    assert r["n_correct"][0] == int((am == y).sum())
    assert r["max_logit"][0] == logits.max() and r["min_logit"][0] == logits.min()
    assert r["max_logit"][0] == logits[np.arange(200), am].max()
    ce = (scipy.special.logsumexp(logits.astype(np.float64), axis=1) - logits[np.arange(200), y]).sum()
    assert r["ce_sum"][0] == pytest.approx(ce, rel=1e-14)


@pytest.mark.parametrize("rows,S", [(200, 1), (200, 7), (64, 64), (5, 8), (130, 3)])
def test_evalops_sliced_equals_full(rows, S):
    rng = np.random.default_rng(18)
    logits = (rng.standard_normal((rows, 11)) * 2).astype(np.float32)
    y = rng.integers(0, 11, rows).astype(np.int32)
    a = evalops.function(logits, y); b = evalops.sliced(logits, y, S)
    for k in a:
        if k == "ce_sum":
            assert b[k][0] == pytest.approx(a[k][0], rel=1e-14)
        else:
            assert np.array_equal(a[k], b[k]), k


def test_evalops_permutation_moves_only_the_concat_output():
    rng = np.random.default_rng(19)
    logits = (rng.standard_normal((90, 13)) * 2).astype(np.float32)
    y = rng.integers(0, 13, 90).astype(np.int32)
    perm = rng.permutation(90)
    a = evalops.sliced(logits, y, 4); b = evalops.sliced(logits[perm], y[perm], 4)
    for k in ("counts", "max_logit", "min_logit", "n_correct"):
        assert np.array_equal(a[k], b[k])
    assert np.array_equal(a["argmax"][perm], b["argmax"])
    assert b["ce_sum"][0] == pytest.approx(a["ce_sum"][0], rel=1e-13)
