"""GPU parity of the conv + batch-norm block as the sliced gradient function
(synk_sliced_grad_conv) against the CPU oracle, through the C ABI.

fp32 cases are held to 1e-4, bf16-input cases to 2e-2, per tensor as
max|got-ref|/max|ref|.  For bf16 the reference is the oracle with its values
rounded to bfloat16 at the same points as the kernels (X, Wc and dz)."""
import numpy as np
import pytest
import torch

import workloads
from helpers import TOL_BF16, TOL_F32, lib_share_sizes, rel_err
from oracle import convblock as oconv, gather as ogather, split as osplit

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def synk():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1710_04162_amd import binding
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def tensors(flat, shape):
    H, W, cin, cout, classes = shape
    b = np.cumsum([0, 9 * cin * cout, cout, cout, cout * classes, classes])
    return [(n, flat[b[i]:b[i + 1]]) for i, n in enumerate(["Wc", "gamma", "beta", "Wf", "bf"])]


def small_cfg(shape, n_data, seed):
    rng = np.random.default_rng(seed)
    H, W, cin, cout, classes = shape
    theta = workloads.convblock_init(shape, rng)
    theta[-classes:] = (rng.standard_normal(classes) * 0.1).astype(np.float32)
    return dict(shape=shape, data=rng.standard_normal((n_data, H * W * cin)).astype(np.float32),
                labels=rng.integers(0, classes, n_data).astype(np.int32), theta=theta)


def run_gpu(synk, cfg, idx, n_workers, n_slices, op, bf16, eps=1e-5, rows=None):
    shape = cfg["shape"]
    cd = synk.SYNK_BF16 if bf16 else synk.SYNK_F32
    P = synk.synk_convblock_param_count(shape)
    assert P == cfg["theta"].size
    rows = lib_share_sizes(synk, len(idx), n_workers) if rows is None else rows   # the library's split rule
    xdt = torch.bfloat16 if bf16 else torch.float32
    x = [torch.zeros((n, cfg["data"].shape[1]), dtype=xdt, device="cuda") for n in rows]
    y = [torch.zeros(n, dtype=torch.int32, device="cuda") for n in rows]
    synk.synk_gather_rows(dev(cfg["data"]), dev(idx), x, labels=dev(cfg["labels"]), dst_labels=y)
    grad = [torch.full((P,), 123.0, device="cuda") for _ in rows]
    loss = torch.full((len(rows),), -1.0, device="cuda")
    ws = torch.empty(synk.synk_sliced_grad_conv_workspace_bytes(shape, cd, rows, n_slices, eps),
                     dtype=torch.uint8, device="cuda")
    synk.synk_sliced_grad_conv(shape, cd, eps, dev(cfg["theta"]), x, y, rows, n_slices, synk.OP[op], grad, loss, ws)
    torch.cuda.synchronize()
    return [g.cpu().numpy() for g in grad], loss.cpu().numpy()


def check(cfg, idx, n_workers, n_slices, op, bf16, got_g, got_l, eps=1e-5):
    tol = TOL_BF16 if bf16 else TOL_F32
    ref = oconv.sliced(cfg["theta"], cfg["shape"], cfg["data"], cfg["labels"], idx, n_workers, n_slices,
                       grad_op=op, eps=eps, bf16_points=bf16)
    for w in range(n_workers):
        for (name, g), (_, r) in zip(tensors(got_g[w], cfg["shape"]), tensors(ref["worker_grads"][w], cfg["shape"])):
            assert rel_err(g, r) < tol, (w, name, rel_err(g, r))
        assert abs(got_l[w] - ref["worker_losses"][w]) < tol * max(1.0, abs(ref["worker_losses"][w])), w


@pytest.mark.parametrize("shape,B,N,S,op", [
    ((4, 4, 8, 8, 5), 6, 2, 1, "mean"),
    ((5, 7, 8, 24, 10), 13, 3, 2, "mean"),      # ragged shares, ragged slices, odd image sizes
    ((5, 7, 8, 24, 10), 13, 3, 2, "sum"),
    ((9, 6, 16, 8, 3), 7, 2, 3, "mean"),
    ((1, 1, 8, 8, 4), 9, 2, 2, "mean"),         # one-pixel images: only the centre tap
    ((3, 1, 8, 16, 4), 5, 1, 1, "mean"),        # one column: no left / right neighbours
    ((12, 12, 72, 72, 17), 5, 2, 1, "mean"),    # channels beyond one 64-wide tile, chunk with few rows
    ((20, 20, 8, 8, 300), 4, 2, 2, "sum"),      # more than one chunk of pixels per image, classes > 256
    ((7, 5, 128, 72, 6), 5, 2, 2, "mean"),      # two 64-channel input chunks, a ragged output-channel tile
    ((3, 61, 64, 64, 4), 3, 1, 1, "mean"),      # the widest rows the padded-patch kernels take
    ((5, 33, 64, 72, 6), 5, 2, 2, "mean"),      # padded-stream weight gradient, ragged output-channel tile
    ((14, 31, 128, 64, 4), 6, 2, 1, "sum"),     # the same over several runs, two input chunks
    ((2, 62, 64, 64, 4), 3, 1, 1, "mean"),      # one pixel wider: the general kernels
    ((4, 33, 64, 40, 5), 300, 3, 2, "mean"),    # more images than CUs: a forward workgroup walks several images
    ((30, 40, 64, 24, 5), 3, 2, 1, "sum"),      # ten tiles an image in runs over the CUs, 24 output channels
    ((1, 1, 64, 8, 3), 5, 2, 1, "mean"),        # one-pixel images of 64 channels: every block is mostly border
    ((70, 3, 64, 64, 4), 4, 2, 2, "mean"),      # tall narrow images: a padded row is 5 positions
    ((3, 3, 8, 512, 4096), 3, 2, 1, "mean"),    # the largest channel and class counts the call takes
    ((4, 4, 8, 256, 10), 7, 2, 2, "sum"),       # wide block: head workgroups of four images across workers / slices
])
@pytest.mark.parametrize("bf16", [False, True])
def test_sliced_conv_block_matches_oracle(synk, shape, B, N, S, op, bf16):
    cfg = small_cfg(shape, 24, seed=sum(shape) + B)
    idx = np.random.default_rng(B).integers(0, 24, B).astype(np.int32)
    g, l = run_gpu(synk, cfg, idx, N, S, op, bf16)
    check(cfg, idx, N, S, op, bf16, g, l)


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        H, W = int(rng.integers(1, 12)), int(rng.integers(1, 40))
        cin = int(rng.choice([8, 16, 24, 64, 72, 128]))
        cout = int(rng.choice([8, 24, 64, 72, 136]))
        classes = int(rng.integers(2, 40))
        N, S = int(rng.integers(1, 5)), int(rng.integers(1, 4))
        B = int(rng.integers(1, 9))
        cases.append(((H, W, cin, cout, classes), B, N, S, str(rng.choice(["mean", "sum"])), bool(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("shape,B,N,S,op,bf16", _random_cases(16, 20171004))
def test_seeded_random_shapes_match_oracle(synk, shape, B, N, S, op, bf16):
    # odd sizes, every kernel variant (general / padded-patch / row-of-taps / ring by width and
    # channel count), empty workers and empty slices when B < N * S
    cfg = small_cfg(shape, 12, seed=sum(shape) * 7 + B)
    idx = np.random.default_rng(B + N).integers(0, 12, B).astype(np.int32)
    g, l = run_gpu(synk, cfg, idx, N, S, op, bf16)
    check(cfg, idx, N, S, op, bf16, g, l)


def test_workers_without_images_get_zeros(synk):
    shape = (4, 5, 8, 8, 6)
    cfg = small_cfg(shape, 10, seed=3)
    idx = np.array([1, 7], dtype=np.int32)           # 2 images over 4 workers: two workers are empty
    g, l = run_gpu(synk, cfg, idx, 4, 2, "mean", False)
    check(cfg, idx, 4, 2, "mean", False, g, l)
    for w in (2, 3):
        assert not g[w].any() and l[w] == 0.0


def test_label_out_of_range_means_no_target_class(synk):
    shape = (3, 3, 8, 8, 4)
    cfg = small_cfg(shape, 6, seed=4)
    cfg["labels"][2] = 9
    idx = np.array([0, 2, 3], dtype=np.int32)
    g, l = run_gpu(synk, cfg, idx, 1, 1, "mean", False)
    assert np.isfinite(g[0]).all() and np.isfinite(l).all()
    # the other images' labels still act: against an oracle call with image 2's
    # loss term replaced by logsumexp alone the bias gradient sums to 1/3
    assert abs(g[0][-4:].sum() - 1.0 / 3.0) < 1e-5


def test_two_calls_reuse_the_workspace(synk):
    shape = (6, 6, 8, 16, 5)
    cfg = small_cfg(shape, 12, seed=5)
    idx = np.arange(8, dtype=np.int32)
    a = run_gpu(synk, cfg, idx, 2, 2, "mean", True)
    b = run_gpu(synk, cfg, idx, 2, 2, "mean", True)
    for x, y in zip(a[0], b[0]):
        assert np.array_equal(x, y)      # run-to-run reproducible: fixed summation orders


@pytest.mark.parametrize("bf16", [False, True])
def test_mid_size_block_spans_many_tiles(synk, bf16):
    # 3 workers x 2 slices, 28 x 28 x 64 -> 64: several 128-pixel tiles per unit with a ragged
    # last one, a full 64-wide channel tile, several runs of the weight gradient
    shape = (28, 28, 64, 64, 100)
    cfg = small_cfg(shape, 16, seed=6)
    idx = np.random.default_rng(6).integers(0, 16, 11).astype(np.int32)
    g, l = run_gpu(synk, cfg, idx, 3, 2, "mean", bf16)
    check(cfg, idx, 3, 2, "mean", bf16, g, l)


def test_full_size_config6_every_worker_against_oracle(synk):
    # the bench's launch configuration; the oracle computes all eight workers (about 2 s each)
    cfg = workloads.config6()
    bf16 = cfg["compute"] == "bf16"
    g, l = run_gpu(synk, cfg, cfg["idx"], cfg["n_workers"], cfg["n_slices"], "mean", bf16, eps=cfg["eps"])
    bounds = osplit.share_bounds(len(cfg["idx"]), cfg["n_workers"])
    worst_mirror, worst_f64 = 0.0, {}
    for w in range(cfg["n_workers"]):
        a, b = bounds[w]
        lr, gr = oconv.function(cfg["theta"], cfg["shape"], ogather.gather_rows(cfg["data"], cfg["idx"][a:b]),
                                ogather.gather_rows(cfg["labels"], cfg["idx"][a:b]), eps=cfg["eps"],
                                bf16_points=bf16)
        for (name, gg), (_, r) in zip(tensors(g[w], cfg["shape"]), tensors(gr, cfg["shape"])):
            assert rel_err(gg, r) < TOL_BF16, (w, name, rel_err(gg, r))
            worst_mirror = max(worst_mirror, rel_err(gg, r))
        assert abs(l[w] - lr) < TOL_BF16 * max(1.0, abs(lr))
        # second distance: against the all-float64 block (no rounding anywhere).  The oracle's own bf16 mode sits
        # 4-5 % from it on the convolution weights at this shape (relu decisions of near-zero normalised values
        # change; bounded on the CPU in tests/test_oracle_convblock.py) and below 2e-3 on the other tensors.
        _, g64 = oconv.function(cfg["theta"], cfg["shape"], ogather.gather_rows(cfg["data"], cfg["idx"][a:b]),
                                ogather.gather_rows(cfg["labels"], cfg["idx"][a:b]), eps=cfg["eps"])
        for (name, gg), (_, r) in zip(tensors(g[w], cfg["shape"]), tensors(g64, cfg["shape"])):
            e = rel_err(gg, r)
            worst_f64[name] = max(worst_f64.get(name, 0.0), e)
            assert e < (1e-1 if name == "Wc" else 1e-2) + TOL_BF16, (w, name, e)
    print("config 6: worst per-tensor error against the oracle rounded at the bf16 points %.2e; against the "
          "float64 oracle %s" % (worst_mirror, ", ".join("%s %.2e" % kv for kv in worst_f64.items())))
    for w in range(cfg["n_workers"]):
        assert np.isfinite(g[w]).all()
        assert abs(g[w][-cfg["shape"][4]:].sum()) < 1e-5      # softmax: the last bias gradient sums to zero


# ------------------------------------------------------------- input indexing folded into the call
def _indexed_equals_gather_then_grad(synk, shape, n_data, B, N, S, bf16, seed, bad_index=False):
    """synk_sliced_grad_conv_indexed == synk_gather_rows + synk_sliced_grad_conv, bit for bit."""
    cfg = small_cfg(shape, n_data, seed)
    rng = np.random.default_rng(seed + 1)
    idx = rng.integers(0, n_data, B).astype(np.int32)
    ref_idx = idx.copy()
    if bad_index:                      # the kernels that read through the list take row 0 for such an index
        idx[1], idx[B - 1] = n_data + 3, -2
        ref_idx[1], ref_idx[B - 1] = 0, 0
    ga, la = run_gpu(synk, cfg, ref_idx, N, S, "mean", bf16)
    cd = synk.SYNK_BF16 if bf16 else synk.SYNK_F32
    P = synk.synk_convblock_param_count(shape)
    data = dev(cfg["data"])
    if bf16:
        data = data.bfloat16()
    gb = [torch.full((P,), 7.0, device="cuda") for _ in range(N)]
    lb = torch.full((N,), -2.0, device="cuda")
    ws = torch.full((synk.synk_sliced_grad_conv_indexed_workspace_bytes(shape, cd, B, N, S),), 0x5A, dtype=torch.uint8,
                    device="cuda")
    for _ in range(2):                 # the second call runs on a workspace the first has used
        synk.synk_sliced_grad_conv_indexed(shape, cd, 1e-5, dev(cfg["theta"]), data, dev(cfg["labels"]), dev(idx), S,
                                           synk.SYNK_MEAN, gb, lb, ws)
    torch.cuda.synchronize()
    for w in range(N):
        assert np.array_equal(gb[w].cpu().numpy().view(np.uint32), ga[w].view(np.uint32)), w
    assert np.array_equal(lb.cpu().numpy().view(np.uint32), la.view(np.uint32))


@pytest.mark.parametrize("shape,n_data,B,N,S,bf16", [
    ((40, 33, 64, 64, 10), 30, 16, 4, 1, True),      # both convolution kernels read through the index list
    ((34, 61, 128, 32, 7), 12, 9, 4, 2, True),       # two 64-channel chunks, ragged shares, two slices
    ((56, 56, 64, 64, 1000), 70, 64, 8, 1, True),    # the configuration's shape
    ((12, 12, 64, 16, 5), 20, 10, 3, 1, True),       # narrow images: the call gathers first
    ((9, 11, 8, 16, 5), 20, 10, 3, 2, False),        # fp32: the call gathers first
])
def test_indexed_conv_call_equals_gather_then_call(synk, shape, n_data, B, N, S, bf16):
    _indexed_equals_gather_then_grad(synk, shape, n_data, B, N, S, bf16, seed=sum(shape) + B)


def test_indexed_conv_call_with_an_index_out_of_range(synk):
    _indexed_equals_gather_then_grad(synk, (40, 33, 64, 64, 10), 30, 16, 4, 1, True, seed=5, bad_index=True)
