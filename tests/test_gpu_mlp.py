"""GPU parity of the sliced gradient function and of the whole synchronous-SGD
step (gather -> sliced grad -> reduce -> momentum update) against the CPU
oracle, through the C ABI.

fp32 cases are held to 1e-4, bf16-input cases to 2e-2, both as per-tensor
max|got-ref|/max|ref|.  For bf16 the reference is the oracle with its values
rounded to bfloat16 at the same points as the kernels (the distance of that
reference to the all-float64 one is a property of bf16 inputs, checked on the
CPU).  A hidden pre-activation that is zero up to accumulation rounding has two
valid relu derivatives; for the column of such a unit either is accepted."""
import numpy as np
import pytest
import torch

import workloads
from helpers import (BF16_VS_F64_FRO, BF16_VS_F64_MAX, TOL_BF16, TOL_F32, lib_share_sizes, mlp_tensors, rel_err,
                     rel_err_either_tie, tie_columns)
from oracle import gather as ogather, mlp as omlp, split as osplit, update as oupdate

pytestmark = pytest.mark.gpu

# |z| below which a hidden pre-activation counts as "zero up to rounding".  fp32:
# accumulation error of a few-thousand-term sum.  bf16: single- against double-precision
# accumulation lets an activation of the layer below round to the neighbouring bf16 value, which
# moves z by up to 5e-4 at the wide configuration's widths (derived from the oracle alone in
# tests/test_oracle_pins.py::test_bf16_tie_threshold_covers_single_precision_accumulation_noise).
TIE_EPS = {"f32": 2e-6, "bf16": 1e-3}


@pytest.fixture(scope="module")
def synk():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1710_04162_amd import binding
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


class Step:
    """Device state of one training setup; every compute step is a libsynk call."""

    def __init__(self, synk, cfg):
        self.s, self.cfg = synk, cfg
        self.dims = cfg["dims"]
        self.bf16 = cfg["compute"] == "bf16"
        self.cd = synk.SYNK_BF16 if self.bf16 else synk.SYNK_F32
        self.P = synk.synk_mlp_param_count(self.dims)
        self.data, self.labels = dev(cfg["data"]), dev(cfg["labels"])
        self.p = dev(cfg["theta"])
        self.v = torch.zeros(self.P, device="cuda")
        self.p_lp = torch.zeros(self.P, dtype=torch.bfloat16, device="cuda") if self.bf16 else None
        if self.bf16:
            synk.synk_cast_bf16(self.p, self.p_lp)

    def gather(self, idx, n_workers):
        B = len(idx)
        self.rows = lib_share_sizes(self.s, B, n_workers)        # the HIP leg sizes its buffers by synk_split
        assert self.rows == osplit.share_sizes(B, n_workers)      # ... which the checker's rule must agree with
        xdt = torch.bfloat16 if self.bf16 else torch.float32
        self.x = [torch.zeros((n, self.dims[0]), dtype=xdt, device="cuda") for n in self.rows]
        self.y = [torch.zeros(n, dtype=torch.int32, device="cuda") for n in self.rows]
        self.s.synk_gather_rows(self.data, dev(idx), self.x, labels=self.labels, dst_labels=self.y)

    def sliced_grad(self, n_slices, op):
        n = len(self.rows)
        self.grad = [torch.full((self.P,), 123.0, device="cuda") for _ in range(n)]
        self.loss = torch.full((n,), -1.0, device="cuda")
        ws = torch.empty(self.s.synk_sliced_grad_workspace_bytes(self.dims, self.cd, self.rows),
                         dtype=torch.uint8, device="cuda")
        self.s.synk_sliced_grad(self.dims, self.cd, self.p, self.p_lp, self.x, self.y, self.rows, n_slices,
                                self.s.OP[op], self.grad, self.loss, ws)
        torch.cuda.synchronize()
        return [g.cpu().numpy() for g in self.grad], self.loss.cpu().numpy()

    def update(self):
        c = self.cfg
        self.loss_out = torch.zeros(1, device="cuda")
        self.s.synk_reduce_sgd_update(self.grad, self.p, self.v, c["lr"], c["momentum"], c["weight_decay"],
                                      p_lp=self.p_lp, loss_in=self.loss, loss_out=self.loss_out)
        torch.cuda.synchronize()


def small_cfg(dims, n_data, compute, seed):
    rng = np.random.default_rng(seed)
    return dict(dims=list(dims), compute=compute,
                data=rng.standard_normal((n_data, dims[0])).astype(np.float32),
                labels=rng.integers(0, dims[-1], n_data).astype(np.int32),
                theta=workloads.mlp_init(dims, rng) + (rng.standard_normal(workloads.mlp_param_count(dims)) * 0.05).astype(np.float32),
                lr=0.01, momentum=0.9, weight_decay=0.0)


def worker_refs(cfg, idx, n_workers, bf16):
    """Per worker: oracle gradient of the unsliced call on the share (what
    mean-aggregated slices must equal), the other-relu-derivative variant, the
    columns to skip and the loss."""
    eps = TIE_EPS["bf16" if bf16 else "f32"]
    out = []
    for (a, b) in osplit.share_bounds(len(idx), n_workers):
        X = ogather.gather_rows(cfg["data"], idx[a:b]); y = ogather.gather_rows(cfg["labels"], idx[a:b])
        tr = []
        l, g = omlp.function(cfg["theta"], cfg["dims"], X, y, bf16_points=bf16, trace=tr)
        _, ga = omlp.function(cfg["theta"], cfg["dims"], X, y, bf16_points=bf16, tie_eps=eps, flip_ties=True)
        skip, n_ties = tie_columns(tr, eps)
        out.append(dict(loss=l, grad=g, alt=ga, skip=skip, ties=n_ties))
    return out


@pytest.mark.parametrize("dims,B,N,S,op", [
    ([20, 16, 10], 12, 3, 2, "mean"),
    ([20, 16, 10], 13, 3, 3, "mean"),     # ragged shares and ragged slices
    ([20, 16, 10], 13, 3, 3, "sum"),
    ([20, 16, 10], 2, 3, 2, "mean"),      # a worker with no rows, slices with no rows
    ([13, 7, 5], 9, 2, 2, "mean"),        # nothing 16-byte aligned: element-wise loads
    ([40, 72, 24, 8], 70, 2, 4, "mean"),  # two hidden layers, several 64-wide tiles, ragged tails
    ([33, 10], 17, 2, 2, "sum"),          # no hidden layer
    ([24, 16, 40], 30, 2, 3, "mean"),     # more classes than the fused last-layer kernel takes
    ([24, 12, 10], 30, 2, 3, "mean"),     # hidden width not a multiple of 8: generic last layer
])
def test_sliced_grad_fp32_matches_sliced_oracle(synk, dims, B, N, S, op):
    cfg = small_cfg(dims, 64, "f32", sum(dims) + B)
    idx = np.random.default_rng(B).integers(0, 64, B).astype(np.int32)
    st = Step(synk, cfg)
    st.gather(idx, N)
    grads, losses = st.sliced_grad(S, op)
    ref = omlp.sliced(cfg["theta"], dims, cfg["data"], cfg["labels"], idx, N, S, op)
    assert sum(r["ties"] for r in worker_refs(cfg, idx, N, False)) == 0    # nothing sits on a relu kink
    for w in range(N):
        if st.rows[w] == 0:
            assert np.all(grads[w] == 0.0) and losses[w] == 0.0
            continue
        assert rel_err(grads[w], ref["worker_grads"][w]) < TOL_F32, w
        assert abs(losses[w] - ref["worker_losses"][w]) < TOL_F32 * abs(ref["worker_losses"][w])


@pytest.mark.parametrize("dims,B,N,S", [
    ([64, 48, 32, 10], 50, 3, 2),
    ([256, 136, 10], 300, 2, 4),      # several tiles in every direction, ragged
    ([64, 48, 40], 50, 3, 2),         # wide last layer: generic softmax path
])
def test_sliced_grad_bf16_small(synk, dims, B, N, S):
    cfg = small_cfg(dims, 400, "bf16", sum(dims))
    idx = np.random.default_rng(B).integers(0, 400, B).astype(np.int32)
    st = Step(synk, cfg)
    st.gather(idx, N)
    grads, losses = st.sliced_grad(S, "mean")
    for w, r in enumerate(worker_refs(cfg, idx, N, True)):
        e = rel_err_either_tie(grads[w], r["grad"], r["alt"], dims, r["skip"])
        assert e < TOL_BF16, (w, e)
        assert abs(losses[w] - r["loss"]) < TOL_BF16 * abs(r["loss"])


@pytest.mark.parametrize("compute", ["f32", "bf16"])
@pytest.mark.parametrize("dims,rows_per_worker,N", [
    ([2048, 1024, 10], 16, 4),        # dW has 512 tiles of 128 x 128: the large-tile path
    ([128, 1024, 1024, 10], 1024, 8), # forward and dX have 512 large tiles
])
def test_large_tile_paths(synk, compute, dims, rows_per_worker, N):
    bf16 = compute == "bf16"
    B = rows_per_worker * N
    cfg = small_cfg(dims, B, compute, 7)
    cfg["data"] = np.abs(cfg["data"])
    idx = np.random.default_rng(1).permutation(B).astype(np.int32)
    st = Step(synk, cfg)
    st.gather(idx, N)
    grads, losses = st.sliced_grad(2, "mean")
    tol = TOL_BF16 if bf16 else TOL_F32
    for w, r in enumerate(worker_refs(cfg, idx, N, bf16)):
        e = rel_err_either_tie(grads[w], r["grad"], r["alt"], dims, r["skip"])
        assert e < tol, (w, e)
        assert abs(losses[w] - r["loss"]) < tol * abs(r["loss"])


def test_largest_tile_path_bf16(synk):
    """32,768 rows: the forward and dX products of the 1024-wide layers take the 256 x 128 tiling."""
    dims, rows_per_worker, N = [64, 1024, 1024, 10], 4096, 8
    B = rows_per_worker * N
    cfg = small_cfg(dims, B, "bf16", 9)
    cfg["data"] = np.abs(cfg["data"])
    idx = np.random.default_rng(2).permutation(B).astype(np.int32)
    st = Step(synk, cfg)
    st.gather(idx, N)
    grads, losses = st.sliced_grad(2, "mean")
    for w, r in enumerate(worker_refs(cfg, idx, N, True)):
        e = rel_err_either_tie(grads[w], r["grad"], r["alt"], dims, r["skip"])
        assert e < TOL_BF16, (w, e)
        assert abs(losses[w] - r["loss"]) < TOL_BF16 * abs(r["loss"])


@pytest.mark.parametrize("compute,rows", [
    ("bf16", [128, 0, 256, 128, 128, 0, 256, 128]),     # whole rounds of four 32-row k-tiles, two empty workers
    ("f32", [64, 192, 0, 64, 128, 64, 64, 64]),         # fp32: rounds of four 16-row k-tiles
    ("bf16", [128, 96, 128, 128, 128, 128, 128, 128]),  # one worker breaks the rounds: the per-tile kernel runs
])
def test_weight_gradient_with_unequal_worker_rows(synk, compute, rows):
    """dW of the 1024 x 1024 layer has 512 large tiles: the tile-walking kernel when every worker's
    row count allows it, with workers of different sizes (and none) in one launch."""
    bf16 = compute == "bf16"
    dims = [128, 1024, 1024, 10]
    B = sum(rows)
    cfg = small_cfg(dims, B, compute, 11)
    cfg["data"] = np.abs(cfg["data"])
    st = Step(synk, cfg)
    xdt = torch.bfloat16 if bf16 else torch.float32
    bounds = np.concatenate([[0], np.cumsum(rows)])
    st.rows = list(rows)
    st.x = [dev(cfg["data"][a:b]).to(xdt) if b > a else torch.zeros((0, dims[0]), dtype=xdt, device="cuda")
            for a, b in zip(bounds[:-1], bounds[1:])]
    st.y = [dev(cfg["labels"][a:b]) if b > a else torch.zeros(0, dtype=torch.int32, device="cuda")
            for a, b in zip(bounds[:-1], bounds[1:])]
    grads, losses = st.sliced_grad(2, "mean")
    eps = TIE_EPS[compute]
    tol = TOL_BF16 if bf16 else TOL_F32
    for w, (a, b) in enumerate(zip(bounds[:-1], bounds[1:])):
        if b == a:
            assert not grads[w].any()                 # a worker without rows contributes the zero gradient
            continue
        X, y = cfg["data"][a:b], cfg["labels"][a:b]
        tr = []
        l, gref = omlp.function(cfg["theta"], dims, X, y, bf16_points=bf16, trace=tr)
        _, galt = omlp.function(cfg["theta"], dims, X, y, bf16_points=bf16, tie_eps=eps, flip_ties=True)
        skip, _ = tie_columns(tr, eps)
        e = rel_err_either_tie(grads[w], gref, galt, dims, skip)
        assert e < tol, (w, e)
        assert abs(losses[w] - l) < tol * abs(l)


def test_slice_count_does_not_change_mean_aggregated_result(synk):
    cfg = small_cfg([40, 32, 10], 100, "f32", 1)
    idx = np.random.default_rng(2).integers(0, 100, 48).astype(np.int32)
    st = Step(synk, cfg)
    st.gather(idx, 2)
    g1, l1 = st.sliced_grad(1, "mean")
    g5, l5 = st.sliced_grad(5, "mean")
    for w in range(2):
        assert rel_err(g5[w], g1[w]) < 1e-6 and abs(l5[w] - l1[w]) < 1e-6 * abs(l1[w])


def full_step_check(synk, cfg, tol, bf16):
    dims, idx, N, S = cfg["dims"], cfg["idx"], cfg["n_workers"], cfg["n_slices"]
    st = Step(synk, cfg)
    st.gather(idx, N)
    grads, losses = st.sliced_grad(S, "mean")
    refs = worker_refs(cfg, idx, N, bf16)
    worst, report = 0.0, {}
    for w, r in enumerate(refs):
        e = rel_err_either_tie(grads[w], r["grad"], r["alt"], dims, r["skip"], report)
        worst = max(worst, e)
        assert e < tol, ("worker grad", w, e)
        assert abs(losses[w] - r["loss"]) < tol * abs(r["loss"])
    print("columns with >= 2 near-zero pre-activations (held to %gx the tolerance): %d, their worst error %.2e"
          % (5.0, report.get("loose_columns", 0), report.get("loose_worst", 0.0)))
    if bf16:
        # The second distance: against the all-float64 oracle (no bf16 rounding anywhere).  This one is a
        # property of feeding the contractions bf16 values (relu decisions of near-zero units change), not
        # of the kernels; the band is the oracle's own bf16-mode-to-float64 distance at this shape (pinned on
        # the CPU in tests/test_oracle_pins.py) plus the tolerance.
        worst64, fro64 = 0.0, 0.0
        for w, (a, b) in enumerate(osplit.share_bounds(len(idx), N)):
            X = ogather.gather_rows(cfg["data"], idx[a:b]); y = ogather.gather_rows(cfg["labels"], idx[a:b])
            _, g64 = omlp.function(cfg["theta"], dims, X, y)
            fro64 = max(fro64, float(np.linalg.norm(grads[w] - g64) / np.linalg.norm(g64)))
            for (name, g), (_, r) in zip(mlp_tensors(grads[w].astype(np.float64), dims), mlp_tensors(g64, dims)):
                worst64 = max(worst64, rel_err(g, r))
        print("against the float64 oracle: worst per-tensor error %.2e, worst whole-gradient (Frobenius) %.2e; "
              "against the oracle rounded at the bf16 points: %.2e" % (worst64, fro64, worst))
        assert worst64 < BF16_VS_F64_MAX + tol and fro64 < BF16_VS_F64_FRO + tol
    st.update()
    v0 = np.zeros_like(cfg["theta"])
    rp, rv, rG, rl = oupdate.reduce_and_update(cfg["theta"], v0, [r["grad"] for r in refs], cfg["lr"],
                                               cfg["momentum"], cfg["weight_decay"], None, [r["loss"] for r in refs])
    ap, av, _, _ = oupdate.reduce_and_update(cfg["theta"], v0, [r["alt"] for r in refs], cfg["lr"],
                                             cfg["momentum"], cfg["weight_decay"])
    skip = {}
    for r in refs:
        for k, cols in r["skip"].items():
            skip.setdefault(k, set()).update(cols)
    assert rel_err_either_tie(st.p.cpu().numpy(), rp, ap, dims, skip) < tol
    # a tie in one worker moves only that worker's share of v: the bound is per tensor as before
    assert rel_err_either_tie(st.v.cpu().numpy(), rv, av, dims, skip) < tol
    assert abs(st.loss_out.item() - rl) < tol * abs(rl)
    if bf16:
        want = ogather.round_to_bf16(st.p.cpu().numpy())
        assert np.array_equal(st.p_lp.float().cpu().numpy().view(np.uint32), want.view(np.uint32))
    return worst, sum(r["ties"] for r in refs)


def test_full_step_config1_fp32(synk):
    cfg = workloads.config1()
    worst, ties = full_step_check(synk, cfg, TOL_F32, False)
    print("config1 worst worker-gradient error %.2e, near-zero pre-activations %d" % (worst, ties))


def test_full_step_config2_bf16_reduced(synk):
    cfg = workloads.config2(n_data=2000, batch=96, dims=(512, 256, 128, 10), n_workers=4, n_slices=3)
    worst, ties = full_step_check(synk, cfg, TOL_BF16, True)
    print("config2 (reduced) worst error %.2e, ties %d" % (worst, ties))


def test_full_step_config2_bf16_full_size(synk):
    cfg = workloads.config2(n_data=8192)       # full model, batch, workers and slices; fewer dataset rows
    worst, ties = full_step_check(synk, cfg, TOL_BF16, True)
    print("config2 worst worker-gradient error %.2e, near-zero pre-activations %d" % (worst, ties))


def test_two_steps_feed_the_updated_parameters_forward(synk):
    cfg = workloads.config1(n_data=1024, batch=128)
    st = Step(synk, cfg)
    theta, v = cfg["theta"].astype(np.float64), np.zeros(len(cfg["theta"]))
    rng = np.random.default_rng(3)
    for step in range(2):
        idx = rng.permutation(1024)[:128].astype(np.int32)
        st.gather(idx, 2)
        st.sliced_grad(4, "mean")
        st.update()
        r = omlp.sliced(theta, cfg["dims"], cfg["data"], cfg["labels"], idx, 2, 4)
        theta, v, _, _ = oupdate.reduce_and_update(theta, v, r["worker_grads"], 0.01, 0.9)
    assert rel_err(st.p.cpu().numpy(), theta) < TOL_F32
    assert rel_err(st.v.cpu().numpy(), v) < 10 * TOL_F32   # second-step v carries first-step rounding of p


def test_sliced_grad_is_bit_reproducible(synk):
    cfg = workloads.config2(n_data=1000, batch=128, dims=(256, 128, 64, 10), n_workers=4, n_slices=2)
    st = Step(synk, cfg)
    st.gather(cfg["idx"], 4)
    g1, l1 = st.sliced_grad(2, "mean")
    g2, l2 = st.sliced_grad(2, "mean")
    assert all(np.array_equal(a, b) for a, b in zip(g1, g2)) and np.array_equal(l1, l2)


def test_step_captured_in_a_graph_replays_like_eager_steps(synk):
    """The three calls of a step launch kernels only (no allocation, no memset, no
    synchronisation), so a caller may capture them into a graph.  Every replay, with eager work
    and synchronisations in between, must leave exactly what the eager step leaves."""
    dims = [64, 48, 10]
    cfg = small_cfg(dims, 200, "bf16", 21)
    idx = np.random.default_rng(3).integers(0, 200, 96).astype(np.int32)
    N, S = 4, 2

    def make():
        st = Step(synk, cfg)
        st.rows = lib_share_sizes(synk, len(idx), N)
        st.x = [torch.zeros((n, dims[0]), dtype=torch.bfloat16, device="cuda") for n in st.rows]
        st.y = [torch.zeros(n, dtype=torch.int32, device="cuda") for n in st.rows]
        st.grad = [torch.zeros(st.P, device="cuda") for _ in st.rows]
        st.loss = torch.zeros(N, device="cuda")
        st.loss_out = torch.zeros(1, device="cuda")
        st.ws = torch.empty(synk.synk_sliced_grad_workspace_bytes(dims, st.cd, st.rows), dtype=torch.uint8,
                            device="cuda")
        st.idx = dev(idx)
        return st

    def step(st, stream=None):
        c = st.cfg
        synk.synk_gather_rows(st.data, st.idx, st.x, labels=st.labels, dst_labels=st.y, stream=stream)
        synk.synk_sliced_grad(dims, st.cd, st.p, st.p_lp, st.x, st.y, st.rows, S, synk.SYNK_MEAN, st.grad, st.loss,
                              st.ws, stream=stream)
        synk.synk_reduce_sgd_update(st.grad, st.p, st.v, c["lr"], c["momentum"], c["weight_decay"], p_lp=st.p_lp,
                                    loss_in=st.loss, loss_out=st.loss_out, stream=stream)

    eager, graphed = make(), make()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step(graphed, stream=side.cuda_stream)
    torch.cuda.synchronize()
    # capture records, it does not run: the graphed state is still the initial one
    assert torch.equal(graphed.p, eager.p)
    scratch = torch.zeros(1 << 16, device="cuda")
    for it in range(4):
        step(eager)
        g.replay()
        scratch.add_(1.0)                    # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(graphed.p, eager.p), it
        assert torch.equal(graphed.v, eager.v), it
        assert torch.equal(graphed.p_lp, eager.p_lp), it
        assert torch.equal(graphed.loss_out, eager.loss_out), it


def test_profile_hook_selects_kernels_of_the_sliced_gradient(synk):
    """An event pair handed in for one kernel of synk_sliced_grad is attached to that launch and to no
    other: it is consumed when the call launches the kernel and stays pending when it does not."""
    cfg = workloads.config2(n_data=1000, batch=256, dims=(128, 64, 64, 10), n_workers=2, n_slices=2)
    st = Step(synk, cfg)
    st.gather(cfg["idx"], 2)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(); b.record()
    torch.cuda.synchronize()
    ref, _ = st.sliced_grad(2, "mean")
    for kernel, launched in [(synk.SYNK_KERNEL_MAIN, True), (synk.SYNK_KERNEL_MLP_FORWARD(2), True),
                             (synk.SYNK_KERNEL_MLP_HEAD, True), (synk.SYNK_KERNEL_MLP_DW(1), True),
                             (synk.SYNK_KERNEL_MLP_FORWARD(3), False), (synk.SYNK_KERNEL_MLP_DX(7), False)]:
        synk.synk_profile_next_launch_of(kernel, a, b)
        got, _ = st.sliced_grad(2, "mean")
        assert synk.synk_profile_pending() == (not launched), kernel
        synk.synk_profile_next_launch_of(kernel, None, None)
        assert not synk.synk_profile_pending()
        if launched:
            assert 0.0005 < a.elapsed_time(b) < 1.0, kernel
        assert all(np.array_equal(x, y) for x, y in zip(got, ref))       # a timed launch computes the same


# ------------------------------------------------------------- input indexing folded into the call
def _indexed_against_gather_then_grad(synk, dims, bf16, n_data, B, N, S, seed, bad_index=False):
    """synk_sliced_grad_indexed == synk_gather_rows + synk_sliced_grad, bit for bit."""
    rng = np.random.default_rng(seed)
    cd = synk.SYNK_BF16 if bf16 else synk.SYNK_F32
    data = torch.from_numpy(rng.standard_normal((n_data, dims[0])).astype(np.float32)).cuda()
    if bf16:
        data = data.bfloat16()
    labels = dev(rng.integers(0, dims[-1], n_data).astype(np.int32))
    theta = workloads.mlp_init(dims, rng) + (rng.standard_normal(workloads.mlp_param_count(dims)) * 0.05).astype(np.float32)
    idx_h = rng.integers(0, n_data, B).astype(np.int32)
    idx_ref = idx_h.copy()
    if bad_index:                     # the fused kernels read row 0 for an index outside the data
        idx_h[3], idx_h[B - 2] = n_data + 5, -7
        idx_ref[3], idx_ref[B - 2] = 0, 0
    P = synk.synk_mlp_param_count(dims)
    p = dev(theta)
    p_lp = torch.zeros(P, dtype=torch.bfloat16, device="cuda") if bf16 else None
    if bf16:
        synk.synk_cast_bf16(p, p_lp)
    rows = lib_share_sizes(synk, B, N)
    x = [torch.zeros((n, dims[0]), dtype=data.dtype, device="cuda") for n in rows]
    y = [torch.zeros(n, dtype=torch.int32, device="cuda") for n in rows]
    synk.synk_gather_rows(data, dev(idx_ref), x, labels=labels, dst_labels=y)
    ga = [torch.full((P,), 5.0, device="cuda") for _ in rows]
    la = torch.full((N,), -1.0, device="cuda")
    ws = torch.empty(synk.synk_sliced_grad_workspace_bytes(dims, cd, rows), dtype=torch.uint8, device="cuda")
    synk.synk_sliced_grad(dims, cd, p, p_lp, x, y, rows, S, synk.SYNK_MEAN, ga, la, ws)
    gb = [torch.full((P,), 7.0, device="cuda") for _ in rows]
    lb = torch.full((N,), -2.0, device="cuda")
    wsi = torch.full((synk.synk_sliced_grad_indexed_workspace_bytes(dims, cd, B, N),), 0x5A, dtype=torch.uint8,
                     device="cuda")
    for _ in range(2):                # the second call runs on a workspace the first has used
        synk.synk_sliced_grad_indexed(dims, cd, p, p_lp, data, labels, dev(idx_h), S, synk.SYNK_MEAN, gb, lb, wsi)
    torch.cuda.synchronize()
    for w in range(N):
        assert torch.equal(ga[w], gb[w]), (w, float((ga[w] - gb[w]).abs().max()))
    assert torch.equal(la, lb)
    return theta, data, labels, idx_ref, [g.cpu().numpy() for g in gb]


@pytest.mark.parametrize("dims,bf16,n_data,B,N,S", [
    ([128, 64, 64, 10], True, 900, 512, 8, 4),      # whole 64-row tiles: the whole-tile product reads through the index
    ([192, 128, 10], True, 700, 256, 4, 2),         # two layers
    ([256, 128, 128, 10], True, 3000, 2048, 8, 1),  # 256 rows a worker
    ([100, 64, 10], False, 500, 256, 8, 4),         # fp32, few rows: the small-batch kernel reads through the index
    ([784, 256, 10], False, 4096, 256, 8, 4),       # the tiny configuration's shape
    ([130, 48, 10], False, 300, 61, 5, 3),          # ragged everything
    ([3072, 1024, 1024, 10], True, 4096, 1024, 8, 4),   # the wide configuration as the benchmark launches it
    ([784, 256, 10], False, 4096, 256, 2, 4),           # the tiny configuration as the benchmark launches it
    ([512, 1024, 1024, 10], True, 9000, 8192, 8, 2),    # 128 x 128 tiles read through the index
    ([512, 1024, 1024, 10], True, 40000, 32768, 8, 2),  # 256 x 128 tiles read through the index
    ([128, 64, 64, 10], True, 900, 500, 8, 4),      # shares that are no whole tiles: the call gathers first
    ([96, 64, 10], False, 5000, 4096, 4, 2),        # fp32 with many rows: MFMA product, the call gathers first
])
def test_indexed_call_equals_gather_then_sliced_grad(synk, dims, bf16, n_data, B, N, S):
    _indexed_against_gather_then_grad(synk, dims, bf16, n_data, B, N, S, seed=B + N)


def test_indexed_call_against_the_oracle_and_index_out_of_range(synk):
    dims, n_data, B, N, S = [100, 64, 10], 500, 256, 8, 4
    theta, data, labels, idx, grads = _indexed_against_gather_then_grad(synk, dims, False, n_data, B, N, S, seed=11)
    ref = omlp.sliced(theta, dims, data.cpu().numpy(), labels.cpu().numpy(), idx, N, S)
    for w in range(N):
        assert rel_err(grads[w], ref["worker_grads"][w]) < TOL_F32, w
    # an index outside the data reads row 0 in the kernels that read through the index: never out of bounds
    _indexed_against_gather_then_grad(synk, dims, False, n_data, B, N, S, seed=12, bad_index=True)
    _indexed_against_gather_then_grad(synk, [128, 64, 64, 10], True, 900, 512, 8, 4, seed=13, bad_index=True)
