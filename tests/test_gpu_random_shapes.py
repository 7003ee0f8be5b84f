"""Seeded random-shape parity cases for the gather, reduce, update, evaluation and MLP kernels:
odd sizes, ragged and empty shares, every alignment path, drawn once from fixed seeds (the cases
are the same on every run).  Each compares the HIP path, through the C ABI, with the CPU oracle."""
import numpy as np
import pytest
import torch

import workloads
from helpers import TOL_BF16, TOL_F32, lib_share_sizes, rel_err, rel_err_either_tie, tie_columns
from oracle import evalops, gather as ogather, mlp as omlp, reduce as oreduce, split as osplit, update as oupdate

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def synk():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1710_04162_amd import binding
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _gather_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        row = int(rng.choice([1, 3, 4, 7, 8, 12, 16, 33, 64, 100, 257, 1024, 3000, 4099]))
        out.append((int(rng.integers(1, 200)), row, int(rng.integers(0, 120)), int(rng.integers(1, 17)),
                    str(rng.choice(["f32", "u8", "i32", "bf16out"]))))
    return out


@pytest.mark.parametrize("n_data,row,batch,n_workers,kind", _gather_cases(24, 171004162))
def test_gather_random_shapes_bit_exact(synk, n_data, row, batch, n_workers, kind):
    rng = np.random.default_rng(n_data * 1000 + row)
    np_dt = {"f32": np.float32, "u8": np.uint8, "i32": np.int32, "bf16out": np.float32}[kind]
    data = (rng.standard_normal((n_data, row)) * 50).astype(np_dt)
    labels = rng.integers(0, 1000, n_data).astype(np.int32)
    idx = rng.integers(0, n_data, batch).astype(np.int32)
    sizes = lib_share_sizes(synk, batch, n_workers)
    assert sizes == osplit.share_sizes(batch, n_workers)
    out_dt = torch.bfloat16 if kind == "bf16out" else torch.from_numpy(np.zeros(1, np_dt)).dtype
    dst = [torch.zeros((max(n, 1), row), dtype=out_dt, device="cuda")[:n] for n in sizes]
    dl = [torch.full((max(n, 1),), -5, dtype=torch.int32, device="cuda")[:n] for n in sizes]
    synk.synk_gather_rows(dev(data), dev(idx), dst, labels=dev(labels), dst_labels=dl)
    torch.cuda.synchronize()
    ref = ogather.gather_shares(data, idx, n_workers)
    refl = ogather.gather_shares(labels, idx, n_workers)
    for w in range(n_workers):
        if kind == "bf16out":
            want = ogather.round_to_bf16(ref[w])
            assert np.array_equal(dst[w].float().cpu().numpy().view(np.uint32), want.view(np.uint32)), w
        else:
            assert np.array_equal(dst[w].cpu().numpy(), ref[w]), w
        assert np.array_equal(dl[w].cpu().numpy(), refl[w]), w


def _reduce_cases(n, seed):
    rng = np.random.default_rng(seed)
    return [(int(rng.integers(1, 17)), int(rng.choice([1, 2, 3, 5, 127, 128, 1023, 4097, 65537, 200003])),
             str(rng.choice(["sum", "mean", "max", "min", "prod"])), int(rng.integers(0, 4))) for _ in range(n)]


@pytest.mark.parametrize("n,length,op,offset", _reduce_cases(24, 171004163))
def test_reduce_and_all_reduce_random_shapes(synk, n, length, op, offset):
    """offset: the buffers start that many floats into their allocation (the 4-byte paths when not 0)."""
    rng = np.random.default_rng(n * 100000 + length)
    host = [rng.uniform(0.5, 2.0, length).astype(np.float32) for _ in range(n)]
    bufs = []
    for h in host:
        t = torch.zeros(length + offset, device="cuda")
        t[offset:] = dev(h)
        bufs.append(t[offset:])
    out = torch.zeros(length + offset, device="cuda")[offset:]
    synk.synk_reduce_buffers(bufs, synk.OP[op], out)
    ref = oreduce.reduce_buffers(host, op)
    if op in ("max", "min"):
        assert np.array_equal(out.cpu().numpy(), ref.astype(np.float32))
    else:
        assert rel_err(out.cpu().numpy(), ref) < TOL_F32
    synk.synk_all_reduce(bufs, op)
    for b in bufs:
        assert torch.equal(b, bufs[0])
    got = bufs[n - 1].cpu().numpy()
    if op in ("max", "min"):
        assert np.array_equal(got, ref.astype(np.float32))
    else:
        assert rel_err(got, ref) < TOL_F32


def _update_cases(n, seed):
    rng = np.random.default_rng(seed)
    return [(str(rng.choice(["momentum", "nesterov", "rmsprop", "adam"])), int(rng.integers(1, 13)),
             int(rng.choice([4, 8, 1000, 1028, 4100, 70004, 262148]))) for _ in range(n)]


HYPER = dict(momentum=dict(lr=0.05, momentum=0.9, weight_decay=1e-3), nesterov=dict(lr=0.05, momentum=0.8, weight_decay=1e-3),
             rmsprop=dict(lr=0.01, rho=0.9, eps=1e-6, weight_decay=1e-3),
             adam=dict(lr=0.01, beta1=0.9, beta2=0.99, eps=1e-8, weight_decay=1e-3))


@pytest.mark.parametrize("rule,n,length", _update_cases(16, 171004164))
def test_fused_reduce_update_random_shapes(synk, rule, n, length):
    rng = np.random.default_rng(n * 7 + length)
    p0 = rng.standard_normal(length).astype(np.float32)
    grads = [(rng.standard_normal(length) * 0.1).astype(np.float32) for _ in range(n)]
    losses = rng.random(n).astype(np.float32)
    p, s1, s2 = dev(p0), torch.full((length,), 1e-3, device="cuda"), torch.full((length,), 2e-4, device="cuda")
    lo = torch.zeros(1, device="cuda")
    p_lp = torch.zeros(length, dtype=torch.bfloat16, device="cuda")
    h = HYPER[rule]
    synk.synk_reduce_update(rule, [dev(g) for g in grads], p, s1, s2 if rule == "adam" else None, step=3, p_lp=p_lp,
                            loss_in=dev(losses), loss_out=lo, **h)
    G = oreduce.reduce_buffers(grads, "mean")
    rp, q1, q2 = oupdate.apply_rule(rule, p0, np.full(length, 1e-3), np.full(length, 2e-4), G, dict(h, t=3))
    assert rel_err(p.cpu().numpy(), rp) < TOL_F32 and rel_err(s1.cpu().numpy(), q1) < TOL_F32
    if rule == "adam":
        assert rel_err(s2.cpu().numpy(), q2) < TOL_F32
    assert abs(lo.item() - float(np.mean(losses.astype(np.float64)))) < TOL_F32
    want = ogather.round_to_bf16(p.cpu().numpy())
    assert np.array_equal(p_lp.float().cpu().numpy().view(np.uint32), want.view(np.uint32))


def _eval_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        classes = int(rng.choice([1, 2, 3, 10, 37, 64, 100, 255, 900, 1000, 1024, 1500, 4096]))
        rows = int(rng.integers(1, 700))
        out.append((rows, classes, int(rng.integers(1, 2 * rows + 2))))
    return out


@pytest.mark.parametrize("rows,classes,n_slices", _eval_cases(20, 171004165))
def test_sliced_eval_random_shapes(synk, rows, classes, n_slices):
    rng = np.random.default_rng(rows * 31 + classes)
    logits = (rng.standard_normal((rows, classes)) * 2.0).astype(np.float32)
    labels = rng.integers(0, classes, rows).astype(np.int32)
    ws = torch.empty(synk.synk_sliced_eval_workspace_bytes(rows, classes, n_slices), dtype=torch.uint8, device="cuda")
    o = dict(ce_sum=torch.zeros(1, device="cuda"), counts=torch.full((classes,), -1, dtype=torch.int32, device="cuda"),
             max_logit=torch.zeros(1, device="cuda"), min_logit=torch.zeros(1, device="cuda"),
             n_correct=torch.zeros(1, dtype=torch.int32, device="cuda"),
             argmax=torch.full((rows,), -1, dtype=torch.int32, device="cuda"))
    synk.synk_sliced_eval(dev(logits), dev(labels), n_slices, o["ce_sum"], o["counts"], o["max_logit"], o["min_logit"],
                          o["n_correct"], o["argmax"], ws)
    got = {k: v.cpu().numpy() for k, v in o.items()}
    ref = evalops.sliced(logits, labels, n_slices)
    for k in ("counts", "n_correct", "argmax"):
        assert np.array_equal(got[k].astype(np.int64), np.asarray(ref[k]).astype(np.int64).reshape(got[k].shape)), k
    assert got["max_logit"][0] == np.float32(ref["max_logit"][0]) and got["min_logit"][0] == np.float32(ref["min_logit"][0])
    assert abs(got["ce_sum"][0] - ref["ce_sum"][0]) <= TOL_F32 * max(abs(ref["ce_sum"][0]), 1.0)


def _mlp_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        L = int(rng.integers(1, 4))
        dims = [int(rng.choice([5, 8, 13, 24, 64, 72, 128, 200]))] + \
               [int(rng.choice([7, 8, 16, 40, 64, 72, 128, 136])) for _ in range(L - 1)] + [int(rng.choice([2, 5, 10, 16, 17, 40]))]
        out.append((dims, int(rng.integers(1, 150)), int(rng.integers(1, 6)), int(rng.integers(1, 5)),
                    str(rng.choice(["mean", "sum"])), bool(rng.integers(0, 2))))
    # whole-tile shapes, so that the direct-to-LDS product kernels take part: rows a multiple of 64 per worker
    out += [([128, 64, 128, 10], 256, 2, 3, "mean", True), ([64, 192, 64, 10], 384, 3, 2, "sum", True),
            ([192, 128, 128, 128, 16], 128, 2, 2, "mean", True)]
    return out


@pytest.mark.parametrize("dims,B,N,S,op,bf16", _mlp_cases(20, 171004166))
def test_sliced_grad_random_shapes(synk, dims, B, N, S, op, bf16):
    rng = np.random.default_rng(sum(dims) * 13 + B)
    n_data = 64
    data = rng.standard_normal((n_data, dims[0])).astype(np.float32)
    labels = rng.integers(0, dims[-1], n_data).astype(np.int32)
    theta = workloads.mlp_init(dims, rng) + (rng.standard_normal(workloads.mlp_param_count(dims)) * 0.05).astype(np.float32)
    idx = rng.integers(0, n_data, B).astype(np.int32)
    cd = synk.SYNK_BF16 if bf16 else synk.SYNK_F32
    P = synk.synk_mlp_param_count(dims)
    rows = lib_share_sizes(synk, B, N)
    xdt = torch.bfloat16 if bf16 else torch.float32
    x = [torch.zeros((n, dims[0]), dtype=xdt, device="cuda") for n in rows]
    y = [torch.zeros(n, dtype=torch.int32, device="cuda") for n in rows]
    synk.synk_gather_rows(dev(data), dev(idx), x, labels=dev(labels), dst_labels=y)
    p = dev(theta)
    p_lp = None
    if bf16:
        p_lp = torch.zeros(P, dtype=torch.bfloat16, device="cuda")
        synk.synk_cast_bf16(p, p_lp)
    grad = [torch.full((P,), 123.0, device="cuda") for _ in rows]
    loss = torch.full((N,), -1.0, device="cuda")
    ws = torch.empty(synk.synk_sliced_grad_workspace_bytes(dims, cd, rows), dtype=torch.uint8, device="cuda")
    synk.synk_sliced_grad(dims, cd, p, p_lp, x, y, rows, S, synk.OP[op], grad, loss, ws)
    torch.cuda.synchronize()
    tol = TOL_BF16 if bf16 else TOL_F32
    eps = 1e-3 if bf16 else 2e-6
    for w, slices in enumerate(osplit.worker_slice_bounds(B, N, S)):
        g = grad[w].cpu().numpy()
        if rows[w] == 0:
            assert not g.any() and loss[w].item() == 0.0
            continue
        # the worker's result = aggregation of its slices' results (each slice one call of the function)
        gs, ga, ls, ns, skip = [], [], [], [], {}
        for (a, b) in slices:
            X, yy = ogather.gather_rows(data, idx[a:b]), ogather.gather_rows(labels, idx[a:b])
            tr = []
            l_s, g_s = omlp.function(theta, dims, X, yy, bf16_points=bf16, trace=tr)
            _, g_a = omlp.function(theta, dims, X, yy, bf16_points=bf16, tie_eps=eps, flip_ties=True)
            sk, _ = tie_columns(tr, eps) if b > a else ({}, 0)
            for k, cols in sk.items():
                skip.setdefault(k, set()).update(cols)
            gs.append(g_s); ga.append(g_a); ls.append(l_s); ns.append(b - a)
        ref = omlp.aggregate_slices(gs, ns, op)
        alt = omlp.aggregate_slices(ga, ns, op)
        rl = omlp.aggregate_slices(ls, ns, op)
        assert rel_err_either_tie(g, ref, alt, dims, skip) < tol, (w, dims)
        assert abs(loss[w].item() - rl) < tol * max(abs(rl), 1e-6)


# ------------------------------------------------------------- maximum worker count
def test_maximum_worker_count_through_the_whole_step(synk):
    """SYNK_MAX_WORKERS = 64 workers: gather, sliced gradient, N-way reduce fused with the update, all-reduce."""
    N, S, B = synk.SYNK_MAX_WORKERS, 2, 200               # shares of 4 and 3 rows
    dims = [24, 16, 10]
    rng = np.random.default_rng(64)
    data = rng.standard_normal((300, dims[0])).astype(np.float32)
    labels = rng.integers(0, dims[-1], 300).astype(np.int32)
    theta = workloads.mlp_init(dims, rng) + (rng.standard_normal(workloads.mlp_param_count(dims)) * 0.05).astype(np.float32)
    idx = rng.integers(0, 300, B).astype(np.int32)
    P = synk.synk_mlp_param_count(dims)
    rows = lib_share_sizes(synk, B, N)
    assert rows == osplit.share_sizes(B, N) and len(rows) == 64
    x = [torch.zeros((n, dims[0]), device="cuda") for n in rows]
    y = [torch.zeros(n, dtype=torch.int32, device="cuda") for n in rows]
    synk.synk_gather_rows(dev(data), dev(idx), x, labels=dev(labels), dst_labels=y)
    p, v = dev(theta), torch.zeros(P, device="cuda")
    grad = [torch.full((P,), 9.0, device="cuda") for _ in rows]
    loss, loss_out = torch.zeros(N, device="cuda"), torch.zeros(1, device="cuda")
    ws = torch.empty(synk.synk_sliced_grad_workspace_bytes(dims, synk.SYNK_F32, rows), dtype=torch.uint8, device="cuda")
    synk.synk_sliced_grad(dims, synk.SYNK_F32, p, None, x, y, rows, S, synk.SYNK_MEAN, grad, loss, ws)
    ref = omlp.sliced(theta, dims, data, labels, idx, N, S)
    for w in range(N):
        assert rel_err(grad[w].cpu().numpy(), ref["worker_grads"][w]) < TOL_F32, w
    synk.synk_reduce_sgd_update(grad, p, v, 0.01, 0.9, 0.0, loss_in=loss, loss_out=loss_out)
    rp, rv, _, rl = oupdate.reduce_and_update(theta, np.zeros(P), ref["worker_grads"], 0.01, 0.9, 0.0, None,
                                              ref["worker_losses"])
    assert rel_err(p.cpu().numpy(), rp) < TOL_F32 and rel_err(v.cpu().numpy(), rv) < TOL_F32
    assert abs(loss_out.item() - rl) < TOL_F32 * abs(rl)
    synk.synk_all_reduce(grad, "sum")
    want = oreduce.reduce_buffers([g for g in ref["worker_grads"]], "sum")
    assert rel_err(grad[63].cpu().numpy(), want) < TOL_F32 and all(torch.equal(g, grad[0]) for g in grad[1:])
    with pytest.raises(synk.SynkError):                   # one more than the maximum is refused, nothing is launched
        synk.synk_reduce_buffers(grad + [grad[0]], synk.SYNK_SUM, torch.zeros(P, device="cuda"))
