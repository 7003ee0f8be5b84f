"""GPU parity of the data-movement and streaming kernels (gather, reduce,
update, six-output evaluation) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import workloads
from helpers import TOL_F32, lib_share_bounds, lib_share_sizes, rel_err
from oracle import collectives as ocoll, evalops, gather as ogather, reduce as oreduce, split as osplit, update as oupdate

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def synk():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1710_04162_amd import binding
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def share_sizes(n, parts):
    """Buffer sizes of the HIP leg: the library's own split rule.  The oracle's split is used on
    the checker side only (gather_shares and the reference bounds)."""
    from paper_1710_04162_amd import binding
    return lib_share_sizes(binding, n, parts)


# ------------------------------------------------------------------ gather
@pytest.mark.parametrize("n_data,row,batch,n_workers,dtype", [
    (300, 784, 256, 2, np.float32),      # config-1 rows (16-byte path)
    (64, 3072, 100, 8, np.float32),      # config-2 rows, ragged shares (100 = 8*12+4)
    (50, 7, 33, 4, np.float32),          # 28-byte rows: 4-byte path
    (40, 13, 9, 16, np.uint8),           # odd byte rows, more workers than some shares
    (20, 5000, 8, 3, np.int32),          # several chunks per row
    (10, 16, 0, 2, np.float32),          # empty index list
])
def test_gather_copy_bit_exact(synk, n_data, row, batch, n_workers, dtype):
    rng = np.random.default_rng(n_data * 7 + row)
    data = (rng.standard_normal((n_data, row)) * 100).astype(dtype)
    labels = rng.integers(0, 1000, n_data).astype(np.int32)
    idx = rng.integers(0, n_data, batch).astype(np.int32)        # duplicates allowed
    sizes = share_sizes(batch, n_workers)
    tdt = torch.from_numpy(np.zeros(1, dtype)).dtype
    dst = [torch.full((max(n, 1), row), 77, dtype=tdt, device="cuda")[:n] for n in sizes]
    dl = [torch.full((max(n, 1),), -5, dtype=torch.int32, device="cuda")[:n] for n in sizes]
    synk.synk_gather_rows(dev(data), dev(idx), dst, labels=dev(labels), dst_labels=dl)
    torch.cuda.synchronize()
    ref = ogather.gather_shares(data, idx, n_workers)
    refl = ogather.gather_shares(labels, idx, n_workers)
    for w in range(n_workers):
        assert np.array_equal(dst[w].cpu().numpy(), ref[w]), w
        assert np.array_equal(dl[w].cpu().numpy(), refl[w]), w


def test_gather_identity_and_permutation(synk):
    rng = np.random.default_rng(5)
    data = rng.standard_normal((128, 96)).astype(np.float32)
    out = [torch.empty((128, 96), device="cuda")]
    synk.synk_gather_rows(dev(data), dev(np.arange(128, dtype=np.int32)), out)
    assert np.array_equal(out[0].cpu().numpy(), data)
    perm = rng.permutation(128).astype(np.int32)
    synk.synk_gather_rows(dev(data), dev(perm), out)
    assert np.array_equal(out[0].cpu().numpy(), data[perm])


def test_probe_of_mfmas_beside_other_instructions_runs(synk):
    """The timing probe (nothing of the method): every variant launches, reports its flops and leaves
    its buffer alone."""
    buf = torch.zeros(64, device="cuda")
    for pid in ([synk.SYNK_PROBE_MFMA_BESIDE_VALU + n for n in (0, 1, 2, 4, 6, 8, 12)] +
                [synk.SYNK_PROBE_MFMA_BESIDE_LDS + n for n in (1, 2, 4)]):
        work = synk.synk_probe_launch(pid, buf, 50)
        assert work == 256 * 4 * 50 * 2 * 32768.0
    torch.cuda.synchronize()
    assert float(buf.abs().sum()) == 0.0


def test_bf16_rounding_over_the_whole_finite_range(synk):
    """The kernels round with the part's conversion instruction: nearest-even for every finite float32,
    denormals and the overflow to infinity included (random bit patterns of every exponent, and the
    edge values), against the oracle's bit arithmetic."""
    rng = np.random.default_rng(950)
    bits = rng.integers(0, 1 << 32, 64 * 4096, dtype=np.uint64).astype(np.uint32)
    bits = bits[(bits & 0x7F800000) != 0x7F800000]                     # finite only
    edge = np.array([0x00000000, 0x80000000, 0x00000001, 0x80000001, 0x00008000, 0x00018000, 0x00007FFF,
                     0x007FFFFF, 0x00800000, 0x3F808000, 0x3F818000, 0xBF808000, 0xBF818000, 0x3F807FFF,
                     0x3F808001, 0x7F7FFFFF, 0xFF7FFFFF, 0x7F7F7FFF, 0x7F7F8000, 0x7F800000, 0xFF800000],
                    dtype=np.uint32)
    bits = np.concatenate([edge, bits])
    n = len(bits) // 64 * 64
    data = bits[:n].view(np.float32).reshape(-1, 64)
    idx = np.arange(data.shape[0], dtype=np.int32)
    dst = [torch.zeros(data.shape, dtype=torch.bfloat16, device="cuda")]
    synk.synk_gather_rows(dev(data), dev(idx), dst)
    got = dst[0].view(torch.int16).cpu().numpy().view(np.uint16)
    with np.errstate(over="ignore"):
        want = (ogather.round_to_bf16(data).view(np.uint32) >> 16).astype(np.uint16)
    assert np.array_equal(got, want), np.flatnonzero(got.ravel() != want.ravel())[:8]


@pytest.mark.parametrize("row,n_workers", [(3072, 8), (10, 3)])
def test_gather_to_bf16_bit_exact(synk, row, n_workers):
    rng = np.random.default_rng(row)
    data = rng.random((77, row), dtype=np.float32)
    data[0, :4] = [1.00390625, 1.01171875, 0.0, 3.0e38]      # ties to even, both directions
    idx = rng.integers(0, 77, 50).astype(np.int32)
    idx[0] = 0
    sizes = share_sizes(50, n_workers)
    dst = [torch.zeros((n, row), dtype=torch.bfloat16, device="cuda") for n in sizes]
    synk.synk_gather_rows(dev(data), dev(idx), dst)
    ref = [ogather.round_to_bf16(r) for r in ogather.gather_shares(data, idx, n_workers)]
    for w in range(n_workers):
        got = dst[w].float().cpu().numpy()
        assert np.array_equal(got.view(np.uint32), ref[w].view(np.uint32)), w


@pytest.mark.parametrize("chw,batch,n_workers", [((3, 224, 224), 16, 8), ((3, 5, 7), 10, 4), ((1, 8, 8), 5, 2)])
def test_gather_u8_normalise_bit_exact(synk, chw, batch, n_workers):
    c = workloads.config4(n_data=24, batch=batch, chw=chw, n_workers=n_workers)
    lut = torch.empty(chw[0] * 256, device="cuda")
    synk.synk_build_norm_lut(c["mean"], c["std"], lut)
    sizes = share_sizes(batch, n_workers)
    dst = [torch.zeros((n,) + chw, device="cuda") for n in sizes]
    dl = [torch.zeros(n, dtype=torch.int32, device="cuda") for n in sizes]
    synk.synk_gather_rows(dev(c["data"]), dev(c["idx"]), dst, lut=lut, channels=chw[0],
                          labels=dev(c["labels"]), dst_labels=dl)
    raw = ogather.gather_shares(c["data"], c["idx"], n_workers)
    refl = ogather.gather_shares(c["labels"], c["idx"], n_workers)
    for w in range(n_workers):
        ref = ogather.normalise_u8(raw[w], c["mean"], c["std"])
        assert np.array_equal(dst[w].cpu().numpy().view(np.uint32), ref.view(np.uint32)), w
        assert np.array_equal(dl[w].cpu().numpy(), refl[w])


def test_gather_out_of_range_index_is_skipped_and_reported(synk):
    data = np.arange(40, dtype=np.float32).reshape(10, 4)
    idx = np.array([3, 10, -1, 9], dtype=np.int32)
    dst = [torch.full((4, 4), -1.0, device="cuda")]
    ws = torch.zeros(synk.synk_gather_workspace_bytes(), dtype=torch.uint8, device="cuda")
    synk.synk_gather_rows(dev(data), dev(idx), dst, flags=synk.SYNK_FLAG_CHECK_INDEX, ws=ws)
    assert synk.synk_poll_error(ws) == -7
    got = dst[0].cpu().numpy()
    assert np.array_equal(got[0], data[3]) and np.array_equal(got[3], data[9])
    assert np.all(got[1:3] == -1.0)
    synk.synk_gather_rows(dev(data), dev(np.array([1, 2], np.int32)), dst, flags=synk.SYNK_FLAG_CHECK_INDEX, ws=ws)
    assert synk.synk_poll_error(ws) == 0


@pytest.mark.parametrize("start,stop,step,n_workers", [(0, 200, 1, 4), (3, 197, 4, 3), (50, 50, 1, 2), (7, 200, 13, 8),
                                                       (0, 200, 200, 2)])
def test_gather_slice_matches_list_form_and_oracle(synk, start, stop, step, n_workers):
    rng = np.random.default_rng(start + stop + step)
    data = rng.standard_normal((200, 40)).astype(np.float32)
    labels = rng.integers(0, 10, 200).astype(np.int32)
    ix = ogather.slice_indexes(start, stop, step)
    sizes = share_sizes(len(ix), n_workers)
    mk = lambda: ([torch.full((max(n, 1), 40), 9.0, device="cuda")[:n] for n in sizes],
                  [torch.full((max(n, 1),), -5, dtype=torch.int32, device="cuda")[:n] for n in sizes])
    d1, l1 = mk()
    synk.synk_gather_slice(dev(data), start, stop, step, d1, labels=dev(labels), dst_labels=l1)
    ref = ogather.gather_shares(data, ix, n_workers)
    refl = ogather.gather_shares(labels, ix, n_workers)
    for w in range(n_workers):
        assert np.array_equal(d1[w].cpu().numpy(), ref[w]) and np.array_equal(l1[w].cpu().numpy(), refl[w])
    if len(ix):
        d2, l2 = mk()
        synk.synk_gather_rows(dev(data), dev(ix.astype(np.int32)), d2, labels=dev(labels), dst_labels=l2)
        assert all(torch.equal(a, b) for a, b in zip(d1, d2)) and all(torch.equal(a, b) for a, b in zip(l1, l2))


def test_gather_slice_to_bf16_and_u8_paths(synk):
    rng = np.random.default_rng(31)
    data = rng.random((64, 24), dtype=np.float32)
    ix = ogather.slice_indexes(2, 60, 3)
    sizes = share_sizes(len(ix), 4)
    dst = [torch.zeros((n, 24), dtype=torch.bfloat16, device="cuda") for n in sizes]
    synk.synk_gather_slice(dev(data), 2, 60, 3, dst)
    for d, r in zip(dst, ogather.gather_shares(data, ix, 4)):
        assert np.array_equal(d.float().cpu().numpy().view(np.uint32), ogather.round_to_bf16(r).view(np.uint32))
    c = workloads.config4(n_data=24, batch=8, chw=(3, 8, 8), n_workers=2)
    lut = torch.empty(3 * 256, device="cuda")
    synk.synk_build_norm_lut(c["mean"], c["std"], lut)
    ix = ogather.slice_indexes(1, 24, 2)
    sizes = share_sizes(len(ix), 2)
    dst = [torch.zeros((n, 3, 8, 8), device="cuda") for n in sizes]
    synk.synk_gather_slice(dev(c["data"]), 1, 24, 2, dst, lut=lut, channels=3)
    for d, r in zip(dst, ogather.gather_shares(c["data"], ix, 2)):
        assert np.array_equal(d.cpu().numpy().view(np.uint32), ogather.normalise_u8(r, c["mean"], c["std"]).view(np.uint32))


@pytest.mark.parametrize("n_rows,row,n_workers,dtype", [(1000, 48, 8, np.float32), (37, 7, 4, np.float32),
                                                        (5, 16, 8, np.int32), (129, 13, 3, np.uint8)])
def test_scatter_rows_is_the_split_of_the_first_dimension(synk, n_rows, row, n_workers, dtype):
    rng = np.random.default_rng(n_rows)
    data = (rng.standard_normal((n_rows, row)) * 50).astype(dtype)
    labels = rng.integers(0, 10, n_rows).astype(np.int32)
    sizes = share_sizes(n_rows, n_workers)
    tdt = torch.from_numpy(np.zeros(1, dtype)).dtype
    dst = [torch.full((max(n, 1), row), 3, dtype=tdt, device="cuda")[:n] for n in sizes]
    dl = [torch.full((max(n, 1),), -1, dtype=torch.int32, device="cuda")[:n] for n in sizes]
    synk.synk_scatter_rows(dev(data), dst, labels=dev(labels), dst_labels=dl)
    for d, l, r, rl in zip(dst, dl, ogather.scatter(data, n_workers), ogather.scatter(labels, n_workers)):
        assert np.array_equal(d.cpu().numpy(), r) and np.array_equal(l.cpu().numpy(), rl)
    # gathering the shares back in worker order returns the array
    if dtype == np.float32:
        back = torch.zeros(n_rows * row, device="cuda")
        synk.synk_reduce_buffers([d.reshape(-1) for d in dst], synk.SYNK_CONCAT, back)
        assert np.array_equal(back.cpu().numpy().reshape(n_rows, row), data)


def test_gather_resident_different_and_same_lists(synk):
    rng = np.random.default_rng(88)
    data = rng.standard_normal((103, 32)).astype(np.float32)
    labels = rng.integers(0, 10, 103).astype(np.int32)
    shares, lshares = ogather.scatter(data, 4), ogather.scatter(labels, 4)
    dsh, dlsh = [dev(s) for s in shares], [dev(s) for s in lshares]
    lists = [rng.integers(0, len(s), k).astype(np.int32) for s, k in zip(shares, (9, 0, 17, 4))]
    dst = [torch.full((max(len(i), 1), 32), 5.0, device="cuda")[:len(i)] for i in lists]
    dl = [torch.full((max(len(i), 1),), -2, dtype=torch.int32, device="cuda")[:len(i)] for i in lists]
    synk.synk_gather_resident(dsh, [dev(i) for i in lists], dst, labels=dlsh, dst_labels=dl)
    for d, l, r, rl in zip(dst, dl, ogather.gather_resident(shares, lists), ogather.gather_resident(lshares, lists)):
        assert np.array_equal(d.cpu().numpy(), r) and np.array_equal(l.cpu().numpy(), rl)
    # the same list on every worker, rounded to bf16 on the way
    one = dev(np.array([2, 0, 2, 7], np.int32))
    dst = [torch.zeros((4, 32), dtype=torch.bfloat16, device="cuda") for _ in range(4)]
    synk.synk_gather_resident(dsh, [one] * 4, dst)
    for d, r in zip(dst, ogather.gather_resident(shares, [np.array([2, 0, 2, 7])] * 4)):
        assert np.array_equal(d.float().cpu().numpy().view(np.uint32), ogather.round_to_bf16(r).view(np.uint32))


def test_gather_resident_reports_out_of_range_over_all_workers(synk):
    shares = [dev(np.arange(12, dtype=np.float32).reshape(3, 4)), dev(np.arange(8, dtype=np.float32).reshape(2, 4))]
    ws = torch.zeros(synk.synk_gather_workspace_bytes(), dtype=torch.uint8, device="cuda")
    dst = [torch.full((2, 4), -1.0, device="cuda") for _ in range(2)]
    lists = [dev(np.array([0, 2], np.int32)), dev(np.array([1, 2], np.int32))]      # 2 is outside share 1
    synk.synk_gather_resident(shares, lists, dst, flags=synk.SYNK_FLAG_CHECK_INDEX, ws=ws)
    assert synk.synk_poll_error(ws) == -7
    assert np.array_equal(dst[1].cpu().numpy()[0], [4, 5, 6, 7]) and np.all(dst[1].cpu().numpy()[1] == -1.0)
    lists[1] = dev(np.array([1, 0], np.int32))
    synk.synk_gather_resident(shares, lists, dst, flags=synk.SYNK_FLAG_CHECK_INDEX, ws=ws)
    assert synk.synk_poll_error(ws) == 0


# ------------------------------------------------------------------ reduce
@pytest.mark.parametrize("n,length", [(1, 5), (2, 1024), (3, 1027), (8, 4099), (5, 3)])
@pytest.mark.parametrize("op", ["sum", "mean", "max", "min", "prod"])
def test_reduce_float_ops(synk, n, length, op):
    rng = np.random.default_rng(n * 100 + length)
    bufs = [rng.uniform(0.5, 2.0, length).astype(np.float32) * rng.choice([-1, 1], length).astype(np.float32)
            for _ in range(n)]
    out = torch.empty(length, device="cuda")
    synk.synk_reduce_buffers([dev(b) for b in bufs], synk.OP[op], out)
    ref = oreduce.reduce_buffers(bufs, op)
    got = out.cpu().numpy()
    if op in ("max", "min"):
        assert np.array_equal(got, ref.astype(np.float32))
    else:
        assert rel_err(got, ref) < TOL_F32


def test_reduce_weighted_mean_unaligned_and_bit_exact_cases(synk):
    rng = np.random.default_rng(3)
    x = rng.standard_normal(1001).astype(np.float32)
    for n in (1, 2, 4, 8):
        out = torch.empty(1001, device="cuda")
        synk.synk_reduce_buffers([dev(x) for _ in range(n)], synk.SYNK_MEAN, out)
        if n <= 2:      # x/2 + x/2 has no rounding: the buffer comes back bit for bit
            assert np.array_equal(out.cpu().numpy(), x)
        else:           # an in-order fp32 fold passes through 3x/n, which rounds
            assert rel_err(out.cpu().numpy(), x) < 1e-6
    out = torch.empty(1001, device="cuda")
    synk.synk_reduce_buffers([dev(x), dev(-x)], synk.SYNK_SUM, out)
    assert np.all(out.cpu().numpy() == 0.0)
    # buffers that are only 4-byte aligned take the scalar path
    big = [dev(np.r_[np.float32(0), rng.standard_normal(515).astype(np.float32)]) for _ in range(3)]
    views = [b[1:] for b in big]
    w = [0.2, 0.3, 0.5]
    out = torch.empty(516, device="cuda")[1:]
    synk.synk_reduce_buffers(views, synk.SYNK_MEAN, out, weights=w)
    ref = oreduce.reduce_buffers([v.cpu().numpy() for v in views], "mean", w)
    assert rel_err(out.cpu().numpy(), ref) < TOL_F32


@pytest.mark.parametrize("op", ["sum", "max", "min", "prod"])
def test_reduce_int_ops_exact(synk, op):
    rng = np.random.default_rng(4)
    hi = 6 if op == "prod" else 100000
    bufs = [rng.integers(-hi, hi, 1003).astype(np.int32) for _ in range(5)]
    out = torch.empty(1003, dtype=torch.int32, device="cuda")
    synk.synk_reduce_buffers([dev(b) for b in bufs], synk.OP[op], out)
    assert np.array_equal(out.cpu().numpy().astype(np.int64), oreduce.reduce_buffers(bufs, op))


def test_reduce_concat(synk):
    rng = np.random.default_rng(6)
    for dt, tdt in ((np.float32, torch.float32), (np.int32, torch.int32)):
        bufs = [(rng.standard_normal(n) * 1000).astype(dt) for n in (5, 0, 1300, 1)]
        out = torch.zeros(1306, dtype=tdt, device="cuda")
        synk.synk_reduce_buffers([dev(b) if b.size else torch.empty(0, dtype=tdt, device="cuda") for b in bufs],
                                 synk.SYNK_CONCAT, out)
        assert np.array_equal(out.cpu().numpy(), oreduce.reduce_buffers(bufs, "concat"))


# ------------------------------------------------------------------ update
@pytest.mark.parametrize("length", [1, 4, 1027, 203530])
def test_sgd_update(synk, length):
    rng = np.random.default_rng(length)
    p = (rng.standard_normal(length) * 0.05).astype(np.float32)
    v = (rng.standard_normal(length) * 0.01).astype(np.float32)
    g = (rng.standard_normal(length) * 1e-3).astype(np.float32)
    dp, dv, lp = dev(p), dev(v), torch.zeros(length, dtype=torch.bfloat16, device="cuda")
    synk.synk_sgd_update(dp, dv, dev(g), 0.1, 0.9, 1e-4, p_lp=lp)
    rp, rv = oupdate.sgd_momentum(p, v, g, 0.1, 0.9, 1e-4)
    assert rel_err(dp.cpu().numpy(), rp) < TOL_F32 and rel_err(dv.cpu().numpy(), rv) < TOL_F32
    # the bf16 copy is the nearest-even rounding of the fp32 value the kernel wrote
    want = ogather.round_to_bf16(dp.cpu().numpy())
    assert np.array_equal(lp.float().cpu().numpy().view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("n,length", [(1, 1000), (2, 203530), (3, 1025), (8, 70001), (16, 513)])
def test_reduce_sgd_update_matches_oracle_and_unfused_calls(synk, n, length):
    c = workloads.config3(n_params=length, n_workers=n)
    grads = [dev(g) for g in c["grads"]]
    p1, v1 = dev(c["p"]), dev(c["v"])
    loss_out = torch.zeros(1, device="cuda")
    synk.synk_reduce_sgd_update(grads, p1, v1, c["lr"], c["momentum"], c["weight_decay"],
                                loss_in=dev(c["losses"]), loss_out=loss_out)
    rp, rv, rG, rl = oupdate.reduce_and_update(c["p"], c["v"], c["grads"], c["lr"], c["momentum"],
                                               c["weight_decay"], None, c["losses"])
    assert rel_err(p1.cpu().numpy(), rp) < TOL_F32
    assert rel_err(v1.cpu().numpy(), rv) < TOL_F32
    assert abs(loss_out.item() - rl) < TOL_F32 * abs(rl)
    # same thing through the two separate entry points
    G = torch.empty(length, device="cuda")
    synk.synk_reduce_buffers(grads, synk.SYNK_MEAN, G)
    assert rel_err(G.cpu().numpy(), rG) < TOL_F32
    p2, v2 = dev(c["p"]), dev(c["v"])
    synk.synk_sgd_update(p2, v2, G, c["lr"], c["momentum"], c["weight_decay"])
    assert rel_err(p2.cpu().numpy(), rp) < TOL_F32 and rel_err(v2.cpu().numpy(), rv) < TOL_F32


def test_reduce_sgd_update_weights_and_closed_form(synk):
    rng = np.random.default_rng(8)
    g = [rng.standard_normal(333).astype(np.float32) for _ in range(3)]
    p = rng.standard_normal(333).astype(np.float32)
    w = [0.5, 0.25, 0.25]
    dp, dv = dev(p), dev(np.zeros(333, np.float32))
    synk.synk_reduce_sgd_update([dev(x) for x in g], dp, dv, 0.05, 0.0, 0.0, weights=w)
    G = 0.5 * g[0].astype(np.float64) + 0.25 * g[1] + 0.25 * g[2]
    assert rel_err(dp.cpu().numpy(), p - 0.05 * G) < TOL_F32       # zero momentum: p - lr*G


RULE_HYPER = dict(
    momentum=dict(lr=0.05, momentum=0.9, weight_decay=1e-4),
    nesterov=dict(lr=0.05, momentum=0.9, weight_decay=1e-4),
    rmsprop=dict(lr=0.01, rho=0.9, eps=1e-6, weight_decay=1e-4),
    adam=dict(lr=0.001, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=1e-4),
)


@pytest.mark.parametrize("rule", ["momentum", "nesterov", "rmsprop", "adam"])
@pytest.mark.parametrize("n,length", [(1, 1000), (3, 1027), (8, 70001), (16, 513)])
def test_reduce_update_rules_match_oracle_over_several_steps(synk, rule, n, length):
    """Sec. 3.3 steps 2-3 with each update rule: three consecutive updates (state carried on
    the device) against the float64 oracle; gradients sized so that every state array moves."""
    rng = np.random.default_rng(900 + n)
    h = RULE_HYPER[rule]
    p = rng.standard_normal(length).astype(np.float32)
    s1 = np.zeros(length, np.float32)
    s2 = np.zeros(length, np.float32)
    dp, d1, d2 = dev(p), dev(s1), dev(s2)
    lp = torch.zeros(length, dtype=torch.bfloat16, device="cuda")
    rp, r1, r2 = p.astype(np.float64), s1.astype(np.float64), s2.astype(np.float64)
    for step in (1, 2, 3):
        grads = [(rng.standard_normal(length) * 0.1).astype(np.float32) for _ in range(n)]
        losses = rng.random(n).astype(np.float32)
        loss_out = torch.zeros(1, device="cuda")
        synk.synk_reduce_update(rule, [dev(g) for g in grads], dp, d1, d2 if rule == "adam" else None,
                                step=step, p_lp=lp, loss_in=dev(losses), loss_out=loss_out, **h)
        G = oreduce.reduce_buffers(grads, "mean")
        rp, r1, r2n = oupdate.apply_rule(rule, rp, r1, r2, G, dict(h, t=step))
        if r2n is not None:
            r2 = r2n
        assert rel_err(dp.cpu().numpy(), rp) < TOL_F32, (rule, step)
        assert rel_err(d1.cpu().numpy(), r1) < TOL_F32, (rule, step)
        if rule == "adam":
            assert rel_err(d2.cpu().numpy(), r2) < TOL_F32, (rule, step)
        else:
            assert not d2.any().item()                       # untouched
        assert abs(loss_out.item() - float(np.mean(losses.astype(np.float64)))) < 1e-6
        want = ogather.round_to_bf16(dp.cpu().numpy())
        assert np.array_equal(lp.float().cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_reduce_update_momentum_rule_equals_the_dedicated_entry_point(synk):
    c = workloads.config3(n_params=40003, n_workers=8)
    grads = [dev(g) for g in c["grads"]]
    p1, v1, p2, v2 = dev(c["p"]), dev(c["v"]), dev(c["p"]), dev(c["v"])
    synk.synk_reduce_sgd_update(grads, p1, v1, c["lr"], c["momentum"], c["weight_decay"])
    synk.synk_reduce_update("momentum", grads, p2, v2, lr=c["lr"], momentum=c["momentum"],
                            weight_decay=c["weight_decay"])
    assert torch.equal(p1, p2) and torch.equal(v1, v2)      # same arithmetic, same order: bit-exact


def test_reduce_update_adam_weights_and_first_step_closed_form(synk):
    rng = np.random.default_rng(77)
    g = [rng.standard_normal(515).astype(np.float32) for _ in range(2)]
    p = rng.standard_normal(515).astype(np.float32)
    dp, dm, dv = dev(p), dev(np.zeros(515, np.float32)), dev(np.zeros(515, np.float32))
    synk.synk_reduce_update("adam", [dev(x) for x in g], dp, dm, dv, lr=0.01, beta1=0.9, beta2=0.999, eps=1e-8,
                            step=1, weights=[0.75, 0.25])
    G = 0.75 * g[0].astype(np.float64) + 0.25 * g[1]
    want = p - 0.01 * G / (np.abs(G) + 1e-8 / np.sqrt(1 - 0.999))   # first step from zero moments
    assert rel_err(dp.cpu().numpy(), want) < TOL_F32


def test_profile_next_launch_times_the_kernel_itself(synk):
    n = 1 << 22
    grads = [torch.randn(n, device="cuda") for _ in range(4)]
    p, v = torch.randn(n, device="cuda"), torch.zeros(n, device="cuda")
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(); b.record()                      # torch creates the events at the first record
    torch.cuda.synchronize()
    ref_p, ref_v = p.clone(), v.clone()
    synk.synk_reduce_sgd_update(grads, ref_p, ref_v, 0.1, 0.9, 0.0)
    synk.synk_profile_next_launch(a, b)
    synk.synk_reduce_sgd_update(grads, p, v, 0.1, 0.9, 0.0)
    torch.cuda.synchronize()
    ms = a.elapsed_time(b)
    # 4 M elements x 48 B = 100 MB: between 8 TB/s (12.6 us) and a very slow 0.2 TB/s
    assert 0.010 < ms < 0.5, ms
    assert torch.equal(p, ref_p) and torch.equal(v, ref_v)      # the timed launch computes the same
    # the pair was consumed: the next call runs untimed and a cancelled pair leaves nothing pending
    synk.synk_profile_next_launch(a, b)
    synk.synk_profile_next_launch(None, None)
    synk.synk_reduce_sgd_update(grads, p, v, 0.1, 0.9, 0.0)
    torch.cuda.synchronize()


# ------------------------------------------------------------- collectives
@pytest.mark.parametrize("n,length", [(1, 5), (2, 4099), (3, 1027), (8, 70001), (16, 513)])
def test_broadcast_is_bit_exact(synk, n, length):
    rng = np.random.default_rng(40 + n)
    src = rng.standard_normal(length).astype(np.float32)
    dsts = [torch.full((length,), -7.0, device="cuda") for _ in range(n)]
    synk.synk_broadcast(dev(src), dsts)
    for d, r in zip(dsts, ocoll.broadcast(src, n)):
        assert np.array_equal(d.cpu().numpy().view(np.uint32), r.view(np.uint32))
    isrc = rng.integers(-2**31, 2**31 - 1, length).astype(np.int32)
    idst = [torch.zeros(length, dtype=torch.int32, device="cuda") for _ in range(n)]
    synk.synk_broadcast(dev(isrc), idst)
    assert all(np.array_equal(d.cpu().numpy(), isrc) for d in idst)


def test_broadcast_unaligned_views(synk):
    src = np.arange(1000, dtype=np.float32)
    big = [torch.zeros(1003, device="cuda") for _ in range(3)]
    dsts = [b[1 + k:1 + k + 1000] for k, b in enumerate(big)]        # 4-byte aligned only
    synk.synk_broadcast(dev(src), dsts)
    for k, b in enumerate(big):
        got = b.cpu().numpy()
        assert np.array_equal(got[1 + k:1001 + k], src) and got[:1 + k].sum() == 0 and got[1001 + k:].sum() == 0


@pytest.mark.parametrize("op", ["sum", "mean", "max", "min", "prod"])
@pytest.mark.parametrize("n,length", [(1, 7), (2, 4099), (3, 1027), (8, 70001), (16, 513)])
def test_all_reduce_matches_oracle_on_every_worker(synk, op, n, length):
    rng = np.random.default_rng(50 + n)
    host = [((rng.random(length) * 1.5 + 0.5) * (1.0 if op == "prod" else rng.choice([-1.0, 1.0]))).astype(np.float32)
            for _ in range(n)]
    bufs = [dev(h) for h in host]
    synk.synk_all_reduce(bufs, op)
    ref = ocoll.all_reduce(host, op)
    for b, r in zip(bufs, ref):
        got = b.cpu().numpy()
        if op in ("max", "min"):
            assert np.array_equal(got, r.astype(np.float32))        # selections are exact
        else:
            assert rel_err(got, r) < TOL_F32
    assert all(torch.equal(b, bufs[0]) for b in bufs)                 # identical bits on every worker


def test_all_reduce_int32_exact_weights_and_parameter_average(synk):
    rng = np.random.default_rng(61)
    ints = [rng.integers(-1000, 1000, 3001).astype(np.int32) for _ in range(5)]
    for op in ("sum", "max", "min"):
        bufs = [dev(x) for x in ints]
        synk.synk_all_reduce(bufs, op)
        ref = ocoll.all_reduce(ints, op)
        assert all(np.array_equal(b.cpu().numpy(), r.astype(np.int32)) for b, r in zip(bufs, ref))
    host = [rng.standard_normal(2050).astype(np.float32) for _ in range(4)]
    w = [0.4, 0.3, 0.2, 0.1]
    bufs = [dev(h) for h in host]
    synk.synk_all_reduce(bufs, "mean", weights=w)
    assert rel_err(bufs[3].cpu().numpy(), ocoll.all_reduce(host, "mean", w)[3]) < TOL_F32
    # App. A: averaging the parameter copies; a second average changes nothing (up to rounding)
    params = [dev(h) for h in host]
    synk.synk_all_reduce(params, "mean")
    once = params[0].clone()
    synk.synk_all_reduce(params, "mean")
    assert rel_err(params[2].cpu().numpy(), once.cpu().numpy().astype(np.float64)) < 1e-6
    # same numbers as reduce-to-one followed by broadcast
    out = torch.empty(2050, device="cuda")
    synk.synk_reduce_buffers([dev(h) for h in host], synk.SYNK_MEAN, out)
    assert torch.equal(out, once)


@pytest.mark.parametrize("lens", [[5], [3, 0, 7, 1], [1000, 1001, 999, 1000, 1000, 1000, 1000, 1000], [0, 0, 4]])
def test_all_gather_is_bit_exact(synk, lens):
    rng = np.random.default_rng(70 + len(lens))
    host = [rng.standard_normal(k).astype(np.float32) for k in lens]
    total = sum(lens)
    dsts = [torch.full((total,), -3.0, device="cuda") for _ in lens]
    synk.synk_all_gather([dev(h) for h in host], dsts)
    for d, r in zip(dsts, ocoll.all_gather(host)):
        assert np.array_equal(d.cpu().numpy().view(np.uint32), r.view(np.uint32))


def test_all_gather_in_place_segments_and_scatter_roundtrip(synk):
    # each worker's share is the matching segment of its own destination (Sec. 4.2: scatter by first dimension)
    whole = np.random.default_rng(72).standard_normal(4101).astype(np.float32)
    bounds = lib_share_bounds(synk, 4101, 4)
    assert bounds == osplit.share_bounds(4101, 4)
    dsts = [torch.zeros(4101, device="cuda") for _ in range(4)]
    srcs = []
    for w, (a, b) in enumerate(bounds):
        dsts[w][a:b] = dev(whole[a:b])
        srcs.append(dsts[w][a:b])
    synk.synk_all_gather(srcs, dsts)
    assert all(np.array_equal(d.cpu().numpy(), whole) for d in dsts)


# -------------------------------------------------------------- sliced eval
def run_eval(synk, logits, labels, n_slices):
    rows, classes = logits.shape
    ws = torch.empty(synk.synk_sliced_eval_workspace_bytes(rows, classes, n_slices), dtype=torch.uint8, device="cuda")
    o = dict(ce_sum=torch.zeros(1, device="cuda"), counts=torch.full((classes,), -1, dtype=torch.int32, device="cuda"),
             max_logit=torch.zeros(1, device="cuda"), min_logit=torch.zeros(1, device="cuda"),
             n_correct=torch.zeros(1, dtype=torch.int32, device="cuda"),
             argmax=torch.full((rows,), -1, dtype=torch.int32, device="cuda"))
    synk.synk_sliced_eval(dev(logits), dev(labels), n_slices, o["ce_sum"], o["counts"], o["max_logit"],
                          o["min_logit"], o["n_correct"], o["argmax"], ws)
    return {k: v.cpu().numpy() for k, v in o.items()}


def check_eval(got, ref):
    for k in ("counts", "n_correct", "argmax"):
        assert np.array_equal(got[k].astype(np.int64), ref[k]), k
    assert got["max_logit"][0] == np.float32(ref["max_logit"][0])
    assert got["min_logit"][0] == np.float32(ref["min_logit"][0])
    assert abs(got["ce_sum"][0] - ref["ce_sum"][0]) <= TOL_F32 * abs(ref["ce_sum"][0])


@pytest.mark.parametrize("rows,classes,n_slices", [
    (2048, 1000, 64),    # config-5 row shape, 32 rows a slice
    (1000, 1000, 7),     # ragged slices, ragged chunks
    (130, 37, 3),        # class count not a multiple of 4: scalar path
    (5, 10, 8),          # more slices than rows
    (300, 4096, 2),      # widest rows
    (64, 1, 1),          # a single class
    (512, 1024, 4),      # branch-free path: full last vector
    (768, 964, 3),       # branch-free path: the last lane group half padding
    (768, 900, 3),       # branch-free path: one valid vector slot in the last lane group
    (256, 1000, 8),      # branch-free path: four blocks a slice
    (72, 1000, 9),       # branch-free path: one block (8 rows) a slice
    (2080, 1000, 65),    # 32 rows a slice but 65 slices: still regular
    (2048, 960, 64),     # branch-free path, 16 padded lanes
    (2048, 896, 64),     # just below the branch-free path's class range
    (1004, 1000, 251),   # 4 rows a slice: not a whole row set, the general path
])
def test_sliced_eval_matches_oracle(synk, rows, classes, n_slices):
    c = workloads.config5(rows=rows, classes=classes, n_slices=n_slices)
    got = run_eval(synk, c["logits"], c["labels"], n_slices)
    check_eval(got, evalops.sliced(c["logits"], c["labels"], n_slices))


def test_sliced_eval_ties_take_the_lowest_class(synk):
    rng = np.random.default_rng(9)
    logits = (rng.standard_normal((96, 200)) * 2).astype(np.float32)
    for i in range(96):        # plant equal maxima in different lanes / vector slots
        a, b = rng.choice(200, 2, replace=False)
        logits[i, a] = logits[i, b] = 50.0
    labels = rng.integers(0, 200, 96).astype(np.int32)
    got = run_eval(synk, logits, labels, 5)
    check_eval(got, evalops.sliced(logits, labels, 5))


def test_sliced_eval_branch_free_path_ties_and_bad_labels(synk):
    rng = np.random.default_rng(19)
    logits = (rng.standard_normal((128, 1000)) * 2).astype(np.float32)
    for i in range(128):       # equal maxima in different lane groups / vector slots, also in the last vector
        a, b = rng.choice(1000, 2, replace=False)
        if i % 4 == 0:
            b = 996 + (i // 4) % 4
        logits[i, a] = logits[i, b] = 60.0
    labels = rng.integers(0, 1000, 128).astype(np.int32)
    got = run_eval(synk, logits, labels, 2)
    check_eval(got, evalops.sliced(logits, labels, 2))


@pytest.mark.parametrize("rows,classes,n_slices", [(64, 1000, 2), (60, 1000, 2), (20, 37, 2)])
def test_sliced_eval_non_finite_rows_stay_in_range(synk, rows, classes, n_slices):
    # outside the contract (inputs must be finite), but nothing may fault: a row of -inf only counts as
    # class 0, a row of NaN only as some class in range; the other rows keep their arg-max
    rng = np.random.default_rng(29)
    logits = (rng.standard_normal((rows, classes)) * 2).astype(np.float32)
    logits[3, :] = -np.inf
    logits[rows - 2, :] = np.nan
    labels = rng.integers(0, classes, rows).astype(np.int32)
    got = run_eval(synk, logits, labels, n_slices)
    arg = got["argmax"].astype(np.int64)
    want = logits.argmax(axis=1)
    ok = np.ones(rows, dtype=bool)
    ok[rows - 2] = False
    want[3] = 0
    assert np.array_equal(arg[ok], want[ok])
    assert 0 <= arg[rows - 2] < classes
    assert np.array_equal(got["counts"].astype(np.int64), np.bincount(arg, minlength=classes))
    assert int(got["n_correct"][0]) == int((arg == labels).sum())


def test_streaming_kernels_are_reproducible(synk):
    c = workloads.config5(rows=4096, classes=1000, n_slices=16)
    a = run_eval(synk, c["logits"], c["labels"], 16)
    b = run_eval(synk, c["logits"], c["labels"], 16)
    assert all(np.array_equal(a[k], b[k]) for k in a)


# ----------------------------------------------- full sizes, as bench.py launches them
def test_config3_full_size_reduce_and_update(synk):
    c = workloads.config3()                                   # 8 x 25,557,032 fp32, 161 tensors
    assert c["n_params"] == 25557032 and len(c["offsets"]) == 162
    grads = [dev(g) for g in c["grads"]]
    p, v = dev(c["p"]), dev(c["v"])
    loss_out = torch.zeros(1, device="cuda")
    synk.synk_reduce_sgd_update(grads, p, v, c["lr"], c["momentum"], c["weight_decay"],
                                loss_in=dev(c["losses"]), loss_out=loss_out)
    rp, rv, _, rl = oupdate.reduce_and_update(c["p"], c["v"], c["grads"], c["lr"], c["momentum"],
                                              c["weight_decay"], None, c["losses"])
    gp, gv = p.cpu().numpy(), v.cpu().numpy()
    for t in range(161):                                      # per tensor, as the tolerance is defined
        a, b = int(c["offsets"][t]), int(c["offsets"][t + 1])
        assert rel_err(gp[a:b], rp[a:b]) < TOL_F32 and rel_err(gv[a:b], rv[a:b]) < TOL_F32, t
    assert abs(loss_out.item() - rl) < TOL_F32 * abs(rl)


@pytest.mark.parametrize("rule", ["nesterov", "rmsprop", "adam"])
def test_config3_full_size_other_update_rules(synk, rule):
    c = workloads.config3()
    h = RULE_HYPER[rule]
    grads = [dev(g) for g in c["grads"]]
    p = dev(c["p"])
    s1 = torch.full_like(p, 1e-4) if rule != "nesterov" else dev(c["v"])
    s2 = torch.full_like(p, 2e-6)
    r1, r2 = s1.cpu().numpy().astype(np.float64), s2.cpu().numpy().astype(np.float64)
    synk.synk_reduce_update(rule, grads, p, s1, s2 if rule == "adam" else None, step=7, **h)
    G = oreduce.reduce_buffers(list(c["grads"]), "mean")
    rp, q1, q2 = oupdate.apply_rule(rule, c["p"], r1, r2, G, dict(h, t=7))
    gp, g1, g2 = p.cpu().numpy(), s1.cpu().numpy(), s2.cpu().numpy()
    for t in range(161):                                      # every tensor, per tensor
        a, b = int(c["offsets"][t]), int(c["offsets"][t + 1])
        assert rel_err(gp[a:b], rp[a:b]) < TOL_F32 and rel_err(g1[a:b], q1[a:b]) < TOL_F32, (rule, t)
        if rule == "adam":
            assert rel_err(g2[a:b], q2[a:b]) < TOL_F32, t


def test_config3_full_size_collectives(synk):
    c = workloads.config3()
    n, P = c["n_workers"], c["n_params"]
    bufs = [dev(g) for g in c["grads"]]
    synk.synk_all_reduce(bufs, "mean")
    ref = oreduce.reduce_buffers(list(c["grads"]), "mean")
    got = bufs[5].cpu().numpy()
    for t in range(161):                                      # every tensor; the other copies must equal this one
        a, b = int(c["offsets"][t]), int(c["offsets"][t + 1])
        assert rel_err(got[a:b], ref[a:b]) < TOL_F32, t
    assert all(torch.equal(b, bufs[0]) for b in bufs[1:])
    src = dev(c["p"])
    synk.synk_broadcast(src, bufs)
    assert all(torch.equal(b, src) for b in bufs)
    bounds = lib_share_bounds(synk, P, n)                      # shares of 3,194,629: not a multiple of 4
    assert bounds == osplit.share_bounds(P, n)
    synk.synk_all_gather([dev(c["v"][a:b] + np.float32(w)) for w, (a, b) in enumerate(bounds)], bufs)
    want = np.concatenate([c["v"][a:b] + np.float32(w) for w, (a, b) in enumerate(bounds)])
    assert np.array_equal(bufs[3].cpu().numpy(), want) and all(torch.equal(b, bufs[0]) for b in bufs[1:])


def test_config4_full_size_gather_sampled_against_oracle(synk):
    n_data, batch, n_workers, chw = 50000, 256, 8, (3, 224, 224)
    row = chw[0] * chw[1] * chw[2]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(workloads.SEED_BASE + 4)
    data = torch.empty((n_data, row), dtype=torch.uint8, device="cuda")          # 7.5 GB on the device
    for a in range(0, n_data, 5000):
        data[a:a + 5000] = torch.randint(0, 256, (5000, row), dtype=torch.uint8, device="cuda", generator=gen)
    small = workloads.config4(n_data=8, batch=8)
    rng = workloads.rng_for(4, salt=1)
    labels = rng.integers(0, 1000, n_data).astype(np.int32)
    idx = rng.integers(0, n_data, batch).astype(np.int32)
    idx[:3] = [0, n_data - 1, idx[5]]                                            # ends and a duplicate
    lut = torch.empty(3 * 256, device="cuda")
    synk.synk_build_norm_lut(small["mean"], small["std"], lut)
    sizes = share_sizes(batch, n_workers)
    dst = [torch.zeros((n, row), device="cuda") for n in sizes]
    dl = [torch.zeros(n, dtype=torch.int32, device="cuda") for n in sizes]
    synk.synk_gather_rows(data, dev(idx), dst, lut=lut, channels=3, labels=dev(labels), dst_labels=dl)
    # the oracle sees exactly the rows the batch names (fetched from the device dataset)
    src_rows = data[torch.from_numpy(idx.astype(np.int64)).cuda()].cpu().numpy().reshape((batch,) + chw)
    ref = ogather.normalise_u8(src_rows, small["mean"], small["std"]).reshape(batch, row)
    got = torch.cat(dst).cpu().numpy()
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    assert np.array_equal(torch.cat(dl).cpu().numpy(), labels[idx])


def test_config5_full_size_properties_and_sampled_rows(synk):
    import scipy.special
    c = workloads.config5()                                   # 65536 x 1000, 64 slices
    logits, labels = c["logits"], c["labels"]
    got = run_eval(synk, logits, labels, 64)
    # rows the oracle computes one by one
    sample = np.random.default_rng(0).choice(65536, 256, replace=False)
    ref = evalops.function(logits[sample], labels[sample])
    assert np.array_equal(got["argmax"][sample].astype(np.int64), ref["argmax"])
    # properties that hold at any size (each equivalence is pinned on the CPU for the oracle)
    am = got["argmax"].astype(np.int64)
    assert np.array_equal(am, np.argmax(logits, axis=1))
    assert np.array_equal(got["counts"].astype(np.int64), np.bincount(am, minlength=1000))
    assert got["counts"].sum() == 65536
    assert got["n_correct"][0] == int((am == labels).sum())
    assert got["max_logit"][0] == logits.max() and got["min_logit"][0] == logits.min()
    ce = (scipy.special.logsumexp(logits.astype(np.float64), axis=1) - logits[np.arange(65536), labels]).sum()
    assert abs(got["ce_sum"][0] - ce) < TOL_F32 * abs(ce)


def test_peak_probes_run_and_report_their_work(synk):
    buf = torch.zeros(1 << 20, device="cuda")                         # 4 MiB
    assert synk.synk_probe_launch(synk.SYNK_PROBE_MFMA_BF16, buf, 10) == 512 * 8 * 10 * 4 * 32768.0
    assert synk.synk_probe_launch(synk.SYNK_PROBE_FILL, buf, 1) == float(4 << 20)
    torch.cuda.synchronize()
    assert torch.equal(buf.view(-1, 4), torch.tensor([1.0, 2.0, 3.0, 4.0], device="cuda").expand(1 << 18, 4))
    before = buf.clone()
    assert synk.synk_probe_launch(synk.SYNK_PROBE_LDS_FETCH, buf, 48) == 256 * 48 * 16384.0
    torch.cuda.synchronize()
    assert torch.equal(buf, before)                                   # the fetch probe only reads
    assert synk.synk_probe_launch(synk.SYNK_PROBE_READ, buf, 1) == float(4 << 20)
    torch.cuda.synchronize()
    assert torch.equal(buf, before)                                   # and so does the read probe
