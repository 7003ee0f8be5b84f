"""The C-ABI library loads without a GPU, exports every symbol the header
declares, and rejects bad arguments on the host before any HIP call."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import split as osplit
from paper_1710_04162_amd import binding as synk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000        # a non-NULL, 16-byte aligned value never dereferenced by the checks
lib = synk.lib


def test_every_declared_symbol_is_exported():
    text = open(os.path.join(ROOT, "include", "synk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(synk_[a-z0-9_]+)\s*\(", text))
    assert {"synk_gather_rows", "synk_sliced_grad", "synk_reduce_buffers", "synk_sgd_update",
            "synk_reduce_sgd_update", "synk_sliced_eval"} <= names
    for n in sorted(names):
        assert hasattr(lib, n), n
    assert synk.synk_version() == 100
    assert synk.synk_status_string(0) == "ok" and "NULL" in synk.synk_status_string(-1)


@pytest.mark.parametrize("count,parts", [(0, 3), (7, 3), (256, 2), (1024, 8), (5, 8), (100, 7)])
def test_split_rule_matches_oracle(count, parts):
    got = synk.synk_split(count, parts)
    ref = [a for a, _ in osplit.share_bounds(count, parts)] + [count]
    assert got == ref


def test_split_rejects_bad_arguments():
    out = (ctypes.c_int64 * 4)()
    assert lib.synk_split(5, 0, out) == -2
    assert lib.synk_split(-1, 2, out) == -2
    assert lib.synk_split(5, 2, None) == -1


def _tbl(*vals):
    return (ctypes.c_void_p * len(vals))(*vals)


def test_reduce_buffers_argument_checks():
    f = lib.synk_reduce_buffers
    two = _tbl(FAKE, FAKE)
    assert f(None, 2, 8, 2, 0, None, None, FAKE, None) == -1
    assert f(two, 2, 8, 2, 0, None, None, None, None) == -1
    assert f(two, 0, 8, 2, 0, None, None, FAKE, None) == -2
    assert f(two, 65, 8, 2, 0, None, None, FAKE, None) == -2
    assert f(two, 2, -1, 2, 0, None, None, FAKE, None) == -2
    assert f(two, 2, 8, 0, 0, None, None, FAKE, None) == -3          # U8 not supported
    assert f(two, 2, 8, 2, 9, None, None, FAKE, None) == -4
    assert f(two, 2, 8, 1, 1, None, None, FAKE, None) == -4          # MEAN on I32
    w = (ctypes.c_float * 2)(0.5, 0.5)
    assert f(two, 2, 8, 2, 0, w, None, FAKE, None) == -4             # weights only with MEAN
    assert f(two, 2, 8, 2, 5, None, None, FAKE, None) == -1          # CONCAT needs lens
    assert f(_tbl(FAKE, FAKE + 2), 2, 8, 2, 0, None, None, FAKE, None) == -5
    assert f(_tbl(FAKE, None), 2, 8, 2, 0, None, None, FAKE, None) == -1
    assert f(two, 2, 0, 2, 0, None, None, FAKE, None) == 0           # empty: no-op, no launch


def test_update_argument_checks():
    f = lib.synk_sgd_update
    assert f(None, FAKE, FAKE, 8, 0.1, 0.9, 0.0, None, None) == -1
    assert f(FAKE, FAKE, FAKE, -1, 0.1, 0.9, 0.0, None, None) == -2
    assert f(FAKE + 4, FAKE, FAKE, 8, 0.1, 0.9, 0.0, None, None) == -5
    assert f(FAKE, FAKE, FAKE, 0, 0.1, 0.9, 0.0, None, None) == 0
    h = lib.synk_reduce_sgd_update
    two = _tbl(FAKE, FAKE)
    assert h(two, 2, 8, None, FAKE, None, 0.1, 0.9, 0.0, None, None, None, None) == -1
    assert h(two, 0, 8, None, FAKE, FAKE, 0.1, 0.9, 0.0, None, None, None, None) == -2
    assert h(two, 2, 8, None, FAKE, FAKE, 0.1, 0.9, 0.0, None, FAKE, None, None) == -1   # loss pair
    assert h(_tbl(FAKE, FAKE + 8), 2, 8, None, FAKE, FAKE, 0.1, 0.9, 0.0, None, None, None, None) == -5
    assert h(two, 2, 0, None, FAKE, FAKE, 0.1, 0.9, 0.0, None, None, None, None) == 0
    assert lib.synk_cast_bf16(None, FAKE, 4, None) == -1


def test_reduce_update_argument_checks():
    f = lib.synk_reduce_update
    two = _tbl(FAKE, FAKE)
    D = synk.UpdateDesc
    mom = D(synk.SYNK_RULE_MOMENTUM, 0.1, 0.9, 0, 0, 0, 0, 0, 1)
    adam = D(synk.SYNK_RULE_ADAM, 0.1, 0, 0, 0.9, 0.999, 1e-8, 0, 1)
    r = ctypes.byref
    assert f(None, two, 2, 8, None, FAKE, FAKE, None, None, None, None, None) == -1
    assert f(r(mom), two, 2, 8, None, FAKE, None, None, None, None, None, None) == -1      # s1 missing
    assert f(r(adam), two, 2, 8, None, FAKE, FAKE, None, None, None, None, None) == -1     # ADAM needs s2
    assert f(r(D(7, 0.1, 0, 0, 0, 0, 0, 0, 1)), two, 2, 8, None, FAKE, FAKE, None, None, None, None, None) == -4
    assert f(r(D(-1, 0.1, 0, 0, 0, 0, 0, 0, 1)), two, 2, 8, None, FAKE, FAKE, None, None, None, None, None) == -4
    assert f(r(mom), two, 65, 8, None, FAKE, FAKE, None, None, None, None, None) == -2
    assert f(r(mom), two, 2, -3, None, FAKE, FAKE, None, None, None, None, None) == -2
    bad_step = D(synk.SYNK_RULE_ADAM, 0.1, 0, 0, 0.9, 0.999, 1e-8, 0, 0)
    assert f(r(bad_step), two, 2, 8, None, FAKE, FAKE, FAKE, None, None, None, None) == -2
    bad_beta = D(synk.SYNK_RULE_ADAM, 0.1, 0, 0, 1.0, 0.999, 1e-8, 0, 1)
    assert f(r(bad_beta), two, 2, 8, None, FAKE, FAKE, FAKE, None, None, None, None) == -2
    assert f(r(adam), two, 2, 8, None, FAKE, FAKE, FAKE + 4, None, None, None, None) == -5
    assert f(r(mom), _tbl(FAKE, FAKE + 8), 2, 8, None, FAKE, FAKE, None, None, None, None, None) == -5
    assert f(r(mom), two, 2, 8, None, FAKE, FAKE, None, None, FAKE, None, None) == -1     # loss pair
    assert f(r(adam), two, 2, 0, None, FAKE, FAKE, FAKE, None, None, None, None) == 0     # empty: no launch
    assert lib.synk_cast_bf16(FAKE, FAKE + 1, 4, None) == -5


def test_gather_argument_checks():
    f = lib.synk_gather_rows
    d2 = _tbl(FAKE, FAKE)

    def call(data=FAKE, n_rows=10, row_elems=8, src=2, idx=FAKE, n_idx=4, dst=d2, nw=2, dd=2, lut=None,
             ch=0, labels=None, dl=None, flags=0, ws=None, wsb=0):
        return f(data, n_rows, row_elems, src, idx, n_idx, dst, nw, dd, lut, ch, labels, dl, flags, ws,
                 wsb, None)

    assert call(data=None) == -1 and call(idx=None) == -1 and call(dst=None) == -1
    assert call(labels=FAKE) == -1                       # labels without dst_labels
    assert call(row_elems=0) == -2 and call(n_idx=-1) == -2 and call(nw=0) == -2 and call(nw=65) == -2
    assert call(src=7) == -3 and call(src=1, dd=2) == -3          # I32 -> F32 is not a listed pair
    assert call(src=0, dd=2) == -1                       # U8 -> F32 needs the table
    assert call(src=0, dd=2, lut=FAKE, ch=3) == -2       # 8 % 3 != 0
    assert call(src=0, dd=2, lut=FAKE, ch=17) == -2
    assert call(flags=1) == -6                           # flag without workspace
    assert call(dst=_tbl(FAKE, None)) == -1              # non-empty share without a buffer
    assert call(dst=_tbl(FAKE, FAKE + 2)) == -5
    assert lib.synk_build_norm_lut(None, None, 3, FAKE, None) == -1
    m = (ctypes.c_float * 3)(1, 2, 3)
    z = (ctypes.c_float * 3)(1, 0, 3)
    assert lib.synk_build_norm_lut(m, z, 3, FAKE, None) == -2      # std == 0
    assert lib.synk_build_norm_lut(m, m, 17, FAKE, None) == -2
    assert lib.synk_poll_error(None, None) == -1


def test_sliced_grad_argument_checks_and_workspace():
    dims = [20, 16, 10]
    assert synk.synk_mlp_param_count(dims) == 20 * 16 + 16 + 16 * 10 + 10
    assert synk.synk_mlp_param_count([3072, 1024, 1024, 10]) == 4206602
    b32 = synk.synk_sliced_grad_workspace_bytes(dims, synk.SYNK_F32, [5, 0, 7])
    b16 = synk.synk_sliced_grad_workspace_bytes(dims, synk.SYNK_BF16, [5, 0, 7])
    assert b32 > 0 and b16 > 0 and b32 % 256 == 0 and b16 % 256 == 0
    with pytest.raises(synk.SynkError) as e:
        synk.synk_sliced_grad_workspace_bytes(dims, synk.SYNK_F32, [0, 0])
    assert e.value.status == -2
    with pytest.raises(synk.SynkError):
        synk.synk_sliced_grad_workspace_bytes([20, 0, 10], synk.SYNK_F32, [4])
    with pytest.raises(synk.SynkError) as e:
        synk.synk_sliced_grad_workspace_bytes(dims, synk.SYNK_U8, [4])
    assert e.value.status == -3

    f = lib.synk_sliced_grad
    d = synk._desc(dims, synk.SYNK_F32)
    rows = (ctypes.c_int64 * 2)(4, 4)
    t2 = _tbl(FAKE, FAKE)

    def call(desc=d, params=FAKE, lp=None, x=t2, y=t2, r=rows, nw=2, ns=2, op=1, grad=t2, loss=FAKE,
             ws=FAKE, wsb=1 << 30):
        return f(ctypes.byref(desc), params, lp, x, y, r, nw, ns, op, grad, loss, ws, wsb, None)

    assert call(params=None) == -1 and call(x=None) == -1 and call(loss=None) == -1
    assert call(ns=0) == -2 and call(nw=0) == -2
    assert call(op=2) == -4
    assert call(desc=synk._desc(dims, synk.SYNK_BF16)) == -1          # bf16 needs params_lp
    assert call(ws=None) == -6 and call(wsb=16) == -6 and call(ws=FAKE + 16) == -6
    assert call(grad=_tbl(FAKE, FAKE + 2)) == -5
    assert call(x=_tbl(FAKE, None)) == -1


def test_sliced_grad_indexed_argument_checks_and_workspace():
    dims = [20, 16, 10]
    plain = synk.synk_sliced_grad_workspace_bytes(dims, synk.SYNK_F32, [4, 3])
    b = synk.synk_sliced_grad_indexed_workspace_bytes(dims, synk.SYNK_F32, 7, 2)
    assert b % 256 == 0 and b >= plain + 7 * 20 * 4 + 7 * 4       # + the gathered rows and their labels
    with pytest.raises(synk.SynkError) as e:
        synk.synk_sliced_grad_indexed_workspace_bytes(dims, synk.SYNK_F32, 0, 2)
    assert e.value.status == -2
    with pytest.raises(synk.SynkError):
        synk.synk_sliced_grad_indexed_workspace_bytes(dims, synk.SYNK_F32, 7, 65)

    f = lib.synk_sliced_grad_indexed
    d = synk._desc(dims, synk.SYNK_F32)
    t2 = _tbl(FAKE, FAKE)

    def call(desc=d, params=FAKE, lp=None, data=FAKE, labels=FAKE, n_data=50, idx=FAKE, n_idx=7, nw=2, ns=2, op=1,
             grad=t2, loss=FAKE, ws=FAKE, wsb=1 << 30):
        return f(ctypes.byref(desc), params, lp, data, labels, n_data, idx, n_idx, nw, ns, op, grad, loss, ws, wsb,
                 None)

    assert call(params=None) == -1 and call(data=None) == -1 and call(labels=None) == -1 and call(idx=None) == -1
    assert call(grad=None) == -1 and call(loss=None) == -1
    assert call(n_idx=0) == -2 and call(n_data=0) == -2 and call(nw=0) == -2 and call(nw=65) == -2 and call(ns=0) == -2
    assert call(op=2) == -4
    assert call(desc=synk._desc(dims, synk.SYNK_BF16)) == -1          # bf16 needs params_lp
    assert call(data=FAKE + 2) == -5 and call(idx=FAKE + 1) == -5 and call(grad=_tbl(FAKE, FAKE + 2)) == -5
    assert call(ws=None) == -6 and call(wsb=b - 1) == -6 and call(ws=FAKE + 16) == -6


def test_sliced_grad_conv_argument_checks_and_workspace():
    shape = (6, 5, 8, 16, 10)
    assert synk.synk_convblock_param_count(shape) == 9 * 8 * 16 + 2 * 16 + 16 * 10 + 10
    assert synk.synk_convblock_param_count((56, 56, 64, 64, 1000)) == 9 * 64 * 64 + 128 + 64 * 1000 + 1000
    b32 = synk.synk_sliced_grad_conv_workspace_bytes(shape, synk.SYNK_F32, [5, 0, 7], 2)
    b16 = synk.synk_sliced_grad_conv_workspace_bytes(shape, synk.SYNK_BF16, [5, 0, 7], 2)
    assert b32 > b16 > 0 and b32 % 256 == 0 and b16 % 256 == 0
    for bad, status in [((6, 5, 7, 16, 10), -2), ((6, 5, 8, 12, 10), -2), ((0, 5, 8, 16, 10), -2),
                        ((6, 5, 8, 520, 10), -2), ((6, 5, 8, 16, 5000), -2), ((6, 5, 8, 16, 0), -2)]:
        with pytest.raises(synk.SynkError) as e:
            synk.synk_sliced_grad_conv_workspace_bytes(bad, synk.SYNK_F32, [4], 1)
        assert e.value.status == status
    with pytest.raises(synk.SynkError) as e:
        synk.synk_sliced_grad_conv_workspace_bytes(shape, synk.SYNK_F32, [0, 0], 1)
    assert e.value.status == -2
    with pytest.raises(synk.SynkError) as e:
        synk.synk_sliced_grad_conv_workspace_bytes(shape, synk.SYNK_U8, [4], 1)
    assert e.value.status == -3
    with pytest.raises(synk.SynkError) as e:
        synk.synk_sliced_grad_conv_workspace_bytes(shape, synk.SYNK_F32, [4], 1, eps=-1.0)
    assert e.value.status == -2

    f = lib.synk_sliced_grad_conv
    d = synk._conv_desc(shape, synk.SYNK_F32, 1e-5)
    rows = (ctypes.c_int64 * 2)(4, 4)
    t2 = _tbl(FAKE, FAKE)

    def call(desc=d, params=FAKE, x=t2, y=t2, r=rows, nw=2, ns=2, op=1, grad=t2, loss=FAKE, ws=FAKE,
             wsb=1 << 30):
        return f(ctypes.byref(desc), params, x, y, r, nw, ns, op, grad, loss, ws, wsb, None)

    assert call(params=None) == -1 and call(x=None) == -1 and call(loss=None) == -1 and call(r=None) == -1
    assert call(ns=0) == -2 and call(nw=0) == -2 and call(nw=65) == -2
    assert call(r=(ctypes.c_int64 * 2)(4, -1)) == -2
    assert call(op=2) == -4
    assert call(ws=None) == -6 and call(wsb=16) == -6 and call(ws=FAKE + 16) == -6
    assert call(grad=_tbl(FAKE, FAKE + 4)) == -5 and call(x=_tbl(FAKE + 8, FAKE)) == -5
    assert call(params=FAKE + 4) == -5
    assert call(x=_tbl(FAKE, None)) == -1 and call(y=_tbl(None, FAKE)) == -1



def test_sliced_grad_conv_indexed_argument_checks_and_workspace():
    shape = (6, 5, 8, 16, 10)
    plain = synk.synk_sliced_grad_conv_workspace_bytes(shape, synk.SYNK_F32, [4, 3], 2)
    b = synk.synk_sliced_grad_conv_indexed_workspace_bytes(shape, synk.SYNK_F32, 7, 2, 2)
    assert b % 256 == 0 and b >= plain + 7 * 6 * 5 * 8 * 4 + 7 * 4          # + the gathered images and labels
    with pytest.raises(synk.SynkError) as e:
        synk.synk_sliced_grad_conv_indexed_workspace_bytes(shape, synk.SYNK_F32, 0, 2, 2)
    assert e.value.status == -2
    f = lib.synk_sliced_grad_conv_indexed
    d = synk._conv_desc(shape, synk.SYNK_F32, 1e-5)
    t2 = _tbl(FAKE, FAKE)

    def call(desc=d, params=FAKE, data=FAKE, labels=FAKE, n_data=50, idx=FAKE, n_idx=7, nw=2, ns=2, op=1, grad=t2,
             loss=FAKE, ws=FAKE, wsb=1 << 30):
        return f(ctypes.byref(desc), params, data, labels, n_data, idx, n_idx, nw, ns, op, grad, loss, ws, wsb, None)

    assert call(params=None) == -1 and call(data=None) == -1 and call(labels=None) == -1 and call(idx=None) == -1
    assert call(grad=None) == -1 and call(loss=None) == -1
    assert call(n_idx=0) == -2 and call(n_data=0) == -2 and call(nw=0) == -2 and call(nw=65) == -2 and call(ns=0) == -2
    assert call(op=2) == -4
    assert call(data=FAKE + 8) == -5 and call(idx=FAKE + 2) == -5 and call(grad=_tbl(FAKE, FAKE + 4)) == -5
    assert call(ws=None) == -6 and call(wsb=b - 1) == -6 and call(ws=FAKE + 16) == -6


def test_sliced_eval_argument_checks_and_workspace():
    # four partial results per (slice, row set of 8 rows)
    assert synk.synk_sliced_eval_workspace_bytes(65536, 1000, 64) >= 4 * 64 * (1024 // 8) * 4
    for bad in [(0, 10, 1), (10, 0, 1), (10, 5000, 1), (10, 10, 0)]:
        with pytest.raises(synk.SynkError) as e:
            synk.synk_sliced_eval_workspace_bytes(*bad)
        assert e.value.status == -2
    f = lib.synk_sliced_eval
    assert f(None, FAKE, 8, 4, 2, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 20, None) == -1
    assert f(FAKE, FAKE, 8, 4, 2, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, None) == -6
    assert f(FAKE, FAKE, 8, 4, 2, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 8, None) == -6
    assert f(FAKE + 1, FAKE, 8, 4, 2, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 20, None) == -5
    # the variant with the fixed array: same checks, and a size limit instead of a workspace
    g = lib.synk_sliced_eval_static
    assert g(None, FAKE, 8, 4, 2, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None) == -1
    assert g(FAKE, FAKE, 0, 4, 2, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None) == -2
    assert g(FAKE + 1, FAKE, 8, 4, 2, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None) == -5
    assert synk.synk_sliced_eval_workspace_bytes(8 * 70000, 4, 1) > (1 << 20)
    assert g(FAKE, FAKE, 8 * 70000, 4, 1, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None) == -6


def test_binding_refuses_host_tensors():
    import torch
    t = torch.zeros(8)
    with pytest.raises(ValueError):
        synk.synk_sgd_update(t, t, t, 0.1, 0.9)


def test_collectives_argument_checks():
    two = _tbl(FAKE, FAKE + 64)
    b = lib.synk_broadcast
    assert b(None, two, 2, 8, 2, None) == -1
    assert b(FAKE, None, 2, 8, 2, None) == -1
    assert b(FAKE, _tbl(FAKE, None), 2, 8, 2, None) == -1
    assert b(FAKE, two, 0, 8, 2, None) == -2
    assert b(FAKE, two, 2, -1, 2, None) == -2
    assert b(FAKE, two, 2, 8, 0, None) == -3
    assert b(FAKE + 2, two, 2, 8, 2, None) == -5
    assert b(FAKE, two, 2, 0, 2, None) == 0
    ar = lib.synk_all_reduce
    w = (ctypes.c_float * 2)(0.5, 0.5)
    assert ar(None, 2, 8, 2, 0, None, None) == -1
    assert ar(two, 65, 8, 2, 0, None, None) == -2
    assert ar(_tbl(FAKE, FAKE), 2, 8, 2, 0, None, None) == -2          # the same buffer twice
    assert ar(two, 2, 8, 3, 0, None, None) == -3
    assert ar(two, 2, 8, 2, 5, None, None) == -4                       # CONCAT is all_gather
    assert ar(two, 2, 8, 1, 1, None, None) == -4                       # MEAN on I32
    assert ar(two, 2, 8, 2, 0, w, None) == -4                          # weights only with MEAN
    assert ar(_tbl(FAKE, FAKE + 66), 2, 8, 2, 0, None, None) == -5
    assert ar(two, 2, 0, 2, 1, w, None) == 0
    ag = lib.synk_all_gather
    lens = (ctypes.c_int64 * 2)(3, 5)
    assert ag(None, lens, 2, 2, two, None) == -1
    assert ag(two, None, 2, 2, two, None) == -1
    assert ag(two, lens, 2, 2, None, None) == -1
    assert ag(two, (ctypes.c_int64 * 2)(3, -1), 2, 2, two, None) == -2
    assert ag(two, lens, 2, 0, two, None) == -3
    assert ag(_tbl(FAKE, FAKE + 3), lens, 2, 2, two, None) == -5
    assert ag(two, lens, 2, 2, _tbl(FAKE, None), None) == -1
    assert ag(two, (ctypes.c_int64 * 2)(0, 0), 2, 2, two, None) == 0


def test_slice_scatter_and_resident_gather_argument_checks():
    one = _tbl(FAKE)
    gs = lib.synk_gather_slice
    assert gs(FAKE, 10, 4, 2, 0, 10, 0, one, 1, 2, None, 0, None, None, None) == -2      # step < 1
    assert gs(FAKE, 10, 4, 2, -1, 10, 1, one, 1, 2, None, 0, None, None, None) == -7
    assert gs(FAKE, 10, 4, 2, 0, 11, 1, one, 1, 2, None, 0, None, None, None) == -7
    assert gs(FAKE, 10, 4, 2, 6, 5, 1, one, 1, 2, None, 0, None, None, None) == -7
    assert gs(None, 10, 4, 2, 0, 10, 1, one, 1, 2, None, 0, None, None, None) == -1
    assert gs(FAKE, 10, 4, 2, 0, 10, 1, one, 0, 2, None, 0, None, None, None) == -2
    assert gs(FAKE, 10, 4, 2, 0, 10, 1, one, 1, 0, None, 0, None, None, None) == -3      # F32 -> U8
    assert gs(FAKE, 10, 4, 2, 5, 5, 1, one, 1, 2, None, 0, None, None, None) == 0        # empty slice
    sc = lib.synk_scatter_rows
    assert sc(None, 10, 4, 2, one, 1, None, None, None) == -1
    assert sc(FAKE, 10, 4, 2, _tbl(None), 1, None, None, None) == -1
    assert sc(FAKE, 10, 0, 2, one, 1, None, None, None) == -2
    assert sc(FAKE, 0, 4, 2, one, 1, None, None, None) == 0
    gr = lib.synk_gather_resident
    rows = (ctypes.c_int64 * 2)(5, 5)
    nidx = (ctypes.c_int64 * 2)(3, 3)
    two = _tbl(FAKE, FAKE + 64)
    assert gr(None, rows, 4, 2, two, nidx, two, 2, 2, None, 0, None, None, 0, None, 0, None) == -1
    assert gr(two, rows, 4, 2, _tbl(FAKE, None), nidx, two, 2, 2, None, 0, None, None, 0, None, 0, None) == -1
    assert gr(two, rows, 4, 2, two, (ctypes.c_int64 * 2)(3, -1), two, 2, 2, None, 0, None, None, 0, None, 0, None) == -2
    assert gr(two, rows, 4, 2, two, nidx, two, 65, 2, None, 0, None, None, 0, None, 0, None) == -2
    assert gr(two, rows, 4, 2, two, nidx, two, 2, 0, None, 0, None, None, 0, None, 0, None) == -3
    assert gr(two, rows, 4, 2, two, nidx, two, 2, 2, None, 0, None, None, 1, None, 0, None) == -6   # flag, no ws
    assert gr(two, rows, 4, 2, two, (ctypes.c_int64 * 2)(0, 0), _tbl(None, None), 2, 2, None, 0, None, None, 0,
              None, 0, None) == 0


def test_profile_next_launch_argument_checks():
    f = lib.synk_profile_next_launch
    assert f(FAKE, None) == -1 and f(None, FAKE) == -1
    assert f(FAKE, FAKE + 8) == 0
    assert f(None, None) == 0          # cancels the pending pair: nothing is left for a later launch


def test_profile_next_launch_of_selects_a_kernel_and_reports_pending():
    f, pending = lib.synk_profile_next_launch_of, lib.synk_profile_pending
    assert pending() == 0
    assert f(synk.SYNK_KERNEL_MLP_FORWARD(2), FAKE, None) == -1
    assert f(-1, FAKE, FAKE + 8) == -2
    assert f(synk.SYNK_KERNEL_MLP_FORWARD(2), FAKE, FAKE + 8) == 0 and pending() == 1
    assert f(synk.SYNK_KERNEL_MAIN, None, None) == 0 and pending() == 0


def test_probe_launch_argument_checks():
    f = lib.synk_probe_launch
    work = ctypes.c_double(0.0)
    assert f(0, None, 64, 10, ctypes.byref(work), None) == -1
    assert f(0, FAKE, 64, 10, None, None) == -1
    assert f(0, FAKE, 64, 0, ctypes.byref(work), None) == -2
    assert f(1, FAKE + 4, 1 << 20, 1, ctypes.byref(work), None) == -2          # misaligned buffer
    assert f(0, FAKE, 2, 10, ctypes.byref(work), None) == -6                    # buffer too small
    assert f(2, FAKE, 1 << 16, 48, ctypes.byref(work), None) == -6              # window of 768 KB not covered
    assert f(2, FAKE, 1 << 20, 49, ctypes.byref(work), None) == -6              # more steps than the window holds
    assert f(3, FAKE, 32767, 1, ctypes.byref(work), None) == -2                 # less than one 32 KB workgroup to read
    assert f(7, FAKE, 1 << 20, 1, ctypes.byref(work), None) == -9
    assert f(synk.SYNK_PROBE_MFMA_BESIDE_VALU + 3, FAKE, 64, 1, ctypes.byref(work), None) == -9     # a count it has no kernel for
    assert f(synk.SYNK_PROBE_MFMA_BESIDE_LDS + 0, FAKE, 64, 1, ctypes.byref(work), None) == -9
    assert f(synk.SYNK_PROBE_MFMA_BESIDE_VALU + 4, FAKE, 2, 1, ctypes.byref(work), None) == -6
