"""ctypes binding of libsynk.so.  Argument marshalling only.

Every function has the name of the C entry point it calls (include/synk.h has
the semantics).  Tensors must already live on the GPU; lists of tensors become
host pointer tables.  A negative status raises SynkError.  Launches go on
torch's current stream unless `stream` (a raw hipStream_t integer) is given.
"""
import ctypes
import os

import torch

__all__ = [
    "SynkError", "lib", "LIB_PATH", "DTYPE", "OP", "Prepared", "prepare",
    "SYNK_U8", "SYNK_I32", "SYNK_F32", "SYNK_BF16",
    "SYNK_SUM", "SYNK_MEAN", "SYNK_MAX", "SYNK_MIN", "SYNK_PROD", "SYNK_CONCAT",
    "SYNK_FLAG_CHECK_INDEX", "SYNK_MAX_WORKERS",
    "synk_version", "synk_status_string", "synk_split", "synk_gather_workspace_bytes",
    "synk_gather_rows", "synk_build_norm_lut", "synk_poll_error", "synk_mlp_param_count",
    "synk_sliced_grad_workspace_bytes", "synk_sliced_grad", "synk_cast_bf16",
    "synk_sliced_grad_indexed_workspace_bytes", "synk_sliced_grad_indexed",
    "synk_sliced_grad_conv_indexed_workspace_bytes", "synk_sliced_grad_conv_indexed",
    "synk_sliced_eval_workspace_bytes", "synk_sliced_eval", "synk_sliced_eval_static",
    "synk_static_scratch_init", "synk_reduce_buffers",
    "synk_sgd_update", "synk_reduce_sgd_update", "synk_reduce_update",
    "synk_broadcast", "synk_all_reduce", "synk_all_gather",
    "synk_gather_slice", "synk_scatter_rows", "synk_gather_resident", "synk_profile_next_launch",
    "synk_profile_next_launch_of", "synk_profile_pending", "synk_probe_launch",
    "SYNK_PROBE_MFMA_BF16", "SYNK_PROBE_FILL", "SYNK_PROBE_LDS_FETCH", "SYNK_PROBE_READ", "SYNK_PROBE_MFMA_BESIDE_VALU", "SYNK_PROBE_MFMA_BESIDE_LDS", "SYNK_KERNEL_MAIN", "SYNK_KERNEL_MLP_HEAD", "SYNK_KERNEL_MLP_BACKWARD_GROUP",
    "SYNK_KERNEL_MLP_FORWARD", "SYNK_KERNEL_MLP_DW", "SYNK_KERNEL_MLP_DX",
    "synk_convblock_param_count", "synk_sliced_grad_conv_workspace_bytes", "synk_sliced_grad_conv",
]

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsynk.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libsynk.so is not built: run `python -m paper_1710_04162_amd.build` "
                      "(there is no fallback path)")
lib = ctypes.CDLL(LIB_PATH)

SYNK_U8, SYNK_I32, SYNK_F32, SYNK_BF16 = 0, 1, 2, 3
SYNK_SUM, SYNK_MEAN, SYNK_MAX, SYNK_MIN, SYNK_PROD, SYNK_CONCAT = 0, 1, 2, 3, 4, 5
SYNK_FLAG_CHECK_INDEX = 1
SYNK_MAX_WORKERS = 64
DTYPE = {torch.uint8: SYNK_U8, torch.int32: SYNK_I32, torch.float32: SYNK_F32,
         torch.bfloat16: SYNK_BF16}
OP = dict(sum=SYNK_SUM, mean=SYNK_MEAN, max=SYNK_MAX, min=SYNK_MIN, prod=SYNK_PROD,
          concat=SYNK_CONCAT)

_vp, _i64, _int, _f32, _sz = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float,
                              ctypes.c_size_t)
_pp = ctypes.POINTER(ctypes.c_void_p)
_pi64 = ctypes.POINTER(ctypes.c_int64)
_pf32 = ctypes.POINTER(ctypes.c_float)


class MlpDesc(ctypes.Structure):
    _fields_ = [("n_layers", _int), ("dims", _pi64), ("compute_dtype", _int)]


class UpdateDesc(ctypes.Structure):
    _fields_ = [("rule", _int), ("lr", _f32), ("momentum", _f32), ("rho", _f32), ("beta1", _f32),
                ("beta2", _f32), ("eps", _f32), ("weight_decay", _f32), ("step", _i64)]


class ConvBlockDesc(ctypes.Structure):
    _fields_ = [("height", _int), ("width", _int), ("c_in", _int), ("c_out", _int), ("classes", _int),
                ("compute_dtype", _int), ("eps", _f32)]


SYNK_RULE_MOMENTUM, SYNK_RULE_NESTEROV, SYNK_RULE_RMSPROP, SYNK_RULE_ADAM = 0, 1, 2, 3
RULE = dict(momentum=SYNK_RULE_MOMENTUM, nesterov=SYNK_RULE_NESTEROV, rmsprop=SYNK_RULE_RMSPROP,
            adam=SYNK_RULE_ADAM)


lib.synk_version.restype = _int
lib.synk_status_string.restype = ctypes.c_char_p
lib.synk_status_string.argtypes = [_int]
lib.synk_split.argtypes = [_i64, _int, _pi64]
lib.synk_gather_workspace_bytes.restype = _sz
lib.synk_gather_rows.argtypes = [_vp, _i64, _i64, _int, _vp, _i64, _pp, _int, _int, _vp, _int, _vp,
                                 _pp, ctypes.c_uint32, _vp, _sz, _vp]
lib.synk_gather_slice.argtypes = [_vp, _i64, _i64, _int, _i64, _i64, _i64, _pp, _int, _int, _vp, _int, _vp, _pp,
                                  _vp]
lib.synk_scatter_rows.argtypes = [_vp, _i64, _i64, _int, _pp, _int, _vp, _pp, _vp]
lib.synk_gather_resident.argtypes = [_pp, _pi64, _i64, _int, _pp, _pi64, _pp, _int, _int, _vp, _int, _pp, _pp,
                                     ctypes.c_uint32, _vp, _sz, _vp]
for _n in ("synk_gather_slice", "synk_scatter_rows", "synk_gather_resident"):
    getattr(lib, _n).restype = _int
lib.synk_profile_next_launch.argtypes = [_vp, _vp]
lib.synk_profile_next_launch.restype = _int
lib.synk_probe_launch.argtypes = [_int, _vp, _sz, _int, ctypes.POINTER(ctypes.c_double), _vp]
lib.synk_probe_launch.restype = _int
lib.synk_profile_pending.argtypes = []
lib.synk_profile_pending.restype = _int
lib.synk_profile_next_launch_of.argtypes = [_int, _vp, _vp]
lib.synk_profile_next_launch_of.restype = _int
lib.synk_build_norm_lut.argtypes = [_pf32, _pf32, _int, _vp, _vp]
lib.synk_poll_error.argtypes = [_vp, _vp]
lib.synk_mlp_param_count.argtypes = [ctypes.POINTER(MlpDesc), _pi64]
lib.synk_sliced_grad_workspace_bytes.argtypes = [ctypes.POINTER(MlpDesc), _pi64, _int,
                                                 ctypes.POINTER(_sz)]
lib.synk_sliced_grad.argtypes = [ctypes.POINTER(MlpDesc), _vp, _vp, _pp, _pp, _pi64, _int, _int,
                                 _int, _pp, _vp, _vp, _sz, _vp]
lib.synk_sliced_grad_indexed_workspace_bytes.argtypes = [ctypes.POINTER(MlpDesc), _i64, _int, ctypes.POINTER(_sz)]
lib.synk_sliced_grad_indexed_workspace_bytes.restype = _int
lib.synk_sliced_grad_indexed.argtypes = [ctypes.POINTER(MlpDesc), _vp, _vp, _vp, _vp, _i64, _vp, _i64, _int, _int,
                                         _int, _pp, _vp, _vp, _sz, _vp]
lib.synk_sliced_grad_indexed.restype = _int
lib.synk_sliced_grad_conv_indexed_workspace_bytes.argtypes = [ctypes.POINTER(ConvBlockDesc), _i64, _int, _int,
                                                              ctypes.POINTER(_sz)]
lib.synk_sliced_grad_conv_indexed_workspace_bytes.restype = _int
lib.synk_sliced_grad_conv_indexed.argtypes = [ctypes.POINTER(ConvBlockDesc), _vp, _vp, _vp, _i64, _vp, _i64, _int, _int,
                                              _int, _pp, _vp, _vp, _sz, _vp]
lib.synk_sliced_grad_conv_indexed.restype = _int
lib.synk_convblock_param_count.argtypes = [ctypes.POINTER(ConvBlockDesc), _pi64]
lib.synk_sliced_grad_conv_workspace_bytes.argtypes = [ctypes.POINTER(ConvBlockDesc), _pi64, _int, _int,
                                                      ctypes.POINTER(_sz)]
lib.synk_sliced_grad_conv.argtypes = [ctypes.POINTER(ConvBlockDesc), _vp, _pp, _pp, _pi64, _int, _int, _int, _pp,
                                      _vp, _vp, _sz, _vp]
for _n in ("synk_convblock_param_count", "synk_sliced_grad_conv_workspace_bytes", "synk_sliced_grad_conv"):
    getattr(lib, _n).restype = _int
lib.synk_cast_bf16.argtypes = [_vp, _vp, _i64, _vp]
lib.synk_sliced_eval_workspace_bytes.argtypes = [_i64, _i64, _int, ctypes.POINTER(_sz)]
lib.synk_sliced_eval.argtypes = [_vp, _vp, _i64, _i64, _int, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz,
                                 _vp]
lib.synk_sliced_eval_static.argtypes = [_vp, _vp, _i64, _i64, _int, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.synk_sliced_eval_static.restype = _int
lib.synk_static_scratch_init.argtypes = []
lib.synk_static_scratch_init.restype = _int
lib.synk_reduce_buffers.argtypes = [_pp, _int, _i64, _int, _int, _pf32, _pi64, _vp, _vp]
lib.synk_sgd_update.argtypes = [_vp, _vp, _vp, _i64, _f32, _f32, _f32, _vp, _vp]
lib.synk_reduce_sgd_update.argtypes = [_pp, _int, _i64, _pf32, _vp, _vp, _f32, _f32, _f32, _vp, _vp,
                                       _vp, _vp]
lib.synk_reduce_update.argtypes = [ctypes.POINTER(UpdateDesc), _pp, _int, _i64, _pf32, _vp, _vp, _vp, _vp,
                                   _vp, _vp, _vp]
lib.synk_reduce_update.restype = _int
lib.synk_broadcast.argtypes = [_vp, _pp, _int, _i64, _int, _vp]
lib.synk_all_reduce.argtypes = [_pp, _int, _i64, _int, _int, _pf32, _vp]
lib.synk_all_gather.argtypes = [_pp, _pi64, _int, _int, _pp, _vp]
for _n in ("synk_broadcast", "synk_all_reduce", "synk_all_gather"):
    getattr(lib, _n).restype = _int
for _n in ("synk_split", "synk_gather_rows", "synk_build_norm_lut", "synk_poll_error",
           "synk_mlp_param_count", "synk_sliced_grad_workspace_bytes", "synk_sliced_grad",
           "synk_cast_bf16", "synk_sliced_eval_workspace_bytes", "synk_sliced_eval",
           "synk_reduce_buffers", "synk_sgd_update", "synk_reduce_sgd_update"):
    getattr(lib, _n).restype = _int


class SynkError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, lib.synk_status_string(status).decode(), status))


def _check(status, where):
    if status != 0:
        raise SynkError(status, where)


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("libsynk takes device tensors only")
    if not t.is_contiguous():
        raise ValueError("libsynk takes dense (contiguous) tensors only")
    return t.data_ptr()


def _table(tensors):
    arr = (ctypes.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = _ptr(t) or None      # an empty tensor may have no storage: NULL
    return arr


def _stream(stream):
    return torch.cuda.current_stream().cuda_stream if stream is None else stream


def _ws(ws):
    return (None, 0) if ws is None else (_ptr(ws), ws.numel() * ws.element_size())


def _desc(dims, compute_dtype):
    arr = (ctypes.c_int64 * len(dims))(*[int(d) for d in dims])
    d = MlpDesc(len(dims) - 1, arr, compute_dtype)
    d._keep = arr
    return d


def synk_version():
    return lib.synk_version()


def synk_status_string(status):
    return lib.synk_status_string(status).decode()


def synk_split(count, parts):
    out = (ctypes.c_int64 * (parts + 1))()
    _check(lib.synk_split(count, parts, out), "synk_split")
    return list(out)


def synk_gather_workspace_bytes():
    return lib.synk_gather_workspace_bytes()


class Prepared:
    """One C call with its arguments already marshalled: calling it repeats the
    call (same pointers, same sizes, same stream).  Keeps the tensors alive.
    For loops that must not pay Python marshalling on every launch."""

    __slots__ = ("fn", "args", "keep", "where")

    def __init__(self, fn, args, keep, where):
        self.fn, self.args, self.keep, self.where = fn, args, keep, where

    def __call__(self):
        status = self.fn(*self.args)
        if status != 0:
            raise SynkError(status, self.where)


def prepare(wrapper, *args, **kwargs):
    """prepare(synk_gather_rows, data, idx, dst, ...) -> Prepared."""
    return wrapper(*args, _prepare=True, **kwargs)


def _run(fn, args, keep, where, _prepare):
    if _prepare:
        return Prepared(fn, args, keep, where)
    _check(fn(*args), where)


def synk_gather_rows(data, idx, dst, lut=None, channels=0, labels=None, dst_labels=None, flags=0,
                     ws=None, stream=None, _prepare=False):
    n_rows = data.shape[0]
    row_elems = 1
    for d in data.shape[1:]:
        row_elems *= int(d)
    wsp, wsb = _ws(ws)
    t_dst = _table(dst)
    t_lab = _table(dst_labels) if dst_labels is not None else None
    args = (_ptr(data), n_rows, row_elems, DTYPE[data.dtype], _ptr(idx), idx.numel(), t_dst, len(dst),
            DTYPE[dst[0].dtype], _ptr(lut), channels, _ptr(labels), t_lab, flags, wsp, wsb, _stream(stream))
    return _run(lib.synk_gather_rows, args, (data, idx, dst, lut, labels, dst_labels, ws, t_dst, t_lab),
                "synk_gather_rows", _prepare)


def synk_build_norm_lut(mean, std, lut, stream=None):
    c = len(mean)
    m = (ctypes.c_float * c)(*[float(x) for x in mean])
    s = (ctypes.c_float * c)(*[float(x) for x in std])
    _check(lib.synk_build_norm_lut(m, s, c, _ptr(lut), _stream(stream)), "synk_build_norm_lut")


def synk_poll_error(ws, stream=None):
    return lib.synk_poll_error(_ptr(ws), _stream(stream))


def synk_mlp_param_count(dims, compute_dtype=SYNK_F32):
    out = ctypes.c_int64(0)
    _check(lib.synk_mlp_param_count(ctypes.byref(_desc(dims, compute_dtype)), ctypes.byref(out)),
           "synk_mlp_param_count")
    return out.value


def synk_sliced_grad_workspace_bytes(dims, compute_dtype, rows):
    out = _sz(0)
    r = (ctypes.c_int64 * len(rows))(*[int(x) for x in rows])
    _check(lib.synk_sliced_grad_workspace_bytes(ctypes.byref(_desc(dims, compute_dtype)), r, len(rows),
                                                ctypes.byref(out)), "synk_sliced_grad_workspace_bytes")
    return out.value


def synk_sliced_grad(dims, compute_dtype, params, params_lp, x, y, rows, n_slices, grad_op, grad, loss,
                     ws, stream=None, _prepare=False):
    r = (ctypes.c_int64 * len(rows))(*[int(v) for v in rows])
    wsp, wsb = _ws(ws)
    desc = _desc(dims, compute_dtype)
    tx, ty, tg = _table(x), _table(y), _table(grad)
    args = (ctypes.byref(desc), _ptr(params), _ptr(params_lp), tx, ty, r, len(rows), n_slices, grad_op,
            tg, _ptr(loss), wsp, wsb, _stream(stream))
    return _run(lib.synk_sliced_grad, args, (desc, params, params_lp, x, y, r, grad, loss, ws, tx, ty, tg),
                "synk_sliced_grad", _prepare)


def synk_sliced_grad_indexed_workspace_bytes(dims, compute_dtype, n_idx, n_workers):
    out = _sz(0)
    _check(lib.synk_sliced_grad_indexed_workspace_bytes(ctypes.byref(_desc(dims, compute_dtype)), n_idx, n_workers,
                                                        ctypes.byref(out)),
           "synk_sliced_grad_indexed_workspace_bytes")
    return out.value


def synk_sliced_grad_indexed(dims, compute_dtype, params, params_lp, data, labels, idx, n_slices, grad_op, grad,
                             loss, ws, stream=None, _prepare=False):
    wsp, wsb = _ws(ws)
    desc = _desc(dims, compute_dtype)
    tg = _table(grad)
    args = (ctypes.byref(desc), _ptr(params), _ptr(params_lp), _ptr(data), _ptr(labels), data.shape[0], _ptr(idx),
            idx.numel(), len(grad), n_slices, grad_op, tg, _ptr(loss), wsp, wsb, _stream(stream))
    return _run(lib.synk_sliced_grad_indexed, args, (desc, params, params_lp, data, labels, idx, grad, loss, ws, tg),
                "synk_sliced_grad_indexed", _prepare)


def _conv_desc(shape, compute_dtype, eps):
    H, W, cin, cout, classes = [int(v) for v in shape]
    return ConvBlockDesc(H, W, cin, cout, classes, compute_dtype, float(eps))


def synk_convblock_param_count(shape, compute_dtype=SYNK_F32, eps=1e-5):
    out = ctypes.c_int64(0)
    _check(lib.synk_convblock_param_count(ctypes.byref(_conv_desc(shape, compute_dtype, eps)), ctypes.byref(out)),
           "synk_convblock_param_count")
    return out.value


def synk_sliced_grad_conv_workspace_bytes(shape, compute_dtype, rows, n_slices, eps=1e-5):
    out = _sz(0)
    r = (ctypes.c_int64 * len(rows))(*[int(x) for x in rows])
    _check(lib.synk_sliced_grad_conv_workspace_bytes(ctypes.byref(_conv_desc(shape, compute_dtype, eps)), r,
                                                     len(rows), n_slices, ctypes.byref(out)),
           "synk_sliced_grad_conv_workspace_bytes")
    return out.value


def synk_sliced_grad_conv(shape, compute_dtype, eps, params, x, y, rows, n_slices, grad_op, grad, loss, ws,
                          stream=None, _prepare=False):
    r = (ctypes.c_int64 * len(rows))(*[int(v) for v in rows])
    wsp, wsb = _ws(ws)
    desc = _conv_desc(shape, compute_dtype, eps)
    tx, ty, tg = _table(x), _table(y), _table(grad)
    args = (ctypes.byref(desc), _ptr(params), tx, ty, r, len(rows), n_slices, grad_op, tg, _ptr(loss), wsp, wsb,
            _stream(stream))
    return _run(lib.synk_sliced_grad_conv, args, (desc, params, x, y, r, grad, loss, ws, tx, ty, tg),
                "synk_sliced_grad_conv", _prepare)


def synk_sliced_grad_conv_indexed_workspace_bytes(shape, compute_dtype, n_idx, n_workers, n_slices, eps=1e-5):
    out = _sz(0)
    _check(lib.synk_sliced_grad_conv_indexed_workspace_bytes(ctypes.byref(_conv_desc(shape, compute_dtype, eps)), n_idx,
                                                             n_workers, n_slices, ctypes.byref(out)),
           "synk_sliced_grad_conv_indexed_workspace_bytes")
    return out.value


def synk_sliced_grad_conv_indexed(shape, compute_dtype, eps, params, data, labels, idx, n_slices, grad_op, grad, loss,
                                  ws, stream=None, _prepare=False):
    wsp, wsb = _ws(ws)
    desc = _conv_desc(shape, compute_dtype, eps)
    tg = _table(grad)
    args = (ctypes.byref(desc), _ptr(params), _ptr(data), _ptr(labels), data.shape[0], _ptr(idx), idx.numel(),
            len(grad), n_slices, grad_op, tg, _ptr(loss), wsp, wsb, _stream(stream))
    return _run(lib.synk_sliced_grad_conv_indexed, args, (desc, params, data, labels, idx, grad, loss, ws, tg),
                "synk_sliced_grad_conv_indexed", _prepare)


def synk_cast_bf16(src, dst, stream=None):
    _check(lib.synk_cast_bf16(_ptr(src), _ptr(dst), src.numel(), _stream(stream)), "synk_cast_bf16")


def synk_sliced_eval_workspace_bytes(rows, classes, n_slices):
    out = _sz(0)
    _check(lib.synk_sliced_eval_workspace_bytes(rows, classes, n_slices, ctypes.byref(out)),
           "synk_sliced_eval_workspace_bytes")
    return out.value


def synk_sliced_eval(logits, labels, n_slices, ce_sum, class_counts, max_logit, min_logit, n_correct,
                     argmax, ws, stream=None, _prepare=False):
    rows, classes = logits.shape
    wsp, wsb = _ws(ws)
    args = (_ptr(logits), _ptr(labels), rows, classes, n_slices, _ptr(ce_sum), _ptr(class_counts),
            _ptr(max_logit), _ptr(min_logit), _ptr(n_correct), _ptr(argmax), wsp, wsb, _stream(stream))
    return _run(lib.synk_sliced_eval, args,
                (logits, labels, ce_sum, class_counts, max_logit, min_logit, n_correct, argmax, ws),
                "synk_sliced_eval", _prepare)


def synk_static_scratch_init():
    _check(lib.synk_static_scratch_init(), "synk_static_scratch_init")


def synk_sliced_eval_static(logits, labels, n_slices, ce_sum, class_counts, max_logit, min_logit, n_correct,
                            argmax, stream=None, _prepare=False):
    rows, classes = logits.shape
    args = (_ptr(logits), _ptr(labels), rows, classes, n_slices, _ptr(ce_sum), _ptr(class_counts),
            _ptr(max_logit), _ptr(min_logit), _ptr(n_correct), _ptr(argmax), _stream(stream))
    return _run(lib.synk_sliced_eval_static, args,
                (logits, labels, ce_sum, class_counts, max_logit, min_logit, n_correct, argmax),
                "synk_sliced_eval_static", _prepare)


def synk_reduce_buffers(bufs, op, out, weights=None, stream=None, _prepare=False):
    n = len(bufs)
    w = (ctypes.c_float * n)(*[float(x) for x in weights]) if weights is not None else None
    lens = (ctypes.c_int64 * n)(*[b.numel() for b in bufs]) if op == SYNK_CONCAT else None
    tb = _table(bufs)
    args = (tb, n, bufs[0].numel(), DTYPE[bufs[0].dtype], op, w, lens, _ptr(out), _stream(stream))
    return _run(lib.synk_reduce_buffers, args, (bufs, out, w, lens, tb), "synk_reduce_buffers", _prepare)


def synk_sgd_update(p, v, g, lr, momentum, weight_decay=0.0, p_lp=None, stream=None, _prepare=False):
    args = (_ptr(p), _ptr(v), _ptr(g), p.numel(), lr, momentum, weight_decay, _ptr(p_lp), _stream(stream))
    return _run(lib.synk_sgd_update, args, (p, v, g, p_lp), "synk_sgd_update", _prepare)


def synk_reduce_sgd_update(grads, p, v, lr, momentum, weight_decay=0.0, weights=None, p_lp=None,
                           loss_in=None, loss_out=None, stream=None, _prepare=False):
    n = len(grads)
    w = (ctypes.c_float * n)(*[float(x) for x in weights]) if weights is not None else None
    tg = _table(grads)
    args = (tg, n, p.numel(), w, _ptr(p), _ptr(v), lr, momentum, weight_decay, _ptr(p_lp), _ptr(loss_in),
            _ptr(loss_out), _stream(stream))
    return _run(lib.synk_reduce_sgd_update, args, (grads, p, v, w, p_lp, loss_in, loss_out, tg),
                "synk_reduce_sgd_update", _prepare)


def synk_reduce_update(rule, grads, p, s1, s2=None, lr=0.0, momentum=0.0, rho=0.0, beta1=0.0, beta2=0.0,
                       eps=0.0, weight_decay=0.0, step=1, weights=None, p_lp=None, loss_in=None,
                       loss_out=None, stream=None, _prepare=False):
    """rule: one of SYNK_RULE_* (or its name).  A prepared call keeps `step` as given:
    prepare one call per step value for ADAM."""
    n = len(grads)
    u = UpdateDesc(RULE[rule] if isinstance(rule, str) else int(rule), lr, momentum, rho, beta1, beta2, eps,
                   weight_decay, int(step))
    w = (ctypes.c_float * n)(*[float(x) for x in weights]) if weights is not None else None
    tg = _table(grads)
    args = (ctypes.byref(u), tg, n, p.numel(), w, _ptr(p), _ptr(s1), _ptr(s2), _ptr(p_lp), _ptr(loss_in),
            _ptr(loss_out), _stream(stream))
    return _run(lib.synk_reduce_update, args, (u, grads, p, s1, s2, w, p_lp, loss_in, loss_out, tg),
                "synk_reduce_update", _prepare)


def synk_broadcast(src, dsts, stream=None, _prepare=False):
    td = _table(dsts)
    args = (_ptr(src), td, len(dsts), src.numel(), DTYPE[src.dtype], _stream(stream))
    return _run(lib.synk_broadcast, args, (src, dsts, td), "synk_broadcast", _prepare)


def synk_all_reduce(bufs, op, weights=None, stream=None, _prepare=False):
    n = len(bufs)
    w = (ctypes.c_float * n)(*[float(x) for x in weights]) if weights is not None else None
    tb = _table(bufs)
    args = (tb, n, bufs[0].numel(), DTYPE[bufs[0].dtype], OP[op] if isinstance(op, str) else int(op), w,
            _stream(stream))
    return _run(lib.synk_all_reduce, args, (bufs, tb, w), "synk_all_reduce", _prepare)


def synk_all_gather(srcs, dsts, stream=None, _prepare=False):
    n = len(srcs)
    if len(dsts) != n:
        raise ValueError("synk_all_gather: one destination per worker")
    lens = (ctypes.c_int64 * n)(*[int(s.numel()) for s in srcs])
    ts, td = _table(srcs), _table(dsts)
    args = (ts, lens, n, DTYPE[srcs[0].dtype], td, _stream(stream))
    return _run(lib.synk_all_gather, args, (srcs, dsts, lens, ts, td), "synk_all_gather", _prepare)


def _row_elems(data):
    n = 1
    for d in data.shape[1:]:
        n *= int(d)
    return n


def synk_gather_slice(data, start, stop, step, dst, lut=None, channels=0, labels=None, dst_labels=None,
                      stream=None, _prepare=False):
    t_dst = _table(dst)
    t_lab = _table(dst_labels) if dst_labels is not None else None
    args = (_ptr(data), data.shape[0], _row_elems(data), DTYPE[data.dtype], int(start), int(stop), int(step),
            t_dst, len(dst), DTYPE[dst[0].dtype], _ptr(lut), channels, _ptr(labels), t_lab, _stream(stream))
    return _run(lib.synk_gather_slice, args, (data, dst, lut, labels, dst_labels, t_dst, t_lab),
                "synk_gather_slice", _prepare)


def synk_scatter_rows(data, dst, labels=None, dst_labels=None, stream=None, _prepare=False):
    t_dst = _table(dst)
    t_lab = _table(dst_labels) if dst_labels is not None else None
    args = (_ptr(data), data.shape[0], _row_elems(data), DTYPE[data.dtype], t_dst, len(dst), _ptr(labels), t_lab,
            _stream(stream))
    return _run(lib.synk_scatter_rows, args, (data, dst, labels, dst_labels, t_dst, t_lab),
                "synk_scatter_rows", _prepare)


def synk_gather_resident(shares, idx, dst, lut=None, channels=0, labels=None, dst_labels=None, flags=0,
                         ws=None, stream=None, _prepare=False):
    """shares, idx, dst (and labels, dst_labels): one tensor per worker."""
    n = len(shares)
    rows = (ctypes.c_int64 * n)(*[int(s.shape[0]) for s in shares])
    nidx = (ctypes.c_int64 * n)(*[int(i.numel()) for i in idx])
    wsp, wsb = _ws(ws)
    t_sh, t_ix, t_dst = _table(shares), _table(idx), _table(dst)
    t_lab = _table(labels) if labels is not None else None
    t_dl = _table(dst_labels) if dst_labels is not None else None
    args = (t_sh, rows, _row_elems(shares[0]), DTYPE[shares[0].dtype], t_ix, nidx, t_dst, n, DTYPE[dst[0].dtype],
            _ptr(lut), channels, t_lab, t_dl, flags, wsp, wsb, _stream(stream))
    return _run(lib.synk_gather_resident, args,
                (shares, idx, dst, lut, labels, dst_labels, ws, rows, nidx, t_sh, t_ix, t_dst, t_lab, t_dl),
                "synk_gather_resident", _prepare)


SYNK_KERNEL_MAIN, SYNK_KERNEL_MLP_HEAD, SYNK_KERNEL_MLP_BACKWARD_GROUP = 0, 1, 2


def SYNK_KERNEL_MLP_FORWARD(l):
    return 16 + l


def SYNK_KERNEL_MLP_DW(l):
    return 32 + l


def SYNK_KERNEL_MLP_DX(l):
    return 48 + l


def synk_profile_next_launch(start, stop):
    """start, stop: torch.cuda.Event(enable_timing=True) that have been recorded once (torch creates
    the underlying hipEvent_t at the first record), or None, None to cancel."""
    synk_profile_next_launch_of(SYNK_KERNEL_MAIN, start, stop)


SYNK_PROBE_MFMA_BF16, SYNK_PROBE_FILL, SYNK_PROBE_LDS_FETCH, SYNK_PROBE_READ = 0, 1, 2, 3
SYNK_PROBE_MFMA_BESIDE_VALU, SYNK_PROBE_MFMA_BESIDE_LDS = 16, 32      # + the number of other instructions


def synk_probe_launch(probe, buf, iters, stream=None):
    """Launches one timing probe; returns the flops or bytes the launch does."""
    work = ctypes.c_double(0.0)
    _check(lib.synk_probe_launch(int(probe), _ptr(buf), buf.numel() * buf.element_size(), int(iters),
                                 ctypes.byref(work), _stream(stream)), "synk_probe_launch")
    return work.value


def synk_profile_pending():
    return bool(lib.synk_profile_pending())


def synk_profile_next_launch_of(kernel, start, stop):
    a = start.cuda_event if start is not None else None
    b = stop.cuda_event if stop is not None else None
    _check(lib.synk_profile_next_launch_of(int(kernel), a, b), "synk_profile_next_launch_of")
