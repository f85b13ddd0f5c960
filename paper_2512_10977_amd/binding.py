"""Thin ctypes binding of libtxops.so: the same entry points as include/txops.h.

Argument marshalling only.  torch tensors are used as device buffers: a tensor
becomes a tx_tensor descriptor (data_ptr, dtype code, sizes, strides) and the
current torch stream is passed as the hipStream_t.  Every call raises TxError
on a negative status.  There is no fallback: if the native library is missing,
loading it raises.
"""
import ctypes
import os

import torch

MAX_DIMS = 8
BOOL, I32, I64, F16, BF16, F32 = range(6)
DTYPE_CODE = {torch.bool: BOOL, torch.int32: I32, torch.int64: I64, torch.float16: F16,
              torch.bfloat16: BF16, torch.float32: F32}
CODE_DTYPE = {v: k for k, v in DTYPE_CODE.items()}

UNARY = {"neg": 0, "abs": 1, "exp": 2, "log": 3, "sqrt": 4, "sigmoid": 5, "tanh": 6, "gelu": 7, "log1p": 8, "expm1": 9,
         "logsigmoid": 10, "logical_not": 11, "sin": 12, "cos": 13, "exp2": 14, "log2": 15, "log10": 16, "rsqrt": 17,
         "reciprocal": 18, "silu": 19, "square": 20, "sign": 21, "floor": 22, "ceil": 23, "trunc": 24, "round": 25, "isnan": 26,
         "isinf": 27, "isfinite": 28, "bitwise_not": 29, "tan": 30, "asin": 31, "acos": 32, "atan": 33, "sinh": 34, "cosh": 35,
         "asinh": 36, "acosh": 37, "atanh": 38, "erf": 39, "erfc": 40, "relu": 41, "frac": 42, "signbit": 43, "hardswish": 44,
         "hardsigmoid": 45, "mish": 46}
BINARY = {"add": 0, "mul": 1, "div": 2, "maximum": 3, "eq": 4, "sub": 5, "minimum": 6, "ne": 7, "lt": 8, "le": 9, "gt": 10,
          "ge": 11, "logical_and": 12, "logical_or": 13, "logical_xor": 14, "pow": 15, "bitwise_and": 16, "bitwise_or": 17,
          "bitwise_xor": 18, "atan2": 19, "fmod": 20, "remainder": 21, "hypot": 22, "copysign": 23, "logaddexp": 24,
          "logaddexp2": 25, "xlogy": 26, "heaviside": 27, "fmax": 28, "fmin": 29, "nextafter": 30, "gcd": 31, "lcm": 32,
          "bitwise_left_shift": 33, "bitwise_right_shift": 34, "floor_divide": 35, "trunc_divide": 36}
REDUCE = {"sum": 0, "mean": 1, "amax": 2, "argmax": 3, "prod": 4, "var": 5, "amin": 6, "argmin": 7, "std": 8, "any": 9,
          "all": 10, "logsumexp": 11, "nansum": 12, "nanmean": 13, "count_nonzero": 14, "norm": 15}

STATUS = {0: "OK", -1: "NULL", -2: "NDIM", -3: "DTYPE", -4: "SHAPE", -5: "DIM", -6: "OVERLAP",
          -7: "EMPTY_REDUCTION", -8: "SCALAR", -9: "WORKSPACE", -10: "INDEX", -11: "LAUNCH", -12: "UNSUPPORTED"}

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libtxops.so")

EXPORTS = ["tx_unary", "tx_add", "tx_sub", "tx_binary", "tx_clamp", "tx_infer_clamp_dtype", "tx_where", "tx_masked_fill", "tx_reduce", "tx_reduce_workspace_bytes", "tx_reduce_static",
           "tx_softmax", "tx_layer_norm", "tx_binary_cross_entropy", "tx_binary_cross_entropy_workspace_bytes", "tx_loss", "tx_loss_workspace_bytes", "tx_cumsum", "tx_cumsum_workspace_bytes", "tx_scan", "tx_scan_workspace_bytes", "tx_gather", "tx_index_select", "tx_scatter_add_",
           "tx_scatter_add_workspace_bytes", "tx_index_add_", "tx_index_add_workspace_bytes", "tx_scatter_reduce_", "tx_scatter_reduce_workspace_bytes",
           "tx_index_put_", "tx_index_put_workspace_bytes", "tx_take", "tx_searchsorted", "tx_masked_select",
           "tx_masked_select_workspace_bytes", "tx_nonzero", "tx_nonzero_workspace_bytes", "tx_infer_binary", "tx_copy", "tx_flip", "tx_roll", "tx_tri", "tx_infer_where", "tx_infer_unary_dtype", "tx_unary_param", "tx_infer_unary_param_dtype", "tx_ternary", "tx_infer_ternary_dtype",
           "tx_infer_reduce", "tx_last_path", "tx_force_path", "tx_strerror", "tx_last_error",
           "tx_set_index_validation", "tx_get_index_validation", "tx_lookback_status"]


class TxError(RuntimeError):
    def __init__(self, status, detail):
        super().__init__("txops error %d (%s): %s" % (status, STATUS.get(status, "?"), detail))
        self.status = status
        self.kind = STATUS.get(status, "?")


class TxTensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("dtype", ctypes.c_int32), ("ndim", ctypes.c_int32),
                ("sizes", ctypes.c_int64 * MAX_DIMS), ("strides", ctypes.c_int64 * MAX_DIMS)]


_lib = None


def lib():
    """Load libtxops.so (built in-tree by build.py).  Raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libtxops.so is not built: run `python -m paper_2512_10977_amd.build` "
                           "(or __graft_entry__.build()) first; there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(TxTensor)
    I64P = ctypes.POINTER(ctypes.c_int64)
    I32P = ctypes.POINTER(ctypes.c_int32)
    V = ctypes.c_void_p
    sig = {
        "tx_unary": ([ctypes.c_int, P, P, V], ctypes.c_int32),
        "tx_add": ([P, P, P, ctypes.c_double, ctypes.c_int64, ctypes.c_int, V], ctypes.c_int32),
        "tx_sub": ([P, P, P, ctypes.c_double, ctypes.c_int64, ctypes.c_int, V], ctypes.c_int32),
        "tx_binary": ([ctypes.c_int, P, P, P, V], ctypes.c_int32),
        "tx_clamp": ([P, P, ctypes.c_int, ctypes.c_double, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                      ctypes.c_int64, ctypes.c_int, V], ctypes.c_int32),
        "tx_infer_clamp_dtype": ([ctypes.c_int32] + [ctypes.c_int] * 4, ctypes.c_int32),
        "tx_where": ([P, P, P, P, V], ctypes.c_int32),
        "tx_masked_fill": ([P, P, P, ctypes.c_double, ctypes.c_int64, ctypes.c_int, V], ctypes.c_int32),
        "tx_reduce": ([ctypes.c_int, P, P, I64P, ctypes.c_int32, ctypes.c_int, ctypes.c_double, V, ctypes.c_size_t, V],
                      ctypes.c_int32),
        "tx_reduce_workspace_bytes": ([ctypes.c_int, P, P, I64P, ctypes.c_int32, ctypes.c_int], ctypes.c_size_t),
        "tx_reduce_static": ([ctypes.c_int, P, P, I64P, ctypes.c_int32, ctypes.c_int, ctypes.c_double, V], ctypes.c_int32),
        "tx_softmax": ([P, P, ctypes.c_int64, ctypes.c_int, V], ctypes.c_int32),
        "tx_layer_norm": ([P, P, ctypes.c_int32, P, P, ctypes.c_double, V], ctypes.c_int32),
        "tx_binary_cross_entropy": ([P, P, P, P, ctypes.c_int, V, ctypes.c_size_t, V], ctypes.c_int32),
        "tx_binary_cross_entropy_workspace_bytes": ([P, P, P, P, ctypes.c_int], ctypes.c_size_t),
        "tx_loss": ([ctypes.c_int, P, P, P, ctypes.c_int, ctypes.c_double, V, ctypes.c_size_t, V], ctypes.c_int32),
        "tx_loss_workspace_bytes": ([ctypes.c_int, P, P, P, ctypes.c_int, ctypes.c_double], ctypes.c_size_t),
        "tx_cumsum": ([P, P, ctypes.c_int64, V, ctypes.c_size_t, V], ctypes.c_int32),
        "tx_scan": ([ctypes.c_int, P, P, ctypes.c_int64, V, ctypes.c_size_t, V], ctypes.c_int32),
        "tx_scan_workspace_bytes": ([ctypes.c_int, P, P, ctypes.c_int64], ctypes.c_size_t),
        "tx_cumsum_workspace_bytes": ([P, P, ctypes.c_int64], ctypes.c_size_t),
        "tx_gather": ([P, P, ctypes.c_int64, P, V], ctypes.c_int32),
        "tx_index_select": ([P, P, ctypes.c_int64, P, V], ctypes.c_int32),
        "tx_scatter_add_": ([P, ctypes.c_int64, P, P, ctypes.c_int, V, ctypes.c_size_t, V], ctypes.c_int32),
        "tx_scatter_add_workspace_bytes": ([P, ctypes.c_int64, P, P, ctypes.c_int], ctypes.c_size_t),
        "tx_index_add_": ([P, ctypes.c_int64, P, P, ctypes.c_double, ctypes.c_int64, ctypes.c_int, ctypes.c_int, V,
                           ctypes.c_size_t, V], ctypes.c_int32),
        "tx_index_add_workspace_bytes": ([P, ctypes.c_int64, P, P, ctypes.c_int], ctypes.c_size_t),
        "tx_scatter_reduce_": ([P, ctypes.c_int64, P, P, ctypes.c_int, ctypes.c_int, V, ctypes.c_size_t, V], ctypes.c_int32),
        "tx_scatter_reduce_workspace_bytes": ([P, ctypes.c_int64, P, P, ctypes.c_int, ctypes.c_int], ctypes.c_size_t),
        "tx_index_put_": ([P, ctypes.POINTER(P), ctypes.c_int32, P, ctypes.c_int, V, ctypes.c_size_t, V], ctypes.c_int32),
        "tx_index_put_workspace_bytes": ([P, ctypes.POINTER(P), ctypes.c_int32, P, ctypes.c_int], ctypes.c_size_t),
        "tx_take": ([P, P, P, V], ctypes.c_int32),
        "tx_searchsorted": ([P, P, P, ctypes.c_int, V], ctypes.c_int32),
        "tx_masked_select": ([P, P, P, P, V, ctypes.c_size_t, V], ctypes.c_int32),
        "tx_masked_select_workspace_bytes": ([P, P, P, P], ctypes.c_size_t),
        "tx_nonzero": ([P, P, P, V, ctypes.c_size_t, V], ctypes.c_int32),
        "tx_nonzero_workspace_bytes": ([P, P, P], ctypes.c_size_t),
        "tx_infer_binary": ([ctypes.c_int, P, P, I32P, I32P, I64P], ctypes.c_int32),
        "tx_infer_where": ([P, P, I32P], ctypes.c_int32),
        "tx_infer_unary_dtype": ([ctypes.c_int, ctypes.c_int32], ctypes.c_int32),
        "tx_copy": ([P, P, V], ctypes.c_int32),
        "tx_flip": ([P, P, ctypes.POINTER(ctypes.c_int64), ctypes.c_int32, V], ctypes.c_int32),
        "tx_roll": ([P, P, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64), ctypes.c_int32, V], ctypes.c_int32),
        "tx_tri": ([P, P, ctypes.c_int64, ctypes.c_int, V], ctypes.c_int32),
        "tx_unary_param": ([ctypes.c_int, P, P, ctypes.c_double, ctypes.c_double, ctypes.c_double, V], ctypes.c_int32),
        "tx_infer_unary_param_dtype": ([ctypes.c_int, ctypes.c_int32], ctypes.c_int32),
        "tx_ternary": ([ctypes.c_int, P, P, P, P, ctypes.c_double, ctypes.c_int64, ctypes.c_int, V], ctypes.c_int32),
        "tx_infer_ternary_dtype": ([ctypes.c_int, P, P, P], ctypes.c_int32),
        "tx_infer_reduce": ([ctypes.c_int, P, I64P, ctypes.c_int32, ctypes.c_int, I32P, I32P, I64P], ctypes.c_int32),
        "tx_set_index_validation": ([ctypes.c_int], None),
        "tx_get_index_validation": ([], ctypes.c_int),
        "tx_lookback_status": ([V, V], ctypes.c_int32),
        "tx_last_path": ([], ctypes.c_char_p),
        "tx_force_path": ([ctypes.c_char_p], None),
        "tx_strerror": ([ctypes.c_int32], ctypes.c_char_p),
        "tx_last_error": ([], ctypes.c_char_p),
    }
    for name, (args, res) in sig.items():
        fn = getattr(L, name)   # raises if the library does not export an entry point
        fn.argtypes = args
        fn.restype = res
    _lib = L
    return L


def desc(t):
    """tx_tensor descriptor of a torch tensor (any device; data is passed as a raw pointer).  A descriptor built
    earlier passes through, so a caller that launches the same operands many times marshals them once."""
    if isinstance(t, TxTensor):
        return t
    d = TxTensor()
    d.data = t.data_ptr() if t.numel() else None
    d.dtype = DTYPE_CODE[t.dtype]
    d.ndim = t.dim()
    for i in range(t.dim()):
        d.sizes[i] = t.size(i)
        d.strides[i] = t.stride(i)
    return d


def current_stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _stream(stream):
    return current_stream() if stream is None else stream


def _check(status):
    if status < 0:
        raise TxError(status, lib().tx_last_error().decode())


def _scalar(v):
    if isinstance(v, bool):
        return float(v), int(v), 1
    if isinstance(v, int):
        return float(v), v, 1
    return float(v), 0, 0


def _dims(dims):
    if dims is None:
        return (ctypes.c_int64 * 1)(), 0
    if isinstance(dims, int):
        dims = [dims]
    dims = list(dims)
    return (ctypes.c_int64 * max(1, len(dims)))(*dims), len(dims)


def _ws(ws):
    if ws is None:
        return None, 0
    return ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


# --------------------------------------------------------------------------- entry points (same names as the C ABI)
def tx_unary(op, out, a, stream=None):
    _check(lib().tx_unary(UNARY[op], desc(out), desc(a), _stream(stream)))


def tx_add(out, a, b, alpha=1, stream=None):
    af, ai, isint = _scalar(alpha)
    _check(lib().tx_add(desc(out), desc(a), desc(b), af, ai, isint, _stream(stream)))


def tx_sub(out, a, b, alpha=1, stream=None):
    af, ai, isint = _scalar(alpha)
    _check(lib().tx_sub(desc(out), desc(a), desc(b), af, ai, isint, _stream(stream)))


def tx_binary(op, out, a, b, stream=None):
    _check(lib().tx_binary(BINARY[op], desc(out), desc(a), desc(b), _stream(stream)))


def tx_clamp(out, x, lo=None, hi=None, stream=None):
    lf, li, lint = _scalar(0 if lo is None else lo)
    hf, hi_i, hint = _scalar(0 if hi is None else hi)
    _check(lib().tx_clamp(desc(out), desc(x), lo is not None, lf, li, lint, hi is not None, hf, hi_i, hint,
                          _stream(stream)))


def tx_infer_clamp_dtype(dtype, lo=None, hi=None):
    rc = lib().tx_infer_clamp_dtype(DTYPE_CODE[dtype], lo is not None, _scalar(0 if lo is None else lo)[2],
                                    hi is not None, _scalar(0 if hi is None else hi)[2])
    _check(rc)
    return CODE_DTYPE[rc]


def tx_index_add_workspace_bytes(self, dim, index, source, deterministic=True):
    return lib().tx_index_add_workspace_bytes(desc(self), dim, desc(index), desc(source), int(deterministic))


def tx_index_add_(self, dim, index, source, alpha=1, deterministic=True, ws=None, stream=None):
    af, ai, isint = _scalar(alpha)
    p, n = _ws(ws)
    _check(lib().tx_index_add_(desc(self), dim, desc(index), desc(source), af, ai, isint, int(deterministic), p, n,
                               _stream(stream)))


SCATTER_REDUCE = {"sum": 0, "prod": 1, "mean": 2, "amax": 3, "amin": 4}


def tx_scatter_reduce_workspace_bytes(self, dim, index, src, reduce, include_self=True):
    return lib().tx_scatter_reduce_workspace_bytes(desc(self), dim, desc(index), desc(src), SCATTER_REDUCE.get(reduce, 9),
                                                   int(include_self))


def tx_scatter_reduce_(self, dim, index, src, reduce, include_self=True, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().tx_scatter_reduce_(desc(self), dim, desc(index), desc(src), SCATTER_REDUCE.get(reduce, 9), int(include_self),
                                    p, n, _stream(stream)))


def _desc_list(tensors):
    ds = [desc(t) for t in tensors]            # kept alive by the returned tuple
    arr = (ctypes.POINTER(TxTensor) * max(1, len(ds)))(*[ctypes.pointer(d) for d in ds])
    return arr, ds


def tx_index_put_workspace_bytes(self, indices, values, accumulate=False):
    arr, keep = _desc_list(indices)
    return lib().tx_index_put_workspace_bytes(desc(self), arr, len(keep), desc(values), int(accumulate))


def tx_index_put_(self, indices, values, accumulate=False, ws=None, stream=None):
    arr, keep = _desc_list(indices)
    p, n = _ws(ws)
    _check(lib().tx_index_put_(desc(self), arr, len(keep), desc(values), int(accumulate), p, n, _stream(stream)))


def tx_take(out, input, index, stream=None):
    _check(lib().tx_take(desc(out), desc(input), desc(index), _stream(stream)))


def tx_searchsorted(out, sorted_sequence, values, right=False, stream=None):
    _check(lib().tx_searchsorted(desc(out), desc(sorted_sequence), desc(values), int(bool(right)), _stream(stream)))


def tx_masked_select_workspace_bytes(out, count, x, mask):
    return lib().tx_masked_select_workspace_bytes(desc(out), desc(count), desc(x), desc(mask))


def tx_masked_select(out, count, x, mask, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().tx_masked_select(desc(out), desc(count), desc(x), desc(mask), p, n, _stream(stream)))


def tx_nonzero_workspace_bytes(out, count, x):
    return lib().tx_nonzero_workspace_bytes(desc(out), desc(count), desc(x))


def tx_nonzero(out, count, x, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().tx_nonzero(desc(out), desc(count), desc(x), p, n, _stream(stream)))


REDUCTION = {"none": 0, "mean": 1, "sum": 2}


def _opt(t):
    return desc(t) if t is not None else None


def tx_layer_norm(out, x, norm_ndim, weight=None, bias=None, eps=1e-5, stream=None):
    _check(lib().tx_layer_norm(desc(out), desc(x), norm_ndim, _opt(weight), _opt(bias), float(eps), _stream(stream)))


def tx_binary_cross_entropy_workspace_bytes(out, input, target, weight=None, reduction="mean"):
    return lib().tx_binary_cross_entropy_workspace_bytes(desc(out), desc(input), desc(target), _opt(weight),
                                                         REDUCTION.get(reduction, 9))


def tx_binary_cross_entropy(out, input, target, weight=None, reduction="mean", ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().tx_binary_cross_entropy(desc(out), desc(input), desc(target), _opt(weight), REDUCTION.get(reduction, 9),
                                         p, n, _stream(stream)))


LOSS = {"mse": 0, "l1": 1, "smooth_l1": 2, "huber": 3}


def tx_loss_workspace_bytes(kind, out, input, target, reduction="mean", param=1.0):
    return lib().tx_loss_workspace_bytes(LOSS.get(kind, 9), desc(out), desc(input), desc(target), REDUCTION.get(reduction, 9),
                                         float(param))


def tx_loss(kind, out, input, target, reduction="mean", param=1.0, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().tx_loss(LOSS.get(kind, 9), desc(out), desc(input), desc(target), REDUCTION.get(reduction, 9), float(param),
                         p, n, _stream(stream)))


def tx_where(out, cond, x, y, stream=None):
    _check(lib().tx_where(desc(out), desc(cond), desc(x), desc(y), _stream(stream)))


def tx_masked_fill(out, self, mask, value, stream=None):
    vf, vi, isint = _scalar(value)
    _check(lib().tx_masked_fill(desc(out), desc(self), desc(mask), vf, vi, isint, _stream(stream)))


def tx_reduce(op, out, x, dims=None, keepdim=False, correction=1.0, ws=None, stream=None):
    arr, n = _dims(dims)
    wp, wb = _ws(ws)
    _check(lib().tx_reduce(REDUCE[op], desc(out), desc(x), arr, n, int(keepdim), float(correction), wp, wb,
                           _stream(stream)))


def tx_reduce_static(op, out, x, dims=None, keepdim=False, correction=1.0, stream=None):
    arr, n = _dims(dims)
    _check(lib().tx_reduce_static(REDUCE[op], desc(out), desc(x), arr, n, int(keepdim), float(correction), _stream(stream)))


def tx_reduce_workspace_bytes(op, out, x, dims=None, keepdim=False):
    arr, n = _dims(dims)
    return lib().tx_reduce_workspace_bytes(REDUCE[op], desc(out), desc(x), arr, n, int(keepdim))


def tx_softmax(out, x, dim=-1, log=False, stream=None):
    _check(lib().tx_softmax(desc(out), desc(x), dim, int(log), _stream(stream)))


def tx_cumsum(out, x, dim=-1, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().tx_cumsum(desc(out), desc(x), dim, wp, wb, _stream(stream)))


def tx_cumsum_workspace_bytes(out, x, dim=-1):
    return lib().tx_cumsum_workspace_bytes(desc(out), desc(x), dim)


SCAN = {"cumsum": 0, "cumprod": 1, "logcumsumexp": 2}


def tx_scan(op, out, x, dim=-1, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().tx_scan(SCAN.get(op, 9), desc(out), desc(x), dim, wp, wb, _stream(stream)))


def tx_scan_workspace_bytes(op, out, x, dim=-1):
    return lib().tx_scan_workspace_bytes(SCAN.get(op, 9), desc(out), desc(x), dim)


def tx_gather(out, src, dim, index, stream=None):
    _check(lib().tx_gather(desc(out), desc(src), dim, desc(index), _stream(stream)))


def tx_index_select(out, src, dim, index, stream=None):
    _check(lib().tx_index_select(desc(out), desc(src), dim, desc(index), _stream(stream)))


def tx_scatter_add_(self, dim, index, src, deterministic=True, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(lib().tx_scatter_add_(desc(self), dim, desc(index), desc(src), int(deterministic), wp, wb,
                                 _stream(stream)))


def tx_scatter_add_workspace_bytes(self, dim, index, src, deterministic=True):
    return lib().tx_scatter_add_workspace_bytes(desc(self), dim, desc(index), desc(src), int(deterministic))


def tx_infer_binary(op, a, b):
    dt, nd = ctypes.c_int32(), ctypes.c_int32()
    sizes = (ctypes.c_int64 * MAX_DIMS)()
    _check(lib().tx_infer_binary(BINARY[op], desc(a), desc(b), ctypes.byref(dt), ctypes.byref(nd), sizes))
    return CODE_DTYPE[dt.value], tuple(sizes[i] for i in range(nd.value))


def tx_infer_where(x, y):
    dt = ctypes.c_int32()
    _check(lib().tx_infer_where(desc(x), desc(y), ctypes.byref(dt)))
    return CODE_DTYPE[dt.value]


def tx_infer_unary_dtype(op, dtype):
    rc = lib().tx_infer_unary_dtype(UNARY[op], DTYPE_CODE[dtype])
    _check(rc)
    return CODE_DTYPE[rc]


UNARY_PARAM = {"leaky_relu": 0, "elu": 1, "celu": 2, "selu": 3, "softplus": 4, "threshold": 5, "hardshrink": 6, "softshrink": 7,
               "logit": 8, "nan_to_num": 9, "round_decimals": 10, "gelu_tanh": 11}
TERNARY = {"addcmul": 0, "addcdiv": 1, "lerp": 2}


def tx_infer_unary_param_dtype(op, dtype):
    rc = lib().tx_infer_unary_param_dtype(UNARY_PARAM.get(op, 99), DTYPE_CODE[dtype])
    _check(rc)
    return CODE_DTYPE[rc]


def tx_unary_param(op, out, a, p0=0.0, p1=0.0, p2=0.0, stream=None):
    _check(lib().tx_unary_param(UNARY_PARAM.get(op, 99), desc(out), desc(a), float(p0), float(p1), float(p2), _stream(stream)))


def tx_infer_ternary_dtype(op, a, b, c=None):
    rc = lib().tx_infer_ternary_dtype(TERNARY.get(op, 99), desc(a), desc(b), _opt(c))
    _check(rc)
    return CODE_DTYPE[rc]


def tx_ternary(op, out, a, b, c=None, value=1, stream=None):
    vf, vi, isint = _scalar(value)
    _check(lib().tx_ternary(TERNARY.get(op, 99), desc(out), desc(a), desc(b), _opt(c), vf, vi, isint, _stream(stream)))


def _i64_list(values):
    values = list(values)
    return (ctypes.c_int64 * max(1, len(values)))(*values), len(values)


def tx_copy(out, x, stream=None):
    _check(lib().tx_copy(desc(out), desc(x), _stream(stream)))


def tx_flip(out, x, dims, stream=None):
    d, n = _i64_list(dims)
    _check(lib().tx_flip(desc(out), desc(x), d, n, _stream(stream)))


def tx_roll(out, x, shifts, dims, stream=None):
    d, n = _i64_list(dims)
    sh, m = _i64_list(shifts)
    if n != m:
        raise ValueError("roll: one shift per dim")
    _check(lib().tx_roll(desc(out), desc(x), sh, d, n, _stream(stream)))


def tx_tri(out, x, diagonal=0, upper=False, stream=None):
    _check(lib().tx_tri(desc(out), desc(x), diagonal, int(bool(upper)), _stream(stream)))


def tx_infer_reduce(op, x, dims=None, keepdim=False):
    arr, n = _dims(dims)
    dt, nd = ctypes.c_int32(), ctypes.c_int32()
    sizes = (ctypes.c_int64 * MAX_DIMS)()
    _check(lib().tx_infer_reduce(REDUCE[op], desc(x), arr, n, int(keepdim), ctypes.byref(dt), ctypes.byref(nd), sizes))
    return CODE_DTYPE[dt.value], tuple(sizes[i] for i in range(nd.value))


def tx_last_path():
    return lib().tx_last_path().decode()


def tx_set_index_validation(on):
    lib().tx_set_index_validation(int(bool(on)))


def tx_get_index_validation():
    return bool(lib().tx_get_index_validation())


def tx_lookback_status(ws, stream=None):
    """Raises TxError(LAUNCH) if a look-back wait gave up in the last call that used `ws`; synchronises the stream."""
    _check(lib().tx_lookback_status(ctypes.c_void_p(ws.data_ptr()), _stream(stream)))


def tx_force_path(name):
    lib().tx_force_path((name or "").encode())


def workspace(nbytes, device="cuda"):
    """A device scratch buffer (plain torch allocation) of at least nbytes, 256-byte granular."""
    n = max(256, (int(nbytes) + 255) // 256 * 256)
    return torch.empty(n, dtype=torch.uint8, device=device)
