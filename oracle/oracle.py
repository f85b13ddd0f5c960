"""ctypes front end of the CPU oracle (test infrastructure only).

Takes torch CPU tensors (torch is used purely as a typed host buffer that can
hold bf16 / fp16), describes them to liboracle.so and returns new CPU tensors.
Nothing in the product imports this module.
"""
import ctypes
import os

import torch

from . import build as _build

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

ERRORS = {-1: "null", -2: "ndim", -3: "dtype", -4: "shape", -5: "dim", -7: "empty_reduction",
          -8: "scalar", -10: "index"}


class OracleError(Exception):
    def __init__(self, code):
        super().__init__("oracle error %d (%s)" % (code, ERRORS.get(code, "?")))
        self.code = code
        self.kind = ERRORS.get(code, "?")


class OrcTensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("dtype", ctypes.c_int32), ("ndim", ctypes.c_int32),
                ("sizes", ctypes.c_int64 * MAX_DIMS), ("strides", ctypes.c_int64 * MAX_DIMS)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = os.environ.get("ORACLE_LIB") or _build.LIB      # ORACLE_LIB: another build of oracle.cpp (the sanitizer test's)
        if not os.path.exists(path):
            _build.build()
        _lib = ctypes.CDLL(path)
        P = ctypes.POINTER(OrcTensor)
        I64P = ctypes.POINTER(ctypes.c_int64)
        I32P = ctypes.POINTER(ctypes.c_int32)
        _lib.orc_unary.argtypes = [ctypes.c_int, P, P]
        _lib.orc_binary.argtypes = [ctypes.c_int, P, P, P, ctypes.c_double, ctypes.c_int64, ctypes.c_int]
        _lib.orc_where.argtypes = [P, P, P, P]
        _lib.orc_clamp.argtypes = [P, P, ctypes.c_int, ctypes.c_double, ctypes.c_int64, ctypes.c_int,
                                   ctypes.c_int, ctypes.c_double, ctypes.c_int64, ctypes.c_int]
        _lib.orc_clamp_result_dtype.argtypes = [ctypes.c_int] * 5
        _lib.orc_masked_fill.argtypes = [P, P, P, ctypes.c_double, ctypes.c_int64, ctypes.c_int]
        _lib.orc_reduce.argtypes = [ctypes.c_int, P, P, I64P, ctypes.c_int32, ctypes.c_int, ctypes.c_double]
        _lib.orc_softmax.argtypes = [P, P, ctypes.c_int64, ctypes.c_int]
        _lib.orc_cumsum.argtypes = [P, P, ctypes.c_int64]
        _lib.orc_layer_norm.argtypes = [P, P, ctypes.c_int32, P, P, ctypes.c_double]
        _lib.orc_bce.argtypes = [P, P, P, P, ctypes.c_int]
        _lib.orc_copy.argtypes = [P, P]
        _lib.orc_flip_roll.argtypes = [ctypes.c_int, P, P, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64), ctypes.c_int32]
        _lib.orc_tri.argtypes = [P, P, ctypes.c_int64, ctypes.c_int]
        _lib.orc_unary_param.argtypes = [ctypes.c_int, P, P, ctypes.c_double, ctypes.c_double, ctypes.c_double]
        _lib.orc_ternary_result_dtype.argtypes = [ctypes.c_int, P, P, P]
        _lib.orc_ternary.argtypes = [ctypes.c_int, P, P, P, P, ctypes.c_double, ctypes.c_int64, ctypes.c_int]
        _lib.orc_scan.argtypes = [ctypes.c_int, P, P, ctypes.c_int64]
        _lib.orc_loss.argtypes = [ctypes.c_int, P, P, P, ctypes.c_int, ctypes.c_double]
        _lib.orc_gather.argtypes = [P, P, ctypes.c_int64, P]
        _lib.orc_index_select.argtypes = [P, P, ctypes.c_int64, P]
        _lib.orc_scatter_add.argtypes = [P, ctypes.c_int64, P, P]
        _lib.orc_index_add.argtypes = [P, ctypes.c_int64, P, P, ctypes.c_double, ctypes.c_int64, ctypes.c_int]
        _lib.orc_take.argtypes = [P, P, P]
        _lib.orc_searchsorted.argtypes = [P, P, P, ctypes.c_int]
        _lib.orc_scatter_reduce.argtypes = [P, ctypes.c_int64, P, P, ctypes.c_int, ctypes.c_int]
        _lib.orc_index_put.argtypes = [P, ctypes.POINTER(P), ctypes.c_int32, P, ctypes.c_int]
        _lib.orc_masked_select.argtypes = [P, P, P, I64P]
        _lib.orc_nonzero.argtypes = [P, P, I64P]
        _lib.orc_infer_binary.argtypes = [ctypes.c_int, P, P, I32P, I32P, I64P]
        _lib.orc_infer_reduce.argtypes = [ctypes.c_int, P, I64P, ctypes.c_int32, ctypes.c_int, I32P, I32P, I64P]
        _lib.orc_unary_result_dtype.argtypes = [ctypes.c_int, ctypes.c_int]
        _lib.orc_where_result_dtype.argtypes = [P, P]
        _lib.orc_reduce_result_dtype.argtypes = [ctypes.c_int, ctypes.c_int]
        _lib.orc_encode.argtypes = [ctypes.c_double, ctypes.c_int]
        _lib.orc_encode.restype = ctypes.c_uint32
        _lib.orc_decode.argtypes = [ctypes.c_uint32, ctypes.c_int]
        _lib.orc_decode.restype = ctypes.c_double
    return _lib


def desc(t):
    assert t.device.type == "cpu", "the oracle works on host memory"
    d = OrcTensor()
    d.data = t.data_ptr()
    d.dtype = DTYPE_CODE[t.dtype]
    d.ndim = t.dim()
    for i in range(t.dim()):
        d.sizes[i] = t.size(i)
        d.strides[i] = t.stride(i)
    return d


def _check(rc):
    if rc != 0:
        raise OracleError(rc)


def _scalar(v):
    """(double, int64, is_int) triple for a Python scalar."""
    if isinstance(v, bool):
        return float(v), int(v), 1
    if isinstance(v, int):
        return float(v), v, 1
    return float(v), 0, 0


def num_threads():
    return lib().orc_num_threads()


def set_num_threads(n):
    """Thread count of later calls (timing control only: one accumulation is never split across threads)."""
    lib().orc_set_num_threads(int(n))


# --------------------------------------------------------------------------- inference
def infer_binary(op, a, b):
    dt, nd = ctypes.c_int32(), ctypes.c_int32()
    sizes = (ctypes.c_int64 * MAX_DIMS)()
    _check(lib().orc_infer_binary(BINARY[op], desc(a), desc(b), ctypes.byref(dt), ctypes.byref(nd), sizes))
    return CODE_DTYPE[dt.value], tuple(sizes[i] for i in range(nd.value))


def infer_reduce(op, x, dims=None, keepdim=False):
    dims = _dims(dims)
    arr = (ctypes.c_int64 * max(1, len(dims)))(*dims)
    dt, nd = ctypes.c_int32(), ctypes.c_int32()
    sizes = (ctypes.c_int64 * MAX_DIMS)()
    _check(lib().orc_infer_reduce(REDUCE[op], desc(x), arr, len(dims), int(keepdim), ctypes.byref(dt),
                                  ctypes.byref(nd), sizes))
    return CODE_DTYPE[dt.value], tuple(sizes[i] for i in range(nd.value))


def unary_result_dtype(op, dtype):
    rc = lib().orc_unary_result_dtype(UNARY[op], DTYPE_CODE[dtype])
    _check(min(rc, 0))
    return CODE_DTYPE[rc]


def where_result_dtype(x, y):
    return CODE_DTYPE[lib().orc_where_result_dtype(desc(x), desc(y))]


# --------------------------------------------------------------------------- elementwise
def unary(op, a, out=None, out_dtype=None):
    if out is None:
        out = torch.empty(a.shape, dtype=out_dtype or unary_result_dtype(op, a.dtype))
    _check(lib().orc_unary(UNARY[op], desc(out), desc(a)))
    return out


def binary(op, a, b, alpha=1, out=None, out_dtype=None):
    if out is None:
        dt, shape = infer_binary(op, a, b)
        out = torch.empty(shape, dtype=out_dtype or dt)
    af, ai, isint = _scalar(alpha)
    _check(lib().orc_binary(BINARY[op], desc(out), desc(a), desc(b), af, ai, isint))
    return out


UNARY_PARAM = {"leaky_relu": 0, "elu": 1, "celu": 2, "selu": 3, "softplus": 4, "threshold": 5, "hardshrink": 6, "softshrink": 7,
               "logit": 8, "nan_to_num": 9, "round_decimals": 10, "gelu_tanh": 11}
TERNARY = {"addcmul": 0, "addcdiv": 1, "lerp": 2}


def unary_param(op, a, p0=0.0, p1=0.0, p2=0.0, out=None):
    if out is None:
        rc = lib().orc_unary_param_result_dtype(UNARY_PARAM.get(op, 99), DTYPE_CODE[a.dtype])
        _check(min(rc, 0))
        out = torch.empty(a.shape, dtype=CODE_DTYPE[rc])
    _check(lib().orc_unary_param(UNARY_PARAM.get(op, 99), desc(out), desc(a), float(p0), float(p1), float(p2)))
    return out


def ternary(op, a, b, c=None, value=1, out=None):
    if out is None:
        rc = lib().orc_ternary_result_dtype(TERNARY.get(op, 99), desc(a), desc(b), _opt(c))
        _check(min(rc, 0))
        ts = [a, b] + ([c] if c is not None else [])
        try:
            shape = torch.broadcast_shapes(*[t.shape for t in ts])
        except RuntimeError:                          # not broadcastable: the oracle reports it
            shape = a.shape
        out = torch.empty(shape, dtype=CODE_DTYPE[rc])
    vf, vi, isint = _scalar(value)
    _check(lib().orc_ternary(TERNARY.get(op, 99), desc(out), desc(a), desc(b), _opt(c), vf, vi, isint))
    return out


def copy(x, out=None, dtype=None, shape=None):
    """x broadcast to `shape` (default: its own) and converted to `dtype` (default: its own), or into `out`."""
    if out is None:
        out = torch.empty(x.shape if shape is None else shape, dtype=dtype or x.dtype)
    _check(lib().orc_copy(desc(out), desc(x)))
    return out


def _i64(values):
    values = list(values)
    return (ctypes.c_int64 * max(1, len(values)))(*values), len(values)


def flip(x, dims, out=None):
    out = torch.empty(x.shape, dtype=x.dtype) if out is None else out
    d, n = _i64(dims)
    _check(lib().orc_flip_roll(0, desc(out), desc(x), d, d, n))
    return out


def roll(x, shifts, dims, out=None):
    out = torch.empty(x.shape, dtype=x.dtype) if out is None else out
    d, n = _i64(dims)
    sh, m = _i64(shifts)
    if n != m:
        raise OracleError(-4)
    _check(lib().orc_flip_roll(1, desc(out), desc(x), d, sh, n))
    return out


def tril(x, diagonal=0, out=None):
    out = torch.empty(x.shape, dtype=x.dtype) if out is None else out
    _check(lib().orc_tri(desc(out), desc(x), diagonal, 0))
    return out


def triu(x, diagonal=0, out=None):
    out = torch.empty(x.shape, dtype=x.dtype) if out is None else out
    _check(lib().orc_tri(desc(out), desc(x), diagonal, 1))
    return out


def clamp(x, lo=None, hi=None, out=None, out_dtype=None):
    lf, li, lint = _scalar(0 if lo is None else lo)
    hf, hi_i, hint = _scalar(0 if hi is None else hi)
    if out is None:
        rc = lib().orc_clamp_result_dtype(DTYPE_CODE[x.dtype], lo is not None, lint, hi is not None, hint)
        _check(min(rc, 0))
        out = torch.empty(x.shape, dtype=out_dtype or CODE_DTYPE[rc])
    _check(lib().orc_clamp(desc(out), desc(x), lo is not None, lf, li, lint, hi is not None, hf, hi_i, hint))
    return out


def where(cond, x, y, out=None):
    if out is None:
        shape = torch.broadcast_shapes(cond.shape, x.shape, y.shape)
        out = torch.empty(shape, dtype=where_result_dtype(x, y))
    _check(lib().orc_where(desc(out), desc(cond), desc(x), desc(y)))
    return out


def masked_fill(self, mask, value, out=None):
    if out is None:
        out = torch.empty(torch.broadcast_shapes(self.shape, mask.shape), dtype=self.dtype)
    vf, vi, isint = _scalar(value)
    _check(lib().orc_masked_fill(desc(out), desc(self), desc(mask), vf, vi, isint))
    return out


# --------------------------------------------------------------------------- reductions
def _dims(dims):
    if dims is None:
        return []
    if isinstance(dims, int):
        return [dims]
    return list(dims)


def reduce(op, x, dims=None, keepdim=False, correction=1.0, out=None, out_dtype=None):
    dl = _dims(dims)
    if out is None:
        dt, shape = infer_reduce(op, x, dl, keepdim)
        out = torch.empty(shape, dtype=out_dtype or dt)
    arr = (ctypes.c_int64 * max(1, len(dl)))(*dl)
    _check(lib().orc_reduce(REDUCE[op], desc(out), desc(x), arr, len(dl), int(keepdim), float(correction)))
    return out


def softmax(x, dim=-1, log=False, out=None, out_dtype=None):
    if out is None:
        out = torch.empty(x.shape, dtype=out_dtype or x.dtype)
    _check(lib().orc_softmax(desc(out), desc(x), dim, int(log)))
    return out


REDUCTION = {"none": 0, "mean": 1, "sum": 2}


def _opt(t):
    return desc(t) if t is not None else None


def layer_norm(x, norm_ndim, weight=None, bias=None, eps=1e-5, out=None):
    if out is None:
        out = torch.empty(x.shape, dtype=x.dtype)
    _check(lib().orc_layer_norm(desc(out), desc(x), norm_ndim, _opt(weight), _opt(bias), float(eps)))
    return out


def binary_cross_entropy(x, target, weight=None, reduction="mean", out=None):
    if out is None:
        out = torch.empty(x.shape if reduction == "none" else (), dtype=x.dtype)
    _check(lib().orc_bce(desc(out), desc(x), desc(target), _opt(weight), REDUCTION.get(reduction, 9)))
    return out


LOSS = {"mse": 0, "l1": 1, "smooth_l1": 2, "huber": 3}


def loss(kind, x, target, reduction="mean", param=1.0, out=None):
    if out is None:
        out = torch.empty(torch.broadcast_shapes(x.shape, target.shape) if reduction == "none" else (), dtype=x.dtype)
    _check(lib().orc_loss(LOSS.get(kind, 9), desc(out), desc(x), desc(target), REDUCTION.get(reduction, 9), ctypes.c_double(param)))
    return out


def cumsum(x, dim=-1, out=None, out_dtype=None):
    if out is None:
        dt = x.dtype if x.dtype.is_floating_point else torch.int64
        out = torch.empty(x.shape, dtype=out_dtype or dt)
    _check(lib().orc_cumsum(desc(out), desc(x), dim))
    return out


SCAN = {"cumsum": 0, "cumprod": 1, "logcumsumexp": 2}


def scan(op, x, dim=-1, out=None, out_dtype=None):
    if out is None:
        dt = x.dtype if x.dtype.is_floating_point else torch.int64
        out = torch.empty(x.shape, dtype=out_dtype or dt)
    _check(lib().orc_scan(SCAN.get(op, 9), desc(out), desc(x), dim))
    return out


# --------------------------------------------------------------------------- indexing
def gather(src, dim, index, out=None):
    if out is None:
        out = torch.empty(index.shape, dtype=src.dtype)
    _check(lib().orc_gather(desc(out), desc(src), dim, desc(index)))
    return out


def index_select(src, dim, index, out=None):
    if out is None:
        if src.dim() == 0:
            shape = ()
        else:
            shape = list(src.shape)
            if not -src.dim() <= dim < src.dim():
                raise OracleError(-5)
            shape[dim] = index.numel()
        out = torch.empty(shape, dtype=src.dtype)
    _check(lib().orc_index_select(desc(out), desc(src), dim, desc(index)))
    return out


def scatter_add_(self, dim, index, src):
    _check(lib().orc_scatter_add(desc(self), dim, desc(index), desc(src)))
    return self


def index_add_(self, dim, index, source, alpha=1):
    af, ai, isint = _scalar(alpha)
    _check(lib().orc_index_add(desc(self), dim, desc(index), desc(source), af, ai, isint))
    return self


SCATTER_REDUCE = {"sum": 0, "prod": 1, "mean": 2, "amax": 3, "amin": 4}


def scatter_reduce_(self, dim, index, src, reduce, include_self=True):
    _check(lib().orc_scatter_reduce(desc(self), dim, desc(index), desc(src), SCATTER_REDUCE.get(reduce, 9), int(include_self)))
    return self


def index_put_(self, indices, values, accumulate=False):
    ds = [desc(i) for i in indices]
    arr = (ctypes.POINTER(OrcTensor) * max(1, len(ds)))(*[ctypes.pointer(d) for d in ds])
    _check(lib().orc_index_put(desc(self), arr, len(ds), desc(values), int(accumulate)))
    return self


def searchsorted(sorted_sequence, values, right=False, out_int32=False):
    out = torch.empty(values.shape, dtype=torch.int32 if out_int32 else torch.int64)
    _check(lib().orc_searchsorted(desc(out), desc(sorted_sequence), desc(values), int(bool(right))))
    return out


def take(input, index, out=None):
    if out is None:
        out = torch.empty(index.shape, dtype=input.dtype)
    _check(lib().orc_take(desc(out), desc(input), desc(index)))
    return out


def masked_select(x, mask):
    cap = 1
    try:
        for s in torch.broadcast_shapes(x.shape, mask.shape):
            cap *= s
    except RuntimeError:
        pass                      # not broadcastable: the oracle call below reports it
    out = torch.empty((cap,), dtype=x.dtype)
    n = ctypes.c_int64()
    _check(lib().orc_masked_select(desc(out), desc(x), desc(mask), ctypes.byref(n)))
    return out[:n.value]


def nonzero(x):
    out = torch.empty((x.numel(), x.dim()), dtype=torch.int64)
    n = ctypes.c_int64()
    _check(lib().orc_nonzero(desc(out), desc(x), ctypes.byref(n)))
    return out[:n.value]


# --------------------------------------------------------------------------- codec hooks
def encode(v, dtype):
    return lib().orc_encode(float(v), DTYPE_CODE[dtype])


def decode(bits, dtype):
    return lib().orc_decode(int(bits), DTYPE_CODE[dtype])
