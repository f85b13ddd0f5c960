"""Drive an operator backend through PyTorch's OpInfo sample generators.

The paper's acceptance criterion (Section 3.3) is that an operator passes every OpInfo sample for every dtype it
supports, "passing" meaning agreement with the ATen CPU operator within a dtype-dependent tolerance (Section 3.2).
This module reproduces that loop for the operators of this library: the sample generators and the reference
operator are the ones that ship inside the installed torch package (used as a test DRIVER: nothing of the suite is
copied here), the backend under test is either the HIP library (GPU tests) or the CPU oracle (CPU tests, which
pins the oracle to the ATen CPU operators on the same samples).

A sample is "unsupported" when it asks for something outside the library's C ABI (a dtype other than the six,
a dtype= / out= keyword, tensor-valued clamp bounds, rounding modes, ...); those are counted and reported, never
silently passed.
"""
import sys
import types
import unittest

import torch

F32, BF16, F16, I32, I64, BOOL = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool
DTYPES = (F32, BF16, F16, I32, I64, BOOL)
# |got - want| <= atol + rtol * |want| against the ATen CPU result (itself computed in fp32 for the half types)
TOL = {F32: (1e-5, 2e-5), BF16: (1.6e-2, 1e-2), F16: (2e-3, 2e-3)}


class Unsupported(Exception):
    pass


def load_op_db():
    """name -> list of OpInfo.  The internal test package needs `expecttest` (absent here: stubbed) and probes the
    GPU's architecture name at import (patched for the import when there is no GPU)."""
    if "expecttest" not in sys.modules:
        try:
            import expecttest  # noqa: F401
        except ImportError:
            stub = types.ModuleType("expecttest")
            stub.TestCase = type("TestCase", (unittest.TestCase,), {})
            sys.modules["expecttest"] = stub
    saved = None
    if not torch.cuda.is_available():
        saved = torch.cuda.get_device_properties
        props = types.SimpleNamespace(gcnArchName="gfx950", major=9, minor=5, multi_processor_count=256,
                                      total_memory=1 << 38, name="none")
        torch.cuda.get_device_properties = lambda *a, **k: props
    try:
        from torch.testing._internal.common_methods_invocations import op_db
    finally:
        if saved is not None:
            torch.cuda.get_device_properties = saved
    db = {}
    for op in op_db:
        db.setdefault(op.name, []).append(op)
    return db


# --------------------------------------------------------------------------- backends
class OracleBackend:
    """The CPU oracle, called on the samples as they are."""
    name = "oracle"

    def __init__(self):
        from oracle import oracle as O
        self.O = O
        self.refused = (O.OracleError,)

    def unary(self, op, x):
        return self.O.unary(op, x)

    def binary(self, op, a, b, alpha=1):
        return self.O.binary(op, a, b, alpha=alpha)

    def clamp(self, x, lo, hi):
        return self.O.clamp(x, lo, hi)

    def where(self, c, x, y):
        return self.O.where(c, x, y)

    def masked_fill(self, x, m, v):
        return self.O.masked_fill(x, m, v)

    def reduce(self, op, x, dims, keepdim, correction=1.0):
        return self.O.reduce(op, x, dims, keepdim, correction)

    def softmax(self, x, dim, log):
        return self.O.softmax(x, dim, log)

    def cumsum(self, x, dim):
        return self.O.cumsum(x, dim)

    def scan(self, op, x, dim):
        return self.O.scan(op, x, dim)

    def unary_param(self, op, x, *params):
        return self.O.unary_param(op, x, *params)

    def copy(self, x, dtype=None, out=None):
        return self.O.copy(x, dtype=dtype, out=out)

    def remap(self, op, x, *args):
        return getattr(self.O, op)(x, *args)

    def empty(self, shape, dtype):
        return torch.empty(shape, dtype=dtype)

    def host(self, t):
        return t

    def ternary(self, op, a, b, c, value):
        return self.O.ternary(op, a, b, c, value)

    def gather(self, x, dim, index):
        return self.O.gather(x, dim, index)

    def index_select(self, x, dim, index):
        return self.O.index_select(x, dim, index)

    def scatter_add(self, x, dim, index, src):
        return self.O.scatter_add_(x.clone(), dim, index, src)

    def index_add(self, x, dim, index, src, alpha):
        return self.O.index_add_(x.clone(), dim, index, src, alpha)

    def scatter_reduce(self, x, dim, index, src, reduce, include_self):
        return self.O.scatter_reduce_(x.clone(), dim, index, src, reduce, include_self)

    def index_put(self, x, indices, values, accumulate):
        return self.O.index_put_(x.clone(), indices, values, accumulate)

    def take(self, x, index):
        return self.O.take(x, index)

    def searchsorted(self, seq, values, right, out_int32):
        return self.O.searchsorted(seq, values, right, out_int32)

    def masked_select(self, x, m):
        return self.O.masked_select(x, m)

    def nonzero(self, x):
        return self.O.nonzero(x)

    def layer_norm(self, x, k, w, b, eps):
        return self.O.layer_norm(x, k, w, b, eps)

    def bce(self, x, t, w, reduction):
        return self.O.binary_cross_entropy(x, t, w, reduction)

    def loss(self, kind, x, t, reduction, param):
        return self.O.loss(kind, x, t, reduction, param)


class LibraryBackend:
    """The HIP library: operands copied to the GPU with their strides, outputs allocated from the library's own
    inference functions, every call through the C ABI binding."""
    name = "library"

    def __init__(self):
        from paper_2512_10977_amd import binding as B
        from tests.parity import to_device_view
        self.B = B
        self.dev = to_device_view
        self.refused = (B.TxError,)

    def _out(self, shape, dtype):
        return torch.empty(tuple(shape), dtype=dtype, device="cuda")

    def _ws(self, nbytes):
        return self.B.workspace(nbytes) if nbytes else None

    def unary(self, op, x):
        out = self._out(x.shape, self.B.tx_infer_unary_dtype(op, x.dtype))
        self.B.tx_unary(op, out, self.dev(x))
        return out.cpu()

    def binary(self, op, a, b, alpha=1):
        da, db = self.dev(a), self.dev(b)
        dt, shape = self.B.tx_infer_binary(op, da, db)
        out = self._out(shape, dt)
        if op == "add":
            self.B.tx_add(out, da, db, alpha)
        elif op == "sub":
            self.B.tx_sub(out, da, db, alpha)
        else:
            self.B.tx_binary(op, out, da, db)
        return out.cpu()

    def clamp(self, x, lo, hi):
        out = self._out(x.shape, self.B.tx_infer_clamp_dtype(x.dtype, lo, hi))
        self.B.tx_clamp(out, self.dev(x), lo, hi)
        return out.cpu()

    def where(self, c, x, y):
        dx, dy = self.dev(x), self.dev(y)
        out = self._out(torch.broadcast_shapes(c.shape, x.shape, y.shape), self.B.tx_infer_where(dx, dy))
        self.B.tx_where(out, self.dev(c), dx, dy)
        return out.cpu()

    def masked_fill(self, x, m, v):
        out = self._out(torch.broadcast_shapes(x.shape, m.shape), x.dtype)
        self.B.tx_masked_fill(out, self.dev(x), self.dev(m), v)
        return out.cpu()

    def reduce(self, op, x, dims, keepdim, correction=1.0):
        dx = self.dev(x)
        dt, shape = self.B.tx_infer_reduce(op, dx, dims, keepdim)
        out = self._out(shape, dt)
        ws = self._ws(self.B.tx_reduce_workspace_bytes(op, out, dx, dims, keepdim))
        self.B.tx_reduce(op, out, dx, dims, keepdim, correction, ws)
        return out.cpu()

    def softmax(self, x, dim, log):
        out = self._out(x.shape, x.dtype)
        self.B.tx_softmax(out, self.dev(x), dim, log)
        return out.cpu()

    def cumsum(self, x, dim):
        dx = self.dev(x)
        out = self._out(x.shape, x.dtype if x.dtype.is_floating_point else I64)
        self.B.tx_cumsum(out, dx, dim, self._ws(self.B.tx_cumsum_workspace_bytes(out, dx, dim)))
        return out.cpu()

    def copy(self, x, dtype=None, out=None):
        if out is None:
            out = self._out(x.shape, dtype or x.dtype)
        self.B.tx_copy(out, self.dev(x) if x.device.type == "cpu" else x)
        return out.cpu() if out.device.type != "cpu" and not getattr(out, "_keep", False) else out

    def remap(self, op, x, *args):
        out = self._out(x.shape, x.dtype)
        if op == "flip":
            self.B.tx_flip(out, self.dev(x), *args)
        elif op == "roll":
            self.B.tx_roll(out, self.dev(x), *args)
        else:
            self.B.tx_tri(out, self.dev(x), args[0], op == "triu")
        return out.cpu()

    def empty(self, shape, dtype):
        return self._out(shape, dtype)

    def host(self, t):
        return t.cpu()

    def unary_param(self, op, x, *params):
        out = self._out(x.shape, self.B.tx_infer_unary_param_dtype(op, x.dtype))
        self.B.tx_unary_param(op, out, self.dev(x), *params)
        return out.cpu()

    def ternary(self, op, a, b, c, value):
        da, db, dc = self.dev(a), self.dev(b), None if c is None else self.dev(c)
        shape = torch.broadcast_shapes(*[t.shape for t in (a, b, c) if t is not None])
        out = self._out(shape, self.B.tx_infer_ternary_dtype(op, da, db, dc))
        self.B.tx_ternary(op, out, da, db, dc, value)
        return out.cpu()

    def scan(self, op, x, dim):
        dx = self.dev(x)
        out = self._out(x.shape, x.dtype if x.dtype.is_floating_point else I64)
        self.B.tx_scan(op, out, dx, dim, self._ws(self.B.tx_scan_workspace_bytes(op, out, dx, dim)))
        return out.cpu()

    def gather(self, x, dim, index):
        out = self._out(index.shape, x.dtype)
        self.B.tx_gather(out, self.dev(x), dim, self.dev(index))
        return out.cpu()

    def index_select(self, x, dim, index):
        shape = list(x.shape)
        if x.dim():
            shape[dim] = index.numel()
        out = self._out(shape, x.dtype)
        self.B.tx_index_select(out, self.dev(x), dim, self.dev(index))
        return out.cpu()

    def scatter_add(self, x, dim, index, src):
        dst, di, ds = x.contiguous().cuda(), self.dev(index), self.dev(src)
        self.B.tx_scatter_add_(dst, dim, di, ds, True, self._ws(self.B.tx_scatter_add_workspace_bytes(dst, dim, di, ds, True)))
        return dst.cpu()

    def index_add(self, x, dim, index, src, alpha):
        dst, di, ds = x.contiguous().cuda(), self.dev(index), self.dev(src)
        self.B.tx_index_add_(dst, dim, di, ds, alpha, True, self._ws(self.B.tx_index_add_workspace_bytes(dst, dim, di, ds, True)))
        return dst.cpu()

    def scatter_reduce(self, x, dim, index, src, reduce, include_self):
        dst, di, ds = x.contiguous().cuda(), self.dev(index), self.dev(src)
        ws = self._ws(self.B.tx_scatter_reduce_workspace_bytes(dst, dim, di, ds, reduce, include_self))
        self.B.tx_scatter_reduce_(dst, dim, di, ds, reduce, include_self, ws)
        return dst.cpu()

    def index_put(self, x, indices, values, accumulate):
        dst, di, dv = x.contiguous().cuda(), [self.dev(i) for i in indices], self.dev(values)
        self.B.tx_index_put_(dst, di, dv, accumulate, self._ws(self.B.tx_index_put_workspace_bytes(dst, di, dv, accumulate)))
        return dst.cpu()

    def take(self, x, index):
        out = self._out(index.shape, x.dtype)
        self.B.tx_take(out, self.dev(x), self.dev(index))
        return out.cpu()

    def searchsorted(self, seq, values, right, out_int32):
        out = self._out(values.shape, I32 if out_int32 else I64)
        self.B.tx_searchsorted(out, self.dev(seq), self.dev(values), right)
        return out.cpu()

    def _select(self, out, nbytes, call):
        count = torch.zeros((1,), dtype=I64, device="cuda")
        call(out, count, self.B.workspace(nbytes(out, count)))
        return out[: int(count.item())].cpu()

    def masked_select(self, x, m):
        dx, dm = self.dev(x), self.dev(m)
        cap = 1
        for s in torch.broadcast_shapes(x.shape, m.shape):
            cap *= s
        return self._select(self._out((cap,), x.dtype), lambda o, c: self.B.tx_masked_select_workspace_bytes(o, c, dx, dm),
                            lambda o, c, ws: self.B.tx_masked_select(o, c, dx, dm, ws))

    def nonzero(self, x):
        dx = self.dev(x)
        return self._select(self._out((x.numel(), x.dim()), I64), lambda o, c: self.B.tx_nonzero_workspace_bytes(o, c, dx),
                            lambda o, c, ws: self.B.tx_nonzero(o, c, dx, ws))

    def layer_norm(self, x, k, w, b, eps):
        out = self._out(x.shape, x.dtype)
        self.B.tx_layer_norm(out, self.dev(x), k, None if w is None else self.dev(w), None if b is None else self.dev(b), eps)
        return out.cpu()

    def bce(self, x, t, w, reduction):
        dx, dt_, dw = self.dev(x), self.dev(t), None if w is None else self.dev(w)
        out = self._out(x.shape if reduction == "none" else (), x.dtype)
        ws = self._ws(self.B.tx_binary_cross_entropy_workspace_bytes(out, dx, dt_, dw, reduction))
        self.B.tx_binary_cross_entropy(out, dx, dt_, dw, reduction, ws)
        return out.cpu()

    def loss(self, kind, x, t, reduction, param):
        dx, dt_ = self.dev(x), self.dev(t)
        out = self._out(torch.broadcast_shapes(x.shape, t.shape) if reduction == "none" else (), x.dtype)
        ws = self._ws(self.B.tx_loss_workspace_bytes(kind, out, dx, dt_, reduction, param))
        self.B.tx_loss(kind, out, dx, dt_, reduction, param, ws)
        return out.cpu()


# --------------------------------------------------------------------------- sample -> backend call
def _tensor_ok(t):
    if t.dtype not in DTYPES:
        raise Unsupported("dtype %s" % t.dtype)
    if any(s < 0 for s in t.stride()):
        raise Unsupported("negative stride")
    return t


def _operand(v):
    """A tensor operand, or a Python scalar as the 0-dim tensor ATen's promotion treats it like."""
    if isinstance(v, torch.Tensor):
        return _tensor_ok(v)
    if isinstance(v, (bool, int, float)):
        return torch.tensor(v)
    raise Unsupported("operand %r" % type(v))


def _no_kwargs(s, allowed=()):
    extra = set(s.kwargs) - set(allowed)
    if extra:
        raise Unsupported("keyword %s" % sorted(extra))


def _scalar(v):
    if isinstance(v, torch.Tensor):
        if v.dim() != 0:
            raise Unsupported("tensor-valued scalar argument")
        return v.item()
    if v is None or isinstance(v, (bool, int, float)):
        return v
    raise Unsupported("scalar %r" % type(v))


def unary(name):
    def run(be, s):
        _no_kwargs(s)
        if s.args:
            raise Unsupported("positional arguments")
        return be.unary(name, _tensor_ok(s.input))
    return run


def gelu(be, s):
    _no_kwargs(s, ("approximate",))
    if s.args:
        raise Unsupported("arguments")
    if s.kwargs.get("approximate", "none") == "tanh":
        return be.unary_param("gelu_tanh", _tensor_ok(s.input))
    return be.unary("gelu", _tensor_ok(s.input))


def binary(name, alpha_ok=False):
    def run(be, s):
        _no_kwargs(s, ("alpha",) if alpha_ok else ())
        if len(s.args) != 1:
            raise Unsupported("arguments")
        return be.binary(name, _operand(s.input), _operand(s.args[0]), _scalar(s.kwargs.get("alpha", 1)))
    return run


def div(be, s):
    _no_kwargs(s, ("rounding_mode",))
    if len(s.args) != 1:
        raise Unsupported("arguments")
    op = {None: "div", "floor": "floor_divide", "trunc": "trunc_divide"}[s.kwargs.get("rounding_mode")]
    return be.binary(op, _operand(s.input), _operand(s.args[0]))


def searchsorted(bucketize):
    def run(be, s):
        _no_kwargs(s, ("right", "out_int32", "side", "sorter"))
        if s.kwargs.get("sorter") is not None:
            raise Unsupported("sorter")
        seq, values = (s.args[0], s.input) if bucketize else (s.input, s.args[0])
        if not isinstance(values, torch.Tensor):
            raise Unsupported("scalar value")
        right = bool(s.kwargs.get("right", False)) or s.kwargs.get("side") == "right"
        return be.searchsorted(_tensor_ok(seq), _tensor_ok(values), right, bool(s.kwargs.get("out_int32", False)))
    return run


def clamp(be, s):
    bounds = dict(zip(("min", "max"), s.args))
    bounds.update(s.kwargs)
    _no_kwargs(types.SimpleNamespace(kwargs=bounds), ("min", "max"))
    lo, hi = bounds.get("min"), bounds.get("max")
    x = _tensor_ok(s.input)
    if any(isinstance(b, torch.Tensor) and b.dim() > 0 for b in (lo, hi)):
        # tensor-valued bounds are outside the clamp entry point (scalar bounds); the same function is
        # min(max(x, lo), hi) on the broadcasting binary entry point
        r = x
        if lo is not None:
            r = be.binary("maximum", r, _operand(lo))
        if hi is not None:
            r = be.binary("minimum", r, _operand(hi))
        return r
    return be.clamp(x, _scalar(lo), _scalar(hi))


def where(be, s):
    _no_kwargs(s)
    return be.where(_tensor_ok(s.args[0]), _operand(s.input), _operand(s.args[1]))


def masked_fill(be, s):
    _no_kwargs(s)
    return be.masked_fill(_tensor_ok(s.input), _tensor_ok(s.args[0]), _scalar(s.args[1]))


def _convert_first(be, x, dtype):
    if dtype not in DTYPES:
        raise Unsupported("dtype %s" % dtype)
    return x if dtype == x.dtype else be.copy(x, dtype=dtype)


def reduction(name, variance=False, index=False):
    def run(be, s):
        kw = dict(s.kwargs)
        args = list(s.args)
        x = _tensor_ok(s.input)
        correction = 1.0
        if variance:
            if args and isinstance(args[0], bool):                   # var(x, unbiased)
                correction = 1.0 if args.pop(0) else 0.0
            if "unbiased" in kw:
                correction = 1.0 if kw.pop("unbiased") else 0.0
            if "correction" in kw:
                c = kw.pop("correction")
                correction = 1.0 if c is None else float(c)
        if args:
            kw["dim"] = args.pop(0)
        if args:
            kw["keepdim"] = args.pop(0)
            if variance and isinstance(kw["keepdim"], bool) and args:
                raise Unsupported("arguments")
        if variance and args:
            raise Unsupported("arguments")
        want_dtype = kw.pop("dtype", None)
        if want_dtype is not None:                                   # dtype=: the input is converted first
            x = _convert_first(be, x, want_dtype)
        if set(kw) - {"dim", "keepdim"}:
            raise Unsupported("keyword %s" % sorted(set(kw) - {"dim", "keepdim"}))
        dim = kw.get("dim")
        if isinstance(dim, (list, tuple)):
            dim = list(dim)
            if index and len(dim) != 1:
                raise Unsupported("several dims")
        r = be.reduce(name, x, dim, bool(kw.get("keepdim", False)), correction)
        # an integer dtype= narrower than the int64 accumulator: wrapping arithmetic commutes with the narrowing
        return r if want_dtype is None or r.dtype == want_dtype else be.copy(r, dtype=want_dtype)
    return run


def softmax(log):
    def run(be, s):
        _no_kwargs(s)
        return be.softmax(_tensor_ok(s.input), s.args[0], log)
    return run


def cumsum(be, s):
    _no_kwargs(s)
    return be.cumsum(_tensor_ok(s.input), s.args[0])


def scan(op):
    def run(be, s):
        _no_kwargs(s, ("dtype",))
        if len(s.args) != 1:
            raise Unsupported("arguments")
        x = _tensor_ok(s.input)
        want_dtype = s.kwargs.get("dtype")
        if want_dtype is not None:
            x = _convert_first(be, x, want_dtype)
        r = be.scan(op, x, s.args[0])
        return r if want_dtype is None or r.dtype == want_dtype else be.copy(r, dtype=want_dtype)
    return run


def gather(be, s):
    _no_kwargs(s)
    return be.gather(_tensor_ok(s.input), s.args[0], _tensor_ok(s.args[1]))


def index_select(be, s):
    _no_kwargs(s)
    return be.index_select(_tensor_ok(s.input), s.args[0], _tensor_ok(s.args[1]))


def scatter_add(be, s):
    _no_kwargs(s)
    return be.scatter_add(_tensor_ok(s.input), s.args[0], _tensor_ok(s.args[1]), _tensor_ok(s.args[2]))


def index_add(be, s):
    _no_kwargs(s, ("alpha",))
    return be.index_add(_tensor_ok(s.input), s.args[0], _tensor_ok(s.args[1]), _tensor_ok(s.args[2]), _scalar(s.kwargs.get("alpha", 1)))


def scatter_reduce(be, s):
    _no_kwargs(s, ("include_self",))
    return be.scatter_reduce(_tensor_ok(s.input), s.args[0], _tensor_ok(s.args[1]), _tensor_ok(s.args[2]), s.args[3],
                             bool(s.kwargs.get("include_self", True)))


def index_put(be, s):
    _no_kwargs(s, ("accumulate",))
    indices = [_tensor_ok(i) for i in s.args[0]]
    if any(i.dtype == BOOL for i in indices):
        raise Unsupported("bool mask as index")
    accumulate = bool(s.kwargs.get("accumulate", False))
    if not accumulate:
        flat = torch.stack([i.reshape(-1) % n for i, n in zip(torch.broadcast_tensors(*indices), s.input.shape)], 1)
        if len(torch.unique(flat, dim=0)) != len(flat):
            raise Unsupported("assignment with repeated destinations (no unique result)")
    return be.index_put(_tensor_ok(s.input), indices, _tensor_ok(s.args[1]), accumulate)


def take(be, s):
    _no_kwargs(s)
    return be.take(_tensor_ok(s.input), _tensor_ok(s.args[0]))


# Indexing operators that are another entry point seen through a view (a descriptor with permuted, sliced or flattened
# sizes and strides): the view is built on the host, the data movement is the library's.
def _front(t, dim):
    return t.movedim(dim, 0) if t.dim() else t


def index_copy(be, s):
    _no_kwargs(s)
    x, dim, index, src = _tensor_ok(s.input), s.args[0], _tensor_ok(s.args[1]), _tensor_ok(s.args[2])
    if index.numel() != len(torch.unique(index)):
        raise Unsupported("assignment with repeated destinations (no unique result)")
    if x.dim() == 0:
        return be.index_put(x.reshape(1), [index.reshape(-1)], src.reshape(-1), False).reshape(())
    r = be.index_put(_front(x, dim), [index.reshape(-1)], _front(src, dim), False)
    return r.movedim(0, dim)


def index_fill(be, s):
    _no_kwargs(s)
    x, dim, index, value = _tensor_ok(s.input), s.args[0], _tensor_ok(s.args[1]), s.args[2]
    v = value.to(x.dtype) if isinstance(value, torch.Tensor) else torch.tensor(value, dtype=x.dtype)
    if v.dim():
        raise Unsupported("tensor-valued fill")
    if x.dim() == 0:
        return be.index_put(x.reshape(1), [index.reshape(-1)], v, False).reshape(())
    return be.index_put(_front(x, dim), [index.reshape(-1)], v, False).movedim(0, dim)


def take_along_dim(be, s):
    _no_kwargs(s, ("dim",))
    x, idx = _tensor_ok(s.input), _tensor_ok(s.args[0])
    dim = s.args[1] if len(s.args) > 1 else s.kwargs.get("dim")
    n = x.numel() if dim is None else x.shape[dim]
    if idx.numel() and int(idx.min()) < 0:                            # negative indices count from the end: remainder by the extent
        idx = be.binary("remainder", idx, torch.tensor(n, dtype=idx.dtype), 1)
    if dim is None:
        return be.gather(x.reshape(-1), 0, idx.reshape(-1))
    d = dim if dim >= 0 else dim + x.dim()
    xs, is_ = list(x.shape), list(idx.shape)
    xs[d], is_[d] = 1, 1
    common = list(torch.broadcast_shapes(xs, is_))
    xs, is_ = list(common), list(common)
    xs[d], is_[d] = x.shape[d], idx.shape[d]
    return be.gather(x.expand(xs), d, idx.expand(is_))


def put(be, s):
    _no_kwargs(s, ("accumulate",))
    x, index, src = _tensor_ok(s.input), _tensor_ok(s.args[0]), _tensor_ok(s.args[1])
    accumulate = bool(s.args[2]) if len(s.args) > 2 else bool(s.kwargs.get("accumulate", False))
    if not accumulate and index.numel() != len(torch.unique(index % max(x.numel(), 1))):
        raise Unsupported("assignment with repeated destinations (no unique result)")
    return be.index_put(x.reshape(-1), [index.reshape(-1)], src.reshape(-1), accumulate).reshape(x.shape)


def scatter_into_view(view_of):
    """select_scatter / slice_scatter / diagonal_scatter: a copy of the input with `src` copied over one view of it."""
    def run(be, s):
        x, src = _tensor_ok(s.input), _tensor_ok(s.args[0])
        out = be.empty(x.shape, x.dtype)
        out._keep = True
        be.copy(x, out=out)
        piece = view_of(out, *s.args[1:], **s.kwargs)
        piece._keep = True
        if piece.numel():
            be.copy(src, out=piece)
        return be.host(out)
    return run


def masked_select(be, s):
    _no_kwargs(s)
    return be.masked_select(_tensor_ok(s.input), _tensor_ok(s.args[0]))


def nonzero(be, s):
    _no_kwargs(s, ("as_tuple",))
    if s.kwargs.get("as_tuple", False) or s.args:
        raise Unsupported("as_tuple")
    return be.nonzero(_tensor_ok(s.input))


def layer_norm(be, s):
    _no_kwargs(s, ("eps", "weight", "bias"))
    x = _tensor_ok(s.input)
    shape = tuple(s.args[0])
    w = s.args[1] if len(s.args) > 1 else s.kwargs.get("weight")
    b = s.args[2] if len(s.args) > 2 else s.kwargs.get("bias")
    if len(s.args) > 3:
        raise Unsupported("arguments")
    return be.layer_norm(x, len(shape), None if w is None else _tensor_ok(w), None if b is None else _tensor_ok(b),
                         float(s.kwargs.get("eps", 1e-5)))


def bce(be, s):
    _no_kwargs(s, ("weight", "reduction"))
    if len(s.args) != 1:
        raise Unsupported("arguments")
    w = s.kwargs.get("weight")
    return be.bce(_tensor_ok(s.input), _tensor_ok(s.args[0]), None if w is None else _tensor_ok(w), s.kwargs.get("reduction", "mean"))


def activation(op, names, defaults):
    """A unary operator with scalar parameters: positional arguments fill `names` in order, then keywords."""
    def run(be, s):
        _no_kwargs(s, tuple(names) + ("inplace",))
        if len(s.args) > len(names) or s.kwargs.get("inplace"):
            raise Unsupported("arguments")
        vals = dict(zip(names, defaults))
        vals.update(dict(zip(names, s.args)))
        vals.update({k: v for k, v in s.kwargs.items() if k != "inplace"})
        if any(isinstance(v, torch.Tensor) for v in vals.values()):
            raise Unsupported("tensor-valued parameter")
        return be.unary_param(op, _tensor_ok(s.input), *[_scalar(vals[n]) for n in names])
    return run


def logit(be, s):
    _no_kwargs(s, ("eps",))
    eps = s.args[0] if s.args else s.kwargs.get("eps")
    x = _tensor_ok(s.input)
    return be.unary_param("logit", x) if eps is None else be.unary_param("logit", x, float(eps), 1)


def nan_to_num(be, s):
    _no_kwargs(s, ("nan", "posinf", "neginf"))
    x = _tensor_ok(s.input)
    vals = dict(zip(("nan", "posinf", "neginf"), s.args))
    vals.update(s.kwargs)
    fi = torch.finfo(x.dtype) if x.dtype.is_floating_point else None
    nan = vals.get("nan")
    pos, neg = vals.get("posinf"), vals.get("neginf")
    return be.unary_param("nan_to_num", x, 0.0 if nan is None else float(nan), (fi.max if fi else 0.0) if pos is None else float(pos),
                          (fi.min if fi else 0.0) if neg is None else float(neg))


def hardtanh(lo, hi):
    def run(be, s):
        _no_kwargs(s, ("min_val", "max_val", "inplace"))
        vals = {"min_val": lo, "max_val": hi}
        vals.update(dict(zip(("min_val", "max_val"), s.args)))
        vals.update({k: v for k, v in s.kwargs.items() if k != "inplace"})
        x = _tensor_ok(s.input)
        bounds = [_scalar(vals["min_val"]), _scalar(vals["max_val"])]
        if not x.dtype.is_floating_point:                  # the operator keeps an integer dtype: its bounds are truncated to it
            bounds = [int(b) for b in bounds]
        return be.clamp(x, *bounds)
    return run


def ternary(op):
    def run(be, s):
        _no_kwargs(s, ("value",))
        if len(s.args) != 2:
            raise Unsupported("arguments")
        return be.ternary(op, _tensor_ok(s.input), _tensor_ok(s.args[0]), _tensor_ok(s.args[1]), _scalar(s.kwargs.get("value", 1)))
    return run


def lerp(be, s):
    _no_kwargs(s)
    a, b, w = _tensor_ok(s.input), _tensor_ok(s.args[0]), s.args[1]
    if isinstance(w, torch.Tensor):
        return be.ternary("lerp", a, b, _tensor_ok(w), 1)
    return be.ternary("lerp", a, b, None, _scalar(w))


def round_(be, s):
    _no_kwargs(s, ("decimals",))
    if s.args:
        raise Unsupported("arguments")
    x = _tensor_ok(s.input)
    if "decimals" in s.kwargs:
        return be.unary_param("round_decimals", x, int(s.kwargs["decimals"]))
    return be.unary("round", x)


def clone(be, s):
    _no_kwargs(s)
    if s.args:
        raise Unsupported("arguments")
    return be.copy(_tensor_ok(s.input))


def flip(dims=None):
    def run(be, s):
        _no_kwargs(s, ("dims",))
        d = dims if dims is not None else (s.args[0] if s.args else s.kwargs["dims"])
        return be.remap("flip", _tensor_ok(s.input), list(d))
    return run


def roll(be, s):
    kw = dict(zip(("shifts", "dims"), s.args))
    kw.update(s.kwargs)
    _no_kwargs(types.SimpleNamespace(kwargs=kw), ("shifts", "dims"))
    if kw.get("dims") is None:
        raise Unsupported("roll of the flattened tensor")
    sh, d = kw["shifts"], kw["dims"]
    return be.remap("roll", _tensor_ok(s.input), [sh] if isinstance(sh, int) else list(sh), [d] if isinstance(d, int) else list(d))


def tri(op):
    def run(be, s):
        _no_kwargs(s, ("diagonal",))
        k = s.args[0] if s.args else s.kwargs.get("diagonal", 0)
        return be.remap(op, _tensor_ok(s.input), int(k))
    return run


def concatenate(stack):
    """cat / stack: the result is allocated and every input is copied into its slice of it (the slices are views,
    descriptors with other offsets and strides), converting to the promoted dtype on the way."""
    def run(be, s):
        _no_kwargs(s, ("dim",))
        tensors = [_tensor_ok(t) for t in s.input]
        dim = s.args[0] if s.args else s.kwargs.get("dim", 0)
        if stack:
            tensors = [t.unsqueeze(dim if dim >= 0 else dim + t.dim() + 1) for t in tensors]
        if not stack and any(t.dim() == 1 and t.numel() == 0 for t in tensors) and any(t.dim() > 1 for t in tensors):
            raise Unsupported("legacy empty operand")
        nd = tensors[0].dim()
        dim = dim if dim >= 0 else dim + nd
        shape = list(tensors[0].shape)
        shape[dim] = sum(t.shape[dim] for t in tensors)
        dtype = tensors[0].dtype
        for t in tensors[1:]:
            dtype = torch.promote_types(dtype, t.dtype)
        if dtype not in DTYPES:
            raise Unsupported("dtype %s" % dtype)
        out = be.empty(shape, dtype)
        at = 0
        for t in tensors:
            piece = out.narrow(dim, at, t.shape[dim])
            piece._keep = True
            if t.numel():
                be.copy(t, out=piece)
            at += t.shape[dim]
        return be.host(out)
    return run


def view_then_copy(be, s, op):
    """A view operator: the view is a descriptor (sizes, strides, offset) that the caller builds - here ATen builds
    it on the host - and the library's part is materialising it with tx_copy."""
    v = op.op(_tensor_ok(s.input), *s.args, **s.kwargs)
    if not isinstance(v, torch.Tensor):
        raise Unsupported("not a single tensor")
    return be.copy(_tensor_ok(v))


VIEW_OPS = ("expand", "expand_as", "broadcast_to", "permute", "transpose", "t", "movedim", "narrow", "select", "squeeze", "unsqueeze",
            "flatten", "reshape", "view", "diagonal", "unfold", "as_strided", "T", "mT")


def vector_norm(be, s):
    kw = dict(s.kwargs)
    args = list(s.args)
    order = args.pop(0) if args else kw.pop("ord", 2)
    if args:
        kw["dim"] = args.pop(0)
    if args:
        kw["keepdim"] = args.pop(0)
    if args or set(kw) - {"dim", "keepdim"}:
        raise Unsupported("keyword %s" % sorted(set(kw) - {"dim", "keepdim"}))
    dim = kw.get("dim")
    if isinstance(dim, (list, tuple)):
        dim = list(dim)
    return be.reduce("norm", _tensor_ok(s.input), dim, bool(kw.get("keepdim", False)), float(order))


def regression_loss(kind, param_name=None):
    def run(be, s):
        _no_kwargs(s, ("reduction",) + ((param_name,) if param_name else ()))
        if len(s.args) != 1:
            raise Unsupported("arguments")
        x, t = _tensor_ok(s.input), _tensor_ok(s.args[0])
        if x.dtype != t.dtype:
            raise Unsupported("input and target of different dtypes")
        return be.loss(kind, x, t, s.kwargs.get("reduction", "mean"), float(s.kwargs.get(param_name, 1.0)) if param_name else 1.0)
    return run


# OpInfo name -> (variant names to take, adapter)
ADAPTERS = {
    "neg": unary("neg"), "abs": unary("abs"), "exp": unary("exp"), "log": unary("log"), "sqrt": unary("sqrt"),
    "sigmoid": unary("sigmoid"), "tanh": unary("tanh"), "log1p": unary("log1p"), "expm1": unary("expm1"),
    "logical_not": unary("logical_not"), "nn.functional.logsigmoid": unary("logsigmoid"), "nn.functional.gelu": gelu,
    "sin": unary("sin"), "cos": unary("cos"), "exp2": unary("exp2"), "log2": unary("log2"), "log10": unary("log10"),
    "rsqrt": unary("rsqrt"), "reciprocal": unary("reciprocal"), "nn.functional.silu": unary("silu"), "square": unary("square"),
    "sign": unary("sign"), "floor": unary("floor"), "ceil": unary("ceil"), "trunc": unary("trunc"), "round": round_,
    "isnan": unary("isnan"), "isinf": unary("isinf"), "isfinite": unary("isfinite"), "bitwise_not": unary("bitwise_not"),
    "bitwise_and": binary("bitwise_and"), "bitwise_or": binary("bitwise_or"), "bitwise_xor": binary("bitwise_xor"),
    "atan2": binary("atan2"),
    "tan": unary("tan"), "asin": unary("asin"), "acos": unary("acos"), "atan": unary("atan"), "sinh": unary("sinh"),
    "cosh": unary("cosh"), "asinh": unary("asinh"), "acosh": unary("acosh"), "atanh": unary("atanh"), "erf": unary("erf"),
    "erfc": unary("erfc"), "frac": unary("frac"), "signbit": unary("signbit"), "nn.functional.relu": unary("relu"),
    "nn.functional.hardswish": unary("hardswish"), "nn.functional.hardsigmoid": unary("hardsigmoid"),
    "nn.functional.mish": unary("mish"),
    "fmod": binary("fmod"), "remainder": binary("remainder"), "hypot": binary("hypot"), "copysign": binary("copysign"),
    "logaddexp": binary("logaddexp"), "logaddexp2": binary("logaddexp2"), "xlogy": binary("xlogy"),
    "heaviside": binary("heaviside"), "fmax": binary("fmax"), "fmin": binary("fmin"), "nextafter": binary("nextafter"),
    "floor_divide": binary("floor_divide"), "div": div, "searchsorted": searchsorted(False), "bucketize": searchsorted(True),
    "gcd": binary("gcd"), "lcm": binary("lcm"), "bitwise_left_shift": binary("bitwise_left_shift"),
    "bitwise_right_shift": binary("bitwise_right_shift"),
    "add": binary("add", True), "sub": binary("sub", True), "mul": binary("mul"), "true_divide": binary("div"),
    "maximum": binary("maximum"), "minimum": binary("minimum"), "eq": binary("eq"), "ne": binary("ne"), "lt": binary("lt"),
    "le": binary("le"), "gt": binary("gt"), "ge": binary("ge"), "logical_and": binary("logical_and"),
    "logical_or": binary("logical_or"), "logical_xor": binary("logical_xor"), "pow": binary("pow"),
    "clamp": clamp, "where": where, "masked_fill": masked_fill,
    "sum": reduction("sum"), "mean": reduction("mean"), "amax": reduction("amax"), "amin": reduction("amin"),
    "argmax": reduction("argmax", index=True), "argmin": reduction("argmin", index=True), "prod": reduction("prod", index=True),
    "var": reduction("var", variance=True), "std": reduction("std", variance=True), "any": reduction("any"),
    "all": reduction("all"), "logsumexp": reduction("logsumexp"),
    "nansum": reduction("nansum"), "nanmean": reduction("nanmean"), "count_nonzero": reduction("count_nonzero"),
    "linalg.vector_norm": vector_norm,
    "softmax": softmax(False), "log_softmax": softmax(True), "cumsum": scan("cumsum"), "cumprod": scan("cumprod"),
    "logcumsumexp": scan("logcumsumexp"),
    "gather": gather, "index_select": index_select, "scatter_add": scatter_add, "index_add": index_add, "take": take,
    "masked_select": masked_select, "nonzero": nonzero, "scatter_reduce": scatter_reduce, "index_put": index_put,
    "nn.functional.layer_norm": layer_norm, "nn.functional.binary_cross_entropy": bce,
    "nn.functional.leaky_relu": activation("leaky_relu", ("negative_slope",), (0.01,)),
    "nn.functional.elu": activation("elu", ("alpha",), (1.0,)), "nn.functional.celu": activation("celu", ("alpha",), (1.0,)),
    "nn.functional.selu": activation("selu", (), ()), "nn.functional.softplus": activation("softplus", ("beta", "threshold"), (1.0, 20.0)),
    "nn.functional.threshold": activation("threshold", ("threshold", "value"), (None, None)),
    "nn.functional.hardshrink": activation("hardshrink", ("lambd",), (0.5,)),
    "nn.functional.softshrink": activation("softshrink", ("lambd",), (0.5,)), "logit": logit, "nan_to_num": nan_to_num,
    "nn.functional.hardtanh": hardtanh(-1.0, 1.0), "nn.functional.relu6": hardtanh(0.0, 6.0),
    "addcmul": ternary("addcmul"), "addcdiv": ternary("addcdiv"), "lerp": lerp,
    "index_copy": index_copy, "index_fill": index_fill, "take_along_dim": take_along_dim, "put": put,
    "select_scatter": scatter_into_view(lambda o, dim, index: o.select(dim, index)),
    "slice_scatter": scatter_into_view(lambda o, dim=0, start=None, end=None, step=1: o[(slice(None),) * (dim % max(o.dim(), 1)) + (slice(start, end, step),)]),
    "diagonal_scatter": scatter_into_view(lambda o, offset=0, dim1=0, dim2=1: o.diagonal(offset, dim1, dim2)),
    "clone": clone, "contiguous": clone, "flip": flip(), "fliplr": flip([1]), "flipud": flip([0]), "roll": roll,
    "tril": tri("tril"), "triu": tri("triu"), "cat": concatenate(False), "stack": concatenate(True),
    "nn.functional.mse_loss": regression_loss("mse"), "nn.functional.l1_loss": regression_loss("l1"),
    "nn.functional.smooth_l1_loss": regression_loss("smooth_l1", "beta"), "nn.functional.huber_loss": regression_loss("huber", "delta"),
}


ADAPTERS.update({name: view_then_copy for name in VIEW_OPS})


# --------------------------------------------------------------------------- operators that are other entry points
# Operators ATen itself defines through other operators (reflected arithmetic, one-sided clamps, unit conversions,
# conversions, copies of views, stacking, splitting, ...): each adapter spells the operator out over the library's
# entry points, and the result is compared with ATen's own operator.
def reflected(name):
    def run(be, s):
        _no_kwargs(s)
        if len(s.args) != 1:
            raise Unsupported("arguments")
        return be.binary(name, _operand(s.args[0]), _operand(s.input))
    return run


def rsub(be, s):
    _no_kwargs(s, ("alpha",))
    return be.binary("sub", _operand(s.args[0]), _operand(s.input), _scalar(s.kwargs.get("alpha", 1)))


def one_sided_clamp(op):
    def run(be, s):
        _no_kwargs(s)
        bound, x = s.args[0], _tensor_ok(s.input)
        if (isinstance(bound, torch.Tensor) and bound.dim() > 0) or x.dtype == torch.bool:
            return be.binary(op, x, _operand(bound))             # (the clamp entry point takes no bool tensor)
        return be.clamp(x, *((_scalar(bound), None) if op == "maximum" else (None, _scalar(bound))))
    return run


def times_constant(c):
    def run(be, s):
        _no_kwargs(s)
        return be.binary("mul", _tensor_ok(s.input), torch.tensor(c))
    return run


def equals_constant(c):
    def run(be, s):
        _no_kwargs(s)
        x = _tensor_ok(s.input)
        if x.dtype == torch.bool:
            raise Unsupported("bool input")
        return be.binary("eq", x, torch.tensor(c))
    return run


def fill_like(value_at, default=None):
    """fill / full_like / zeros_like / ones_like: masked_fill under a mask that is true everywhere."""
    def run(be, s):
        kw = dict(s.kwargs)
        want_dtype = kw.pop("dtype", None)
        args = list(s.args)
        if value_at is not None and "value" in kw:
            args.insert(value_at, kw.pop("value"))
        for k in ("memory_format", "layout", "pin_memory", "requires_grad"):
            kw.pop(k, None)
        if kw:
            raise Unsupported("keyword %s" % sorted(kw))
        x = _tensor_ok(s.input)
        v = _scalar(args[value_at]) if value_at is not None else default
        if want_dtype is not None and want_dtype != x.dtype:
            if want_dtype not in DTYPES:
                raise Unsupported("dtype %s" % want_dtype)
            x = be.copy(x, dtype=want_dtype)
        return be.masked_fill(x, torch.ones((), dtype=torch.bool), v)
    return run


def softmin(be, s):
    _no_kwargs(s, ("dtype",))
    x = _tensor_ok(s.input)
    if s.kwargs.get("dtype") is not None:
        x = _convert_first(be, x, s.kwargs["dtype"])
    return be.softmax(be.unary("neg", x), s.args[0], False)


def softsign(be, s):
    _no_kwargs(s)
    x = _tensor_ok(s.input)
    return be.binary("div", x, be.binary("add", be.unary("abs", x), torch.tensor(1)))


def tanhshrink(be, s):
    _no_kwargs(s)
    x = _tensor_ok(s.input)
    return be.binary("sub", x, be.unary("tanh", x))


def copy_of_view(view):
    def run(be, s):
        x = _tensor_ok(s.input)
        v = x if view == "alias" else getattr(torch.Tensor, view)(x, *s.args, **s.kwargs)
        return be.copy(_tensor_ok(v))
    return run


def convert_to(dtype):
    def run(be, s):
        _no_kwargs(s, ("memory_format",))
        return be.copy(_tensor_ok(s.input), dtype=dtype)
    return run


def several(*adapters_and_filters):
    """An operator with several results: one adapter per result, each seeing the same sample."""
    def run(be, s):
        return tuple(a(be, s) for a in adapters_and_filters)
    return run


def _with_kwargs(s, **changes):
    kw = dict(s.kwargs)
    for k, v in changes.items():
        if v is _DROP:
            kw.pop(k, None)
        else:
            kw[k] = v
    return types.SimpleNamespace(input=s.input, args=s.args, kwargs=kw)


_DROP = object()


def aminmax(be, s):
    _no_kwargs(s, ("dim", "keepdim"))
    if s.args:
        raise Unsupported("arguments")
    x = _tensor_ok(s.input)
    dim, keep = s.kwargs.get("dim"), bool(s.kwargs.get("keepdim", False))
    return be.reduce("amin", x, dim, keep), be.reduce("amax", x, dim, keep)


def extremum(value_op, index_op, binary_op):
    """max / min: with another tensor the elementwise operator; with a dim the pair (values, indices); alone the
    extremum of everything."""
    def run(be, s):
        x = _tensor_ok(s.input)
        if s.args and isinstance(s.args[0], torch.Tensor):
            _no_kwargs(s)
            return be.binary(binary_op, x, _operand(s.args[0]))
        args, kw = list(s.args), dict(s.kwargs)
        if args:
            kw["dim"] = args.pop(0)
        if args:
            kw["keepdim"] = args.pop(0)
        if args or set(kw) - {"dim", "keepdim"}:
            raise Unsupported("arguments")
        if "dim" not in kw:
            return be.reduce(value_op, x, None, False)
        if x.dtype == torch.bool:
            raise Unsupported("bool input with a dim")            # no argmax / argmin of bool in ATen or here
        keep = bool(kw.get("keepdim", False))
        return be.reduce(value_op, x, kw["dim"], keep), be.reduce(index_op, x, kw["dim"], keep)
    return run


def moments(name):
    """std_mean / var_mean: the pair (spread, mean) from two reductions."""
    spread = reduction(name, variance=True)
    mean = reduction("mean")

    def run(be, s):
        args = [a for a in s.args]
        kw = dict(s.kwargs)
        if args and isinstance(args[0], bool):                       # (x, unbiased)
            mean_s = types.SimpleNamespace(input=s.input, args=(), kwargs={})
        else:
            mkw = {k: v for k, v in kw.items() if k in ("dim", "keepdim")}
            mean_s = types.SimpleNamespace(input=s.input, args=tuple(args[:2]), kwargs=mkw)
            if len(args) > 2:
                raise Unsupported("arguments")
        return spread(be, s), mean(be, mean_s)
    return run


def repeat(tile):
    """repeat / tile: a copy of the view that reads every source element r times over (stride 0 along the new
    dims), reshaped on the host."""
    def run(be, s):
        _no_kwargs(s)
        x = _tensor_ok(s.input)
        reps = list(s.args[0]) if len(s.args) == 1 and isinstance(s.args[0], (list, tuple, torch.Size)) else list(s.args)
        if tile and len(reps) < x.dim():
            reps = [1] * (x.dim() - len(reps)) + reps
        if len(reps) < x.dim():
            raise Unsupported("fewer repeats than dims")
        shape = [1] * (len(reps) - x.dim()) + list(x.shape)
        v = x.reshape(shape)
        inter, final = [], []
        for r, n in zip(reps, shape):
            inter += [r, n]
            final.append(r * n)
        idx = tuple(i for n in range(len(shape)) for i in (None, slice(None)))
        v = v[idx].expand(inter)
        return be.copy(_tensor_ok(v)).reshape(final)
    return run


def rot90(be, s):
    kw = dict(zip(("k", "dims"), s.args))
    kw.update(s.kwargs)
    k, dims = kw.get("k", 1) % 4, list(kw.get("dims", (0, 1)))
    x = _tensor_ok(s.input)
    if k == 0:
        return be.copy(x)
    if k == 2:
        return be.remap("flip", x, dims)
    return be.remap("flip", x, [dims[1] if k == 1 else dims[0]]).transpose(dims[0], dims[1])


def outer(be, s):
    _no_kwargs(s)
    return be.binary("mul", _tensor_ok(s.input).unsqueeze(1), _tensor_ok(s.args[0]).unsqueeze(0))


def trace(be, s):
    _no_kwargs(s)
    return be.reduce("sum", _tensor_ok(s.input).diagonal(), None, False)


def dist(be, s):
    _no_kwargs(s)
    p = float(s.args[1]) if len(s.args) > 1 else 2.0
    d = be.binary("sub", _tensor_ok(s.input), _tensor_ok(s.args[0]))
    return be.reduce("norm", d, None, False, p)


def normalize(be, s):
    kw = dict(zip(("p", "dim", "eps"), s.args))
    kw.update(s.kwargs)
    _no_kwargs(types.SimpleNamespace(kwargs=kw), ("p", "dim", "eps"))
    x = _tensor_ok(s.input)
    n = be.reduce("norm", x, [kw.get("dim", 1)], True, float(kw.get("p", 2.0)))
    return be.binary("div", x, be.clamp(n, float(kw.get("eps", 1e-12)), None))


def ldexp(be, s):
    _no_kwargs(s)
    x, e = _operand(s.input), _operand(s.args[0])
    p = be.binary("pow", torch.tensor(2.0), e)
    # ATen's 2.0 is a scalar, which never widens a floating tensor: a 0-dim exponent keeps its own dtype
    want = e.dtype if e.dtype.is_floating_point else F32
    return be.binary("mul", x, p if p.dtype == want else be.copy(p, dtype=want))


def glu(be, s):
    _no_kwargs(s, ("dim",))
    dim = s.args[0] if s.args else s.kwargs.get("dim", -1)
    x = _tensor_ok(s.input)
    half = x.shape[dim] // 2
    return be.binary("mul", x.narrow(dim, 0, half), be.unary("sigmoid", x.narrow(dim, half, half)))


def prelu(be, s):
    _no_kwargs(s, ("weight",))
    x, w = _tensor_ok(s.input), _tensor_ok(s.args[0] if s.args else s.kwargs["weight"])
    if w.numel() != 1 and x.dim() >= 2:
        w = w.reshape([1, -1] + [1] * (x.dim() - 2))
    elif x.dim() == 0:
        w = w.reshape(())
    return be.where(be.binary("gt", x, torch.tensor(0)), x, be.binary("mul", w, x))


def rms_norm(be, s):
    kw = dict(zip(("normalized_shape", "weight", "eps"), s.args))
    kw.update(s.kwargs)
    _no_kwargs(types.SimpleNamespace(kwargs=kw), ("normalized_shape", "weight", "eps"))
    x = _tensor_ok(s.input)
    dims = list(range(x.dim() - len(kw["normalized_shape"]), x.dim()))
    eps = kw.get("eps")
    eps = torch.finfo(x.dtype).eps if eps is None else float(eps)
    xf = x if x.dtype == F32 else be.copy(x, dtype=F32)          # ATen normalises in fp32 and rounds once
    ms = be.reduce("mean", be.unary("square", xf), dims, True)
    r = be.binary("mul", xf, be.unary("rsqrt", be.binary("add", ms, torch.tensor(eps))))
    r = r if x.dtype == F32 else be.copy(r, dtype=x.dtype)
    return r if kw.get("weight") is None else be.binary("mul", r, _tensor_ok(kw["weight"]))


def diff(be, s):
    kw = dict(zip(("n", "dim", "prepend", "append"), s.args))
    kw.update(s.kwargs)
    _no_kwargs(types.SimpleNamespace(kwargs=kw), ("n", "dim", "prepend", "append"))
    x, dim = _tensor_ok(s.input), kw.get("dim", -1)
    if kw.get("n", 1) == 0:                                      # ATen hands the input back, whatever else was passed
        return be.copy(x)
    parts = [_tensor_ok(t) for t in (kw.get("prepend"), x, kw.get("append")) if t is not None]
    if len(parts) > 1:
        x = concatenate(False)(be, types.SimpleNamespace(input=parts, args=(dim,), kwargs={}))
    for _ in range(kw.get("n", 1)):
        length = x.shape[dim]
        if length == 0:
            break
        x = be.binary("logical_xor" if x.dtype == torch.bool else "sub", x.narrow(dim, 1, length - 1), x.narrow(dim, 0, length - 1))
    return x if x is not s.input else be.copy(x)


def stacked(prepare, dim_of):
    """hstack / vstack / dstack / column_stack: cat after the host has reshaped the operands."""
    cat = concatenate(False)

    def run(be, s):
        _no_kwargs(s)
        tensors = [prepare(t) for t in s.input]
        return cat(be, types.SimpleNamespace(input=tensors, args=(dim_of(tensors),), kwargs={}))
    return run


def copies_of_views(be, s, op):
    """An operator whose results are views of its inputs: each is materialised with tx_copy."""
    v = op.op(s.input, *s.args, **s.kwargs)
    if isinstance(v, torch.Tensor):
        return be.copy(_tensor_ok(v))
    return tuple(be.copy(_tensor_ok(t)) for t in v)


MULTI_VIEW_OPS = ("split", "split_with_sizes", "chunk", "unbind", "tensor_split", "hsplit", "vsplit", "dsplit", "unsafe_chunk",
                  "unsafe_split", "split_with_sizes_copy", "unbind_copy", "atleast_1d", "atleast_2d", "atleast_3d",
                  "broadcast_tensors", "meshgrid")
IDENTITY_VIEW_OPS = ("ravel", "view_as", "reshape_as", "unflatten", "H", "mH", "real", "conj", "conj_physical", "resolve_conj",
                     "resolve_neg", "positive", "squeeze_copy")

ADAPTERS.update({
    "__radd__": reflected("add"), "__rmul__": reflected("mul"), "__rsub__": reflected("sub"), "__rdiv__": reflected("div"),
    "__rmod__": reflected("remainder"), "__rpow__": reflected("pow"), "__rand__": reflected("bitwise_and"),
    "__ror__": reflected("bitwise_or"), "__rxor__": reflected("bitwise_xor"), "rsub": rsub,
    "clamp_min": one_sided_clamp("maximum"), "clamp_max": one_sided_clamp("minimum"),
    "deg2rad": times_constant(3.14159265358979323846 / 180.0), "rad2deg": times_constant(180.0 / 3.14159265358979323846),
    "isposinf": equals_constant(float("inf")), "isneginf": equals_constant(float("-inf")), "sgn": unary("sign"),
    "fill": fill_like(0), "full_like": fill_like(0), "zeros_like": fill_like(None, 0), "ones_like": fill_like(None, 1),
    "nn.functional.softmin": softmin, "nn.functional.softsign": softsign, "nn.functional.tanhshrink": tanhshrink,
    "expand_copy": copy_of_view("expand"), "permute_copy": copy_of_view("permute"), "t_copy": copy_of_view("t"),
    "transpose_copy": copy_of_view("transpose"), "view_copy": copy_of_view("view"), "unsqueeze_copy": copy_of_view("unsqueeze"),
    "diagonal_copy": copy_of_view("diagonal"), "narrow_copy": copy_of_view("narrow"), "as_strided_copy": copy_of_view("as_strided"),
    "alias_copy": copy_of_view("alias"), "unfold_copy": copy_of_view("unfold"),
    "float": convert_to(F32), "half": convert_to(F16), "bfloat16": convert_to(BF16), "int": convert_to(I32), "long": convert_to(I64),
    "bool": convert_to(torch.bool),
    "aminmax": aminmax, "max": extremum("amax", "argmax", "maximum"), "min": extremum("amin", "argmin", "minimum"),
    "std_mean": moments("std"), "var_mean": moments("var"),
    "repeat": repeat(False), "tile": repeat(True), "rot90": rot90, "outer": outer, "trace": trace, "dist": dist,
    "nn.functional.normalize": normalize, "ldexp": ldexp, "nn.functional.glu": glu, "nn.functional.prelu": prelu,
    "nn.functional.rms_norm": rms_norm, "diff": diff,
    "hstack": stacked(torch.atleast_1d, lambda ts: 0 if ts[0].dim() == 1 else 1),
    "vstack": stacked(torch.atleast_2d, lambda ts: 0), "dstack": stacked(torch.atleast_3d, lambda ts: 2),
    "column_stack": stacked(lambda t: t.reshape(t.numel(), 1) if t.dim() <= 1 else t, lambda ts: 1),
})
ADAPTERS.update({name: view_then_copy for name in IDENTITY_VIEW_OPS})
ADAPTERS.update({name: copies_of_views for name in MULTI_VIEW_OPS})


def compare(got, want):
    """None if got matches the ATen CPU result, else a short description."""
    if isinstance(want, (tuple, list)):
        if not isinstance(got, (tuple, list)) or len(got) != len(want):
            return "%r results, ATen %d" % (len(got) if isinstance(got, (tuple, list)) else type(got), len(want))
        for i, (g, w) in enumerate(zip(got, want)):
            bad = compare(g, w)
            if bad is not None:
                return "result %d: %s" % (i, bad)
        return None
    if not isinstance(want, torch.Tensor):
        return "reference returned %r" % type(want)
    if got.dtype != want.dtype:
        return "dtype %s, ATen %s" % (got.dtype, want.dtype)
    if tuple(got.shape) != tuple(want.shape):
        return "shape %s, ATen %s" % (tuple(got.shape), tuple(want.shape))
    if not want.dtype.is_floating_point:
        bad = got != want
        return None if not bad.any() else "%d of %d integer / bool elements differ" % (int(bad.sum()), bad.numel())
    rtol, atol = TOL[want.dtype]
    g, w = got.double(), want.double()
    ok = torch.where(w.isfinite() & g.isfinite(), (g - w).abs() <= atol + rtol * w.abs(), (g == w) | (g.isnan() & w.isnan()))
    if ok.all():
        return None
    i = (~ok).nonzero()[0].tolist()
    return "%d of %d outside tolerance, first at %s: %r vs ATen %r" % (int((~ok).sum()), ok.numel(), i, got[tuple(i)].item(),
                                                                     want[tuple(i)].item())


SCALAR_LOOP_REFERENCE = ("fmod", "remainder")


def _scalar_loop_reference(op, s, want):
    """ATen's vectorised fmod / remainder return NaN once |a / b| leaves their routine's range (a divisor near the
    smallest normal number does it); ATen's scalar loop, which 0-dim operands take, returns the exact remainder.  The NaN
    elements of the reference are evaluated again that way, so the reference stays ATen's CPU operator."""
    if not (isinstance(want, torch.Tensor) and want.dtype.is_floating_point and want.isnan().any()):
        return want
    a, b = torch.broadcast_tensors(torch.as_tensor(s.input), torch.as_tensor(s.args[0]))
    want = want.clone()
    for i in want.isnan().nonzero().tolist():
        want[tuple(i)] = op.op(a[tuple(i)].to(want.dtype), b[tuple(i)].to(want.dtype))
    return want


def sweep(backend, names=None, db=None):
    """Runs every OpInfo sample of every adapted operator and dtype.  Returns {op: {"samples", "supported", "passed",
    "unsupported": {reason: n}, "failures": [...]}}."""
    db = db or load_op_db()
    report = {}
    for name, adapter in ADAPTERS.items():
        if names and name not in names:
            continue
        rec = report.setdefault(name, {"samples": 0, "supported": 0, "passed": 0, "unsupported": {}, "failures": []})
        for op in db.get(name, []):
            for dt in DTYPES:
                if dt not in op.supported_dtypes("cpu"):
                    continue
                for s in op.sample_inputs("cpu", dt, requires_grad=False):
                    rec["samples"] += 1
                    label = "%s%s %s %s" % (name, "/" + op.variant_test_name if op.variant_test_name else "", dt, _describe(s))
                    try:
                        want = op.op(s.input, *s.args, **s.kwargs)
                        if name in SCALAR_LOOP_REFERENCE:
                            want = _scalar_loop_reference(op, s, want)
                    except Exception as e:                              # the reference refuses this sample itself
                        rec["unsupported"]["ATen raised"] = rec["unsupported"].get("ATen raised", 0) + 1
                        continue
                    try:
                        got = adapter(backend, s, op) if adapter in (view_then_copy, copies_of_views) else adapter(backend, s)
                    except Unsupported as e:
                        key = str(e)
                        rec["unsupported"][key] = rec["unsupported"].get(key, 0) + 1
                        continue
                    except backend.refused as e:
                        rec["supported"] += 1
                        rec["failures"].append("%s: %s refused: %s" % (label, backend.name, e))
                        continue
                    rec["supported"] += 1
                    bad = compare(got, want)
                    if bad is None:
                        rec["passed"] += 1
                    else:
                        rec["failures"].append("%s: %s" % (label, bad))
    return report


def _describe(s):
    def d(v):
        if isinstance(v, torch.Tensor):
            return "T%s%s" % (list(v.shape), "" if v.is_contiguous() else "nc")
        if isinstance(v, (list, tuple)):
            return "(" + ",".join(d(x) for x in v) + ")"
        return repr(v)
    return "%s %s %s" % (d(s.input), [d(a) for a in s.args], {k: d(v) for k, v in s.kwargs.items()})


def summarise(report):
    lines = ["%-36s %8s %10s %8s  %s" % ("operator", "samples", "supported", "passed", "unsupported (reason: count)")]
    for name, r in sorted(report.items()):
        lines.append("%-36s %8d %10d %8d  %s" % (name, r["samples"], r["supported"], r["passed"],
                                               "; ".join("%s: %d" % kv for kv in sorted(r["unsupported"].items()))))
    return "\n".join(lines)


def check(report):
    """Assertion helper for the tests: every supported sample passed, and every operator had supported samples."""
    problems = []
    for name, r in sorted(report.items()):
        if r["supported"] == 0:
            problems.append("%s: no supported sample out of %d" % (name, r["samples"]))
        problems.extend(r["failures"])
    assert not problems, "%d problems\n%s\n\n%s" % (len(problems), "\n".join(p[:400] for p in problems[:40]), summarise(report))


if __name__ == "__main__":
    import warnings
    warnings.filterwarnings("ignore")
    which = sys.argv[1] if len(sys.argv) > 1 else "oracle"
    rep = sweep(LibraryBackend() if which == "library" else OracleBackend())
    print(summarise(rep))
    tot = [sum(r[k] for r in rep.values()) for k in ("samples", "supported", "passed")]
    print("total: %d samples, %d supported, %d passed, %d operators" % (tot[0], tot[1], tot[2], len(rep)))
    for r in rep.values():
        for f in r["failures"]:
            print("FAIL", f[:400])
