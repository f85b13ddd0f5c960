"""GPU parity: index_add_, take, masked_select, nonzero (HIP library through the C ABI) vs. the CPU oracle.

index_add_ on floating dtypes is held to rel 1e-5 (fp32) / 1e-2 (half) of max(|oracle|, scale) with scale the root
of the sum of squares of everything that lands on an element; everything else is bit-exact.
"""
import itertools

import pytest
import torch

from oracle import oracle as O
from paper_2512_10977_amd import binding as B
from paper_2512_10977_amd import inputs as I
from tests.parity import assert_exact, assert_rel, to_device_view

pytestmark = pytest.mark.gpu
F32, BF16, F16, I32, I64, BOOL = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool
ALL = [F32, BF16, F16, I32, I64, BOOL]


def index_add_scale(self_cpu, dim, idx_cpu, src_cpu, alpha):
    s2 = self_cpu.double() ** 2
    s2.index_add_(dim, idx_cpu.long().reshape(-1), (src_cpu.double() * float(alpha)) ** 2)
    return s2.sqrt()


def check_index_add(self_cpu, dim, idx_cpu, src_cpu, alpha=1, deterministic=True, what=""):
    want = O.index_add_(self_cpu.clone(), dim, idx_cpu, src_cpu, alpha)
    dst = to_device_view(self_cpu).clone() if self_cpu.is_contiguous() else to_device_view(self_cpu)
    idx, src = to_device_view(idx_cpu), to_device_view(src_cpu)
    nbytes = B.tx_index_add_workspace_bytes(dst, dim, idx, src, deterministic)
    ws = B.workspace(nbytes) if nbytes else None
    B.tx_index_add_(dst, dim, idx, src, alpha, deterministic, ws)
    used = B.tx_last_path()
    torch.cuda.synchronize()
    what = "index_add %s self%s n=%d dim=%d alpha=%r %s [%s]" % (self_cpu.dtype, tuple(self_cpu.shape), idx_cpu.numel(), dim,
                                                               alpha, what, used)
    if not self_cpu.dtype.is_floating_point:
        assert_exact(dst, want, what)
    else:
        assert_rel(dst, want, 1e-5 if self_cpu.dtype == F32 else 1e-2, index_add_scale(self_cpu, dim, idx_cpu, src_cpu, alpha), what)
    return used


def test_index_add_sweep():
    g = torch.Generator().manual_seed(400)
    for dt in (F32, BF16, F16, I32, I64):
        for shape, dim, n in [((50, 64), 0, 300), ((50, 64), 1, 40), ((6, 20, 48), 1, 77), ((6, 20, 48), -1, 9), ((33,), 0, 100),
                              ((40, 7), 0, 5), ((5000, 32), 0, 9000)]:
            s = I.typed(shape, dt, seed=401)
            sshape = list(shape)
            sshape[dim] = n
            src = I.typed(tuple(sshape), dt, seed=402)
            idx = torch.randint(0, shape[dim], (n,), generator=g)
            for alpha in ((1, -3) if not dt.is_floating_point else (1, 0.375, -2)):
                check_index_add(s, dim, idx, src, alpha)
            check_index_add(s, dim, idx.to(I32), src, what="int32 index")
        # views: strided self rows, strided source, strided index
        s = I.typed((50, 128), dt, seed=403)
        src = I.typed((60, 128), dt, seed=404)
        idx = torch.randint(0, 25, (120,), generator=g)
        check_index_add(s[::2], 0, idx[::2], src, what="strided self, index")
        check_index_add(s[:, ::2], 0, idx[:60], src[:, ::2], what="strided columns")
        check_index_add(torch.tensor(2, dtype=dt), 0, torch.tensor([0]), torch.tensor(3, dtype=dt), 2, what="0-dim")
        check_index_add(s, 0, torch.zeros((0,), dtype=I64), src[:0], what="no indices")
    # bool: OR of the selected source rows (alpha = False adds nothing)
    sb, srcb = I.booleans((40, 64), 0.1, seed=409), I.booleans((300, 64), 0.05, seed=410)
    ib = torch.randint(0, 40, (300,), generator=g)
    check_index_add(sb, 0, ib, srcb, True, what="bool")
    check_index_add(sb, 0, ib, srcb, False, what="bool, alpha False")
    check_index_add(sb.t().contiguous(), 1, ib, srcb.t().contiguous(), True, what="bool dim 1")
    # fp32 atomics (not reproducible, same tolerance)
    s, src = I.typed((64, 256), F32, seed=405), I.typed((5000, 256), F32, seed=406)
    assert check_index_add(s, 0, torch.randint(0, 64, (5000,), generator=g), src, 0.5, deterministic=False) == "scatter-atomic"


def test_index_add_full_size_rows_and_errors():
    rows = I.zipf_rows(1 << 20, 65536, 1.1, seed=4)
    for dt, alpha in ((F32, 1), (F32, 0.5), (I32, -3), (BF16, 1)):
        s = I.typed((65536, 256), dt, seed=407)
        src = I.typed((1 << 20, 256), dt, seed=408)
        assert check_index_add(s, 0, rows, src, alpha) == "scatter-sort-rows"
    d = lambda *s, dt=F32: torch.zeros(s, dtype=dt, device="cuda")
    ix = lambda *v: torch.tensor(v, device="cuda")
    for args, kind in (((d(4, 3), 0, ix(0, 1), d(3, 3)), "SHAPE"), ((d(4, 3), 0, ix(0, 1), d(2, 4)), "SHAPE"),
                       ((d(4, 3), 2, ix(0, 1), d(2, 3)), "DIM"), ((d(4, 3), 0, ix(0.0, 1.0), d(2, 3)), "DTYPE"),
                       ((d(4, 3), 0, ix(0, 1), d(2, 3, dt=BF16)), "DTYPE"),
                       ((d(4, 3), 0, ix(0, 1).view(1, 2), d(2, 3)), "SHAPE"), ((d(4, 3, dt=I64), 0, ix(0, 1), d(2, 3, dt=I64), 0.5), "SCALAR")):
        with pytest.raises(B.TxError) as e:
            B.tx_index_add_(*args)
        assert e.value.kind == kind, (kind, e.value.kind)
    with pytest.raises(B.TxError) as e:
        B.tx_index_add_(d(40, 64), 0, ix(0, 1), d(2, 64), 1, True, None)
    assert e.value.kind == "WORKSPACE"


def check_take(x_cpu, idx_cpu, out_like=None, what=""):
    want = O.take(x_cpu, idx_cpu)
    out = torch.empty(want.shape, dtype=want.dtype, device="cuda") if out_like is None else to_device_view(out_like)
    B.tx_take(out, to_device_view(x_cpu), to_device_view(idx_cpu))
    used = B.tx_last_path()
    torch.cuda.synchronize()
    assert_exact(out, want, "take %s %s idx%s %s [%s]" % (x_cpu.dtype, tuple(x_cpu.shape), tuple(idx_cpu.shape), what, used))
    return used


def test_take_sweep():
    g = torch.Generator().manual_seed(410)
    for dt in ALL:
        x = I.typed((7, 13, 5), dt, seed=411) if dt != BOOL else I.booleans((7, 13, 5), 0.5, seed=411)
        n = x.numel()
        idx = torch.randint(-n, n, (9, 31), generator=g)
        assert check_take(x, idx) == "take"
        check_take(x, idx.to(I32), what="int32 index")
        assert check_take(x.permute(2, 0, 1), idx, what="permuted") == "take-strided"
        assert check_take(x[:, ::2, 1:4], torch.randint(-63, 63, (50,), generator=g), what="sliced") == "take-strided"
        check_take(x, idx.t(), what="strided index")
        check_take(x, idx, out_like=torch.empty((31, 9), dtype=dt).t(), what="strided out")
        check_take(x, torch.zeros((0, 4), dtype=I64), what="empty index")
        check_take(torch.tensor(3, dtype=I64).to(dt), torch.tensor([0, -1, 0]), what="0-dim input")
        check_take(x, torch.tensor(-1), what="0-dim index")
    d = lambda *s, dt=F32: torch.zeros(s, dtype=dt, device="cuda")
    for args, kind in (((d(3), d(5), d(3)), "DTYPE"), ((d(3, dt=I32), d(5), d(3, dt=I64)), "DTYPE"), ((d(4), d(5), d(3, dt=I64)), "SHAPE"),
                       ((d(3), d(0), d(3, dt=I64)), "INDEX")):
        with pytest.raises(B.TxError) as e:
            B.tx_take(*args)
        assert e.value.kind == kind, (kind, e.value.kind)


def test_take_full_size():
    x = I.typed((8192, 8192), F32, seed=412)
    idx = torch.randint(-x.numel(), x.numel(), (4096, 4096), generator=torch.Generator().manual_seed(413))
    assert check_take(x, idx) == "take"
    assert check_take(x.t(), idx[:1024], what="transposed input") == "take-strided"


def run_select(fn_bytes, fn, out, what):
    count = torch.full((1,), -7, dtype=I64, device="cuda")
    ws = B.workspace(fn_bytes(out, count))
    fn(out, count, ws)
    used = B.tx_last_path()
    torch.cuda.synchronize()
    if used in ("select-fused", "nonzero-fused"):
        B.tx_lookback_status(ws)                       # raises if a bounded look-back wait gave up
    return int(count.item()), used


def check_masked_select(x_cpu, m_cpu, capacity=None, what=""):
    want = O.masked_select(x_cpu, m_cpu)
    x, m = to_device_view(x_cpu), to_device_view(m_cpu)
    total = 1
    for s in torch.broadcast_shapes(x_cpu.shape, m_cpu.shape):
        total *= s
    cap = total if capacity is None else capacity
    out = torch.full((cap + 3,), 0, dtype=x_cpu.dtype, device="cuda")[:cap]       # a guard zone after the buffer
    guard = out.storage_offset()
    n, used = run_select(lambda o, c: B.tx_masked_select_workspace_bytes(o, c, x, m), lambda o, c, ws: B.tx_masked_select(o, c, x, m, ws),
                         out, what)
    what = "masked_select %s x%s mask%s %s [%s]" % (x_cpu.dtype, tuple(x_cpu.shape), tuple(m_cpu.shape), what, used)
    assert n == want.numel(), (what, n, want.numel())
    k = min(n, cap)
    assert_exact(out[:k], want[:k], what)
    return used


def check_nonzero(x_cpu, capacity=None, what=""):
    want = O.nonzero(x_cpu)
    x = to_device_view(x_cpu)
    cap = x_cpu.numel() if capacity is None else capacity
    out = torch.full((cap, x_cpu.dim()), -1, dtype=I64, device="cuda")
    n, used = run_select(lambda o, c: B.tx_nonzero_workspace_bytes(o, c, x), lambda o, c, ws: B.tx_nonzero(o, c, x, ws), out, what)
    what = "nonzero %s %s %s [%s]" % (x_cpu.dtype, tuple(x_cpu.shape), what, used)
    assert n == want.shape[0], (what, n, want.shape[0])
    k = min(n, cap)
    assert_exact(out[:k], want[:k], what)
    if cap > k:
        assert (out[k:] == -1).all(), what + ": rows past the count were written"
    return used


def test_masked_select_sweep():
    for dt in ALL:
        for shape in [(7, 13, 5), (4096,), (4097,), (3, 5000), (1,), ()]:
            x = I.typed(shape, dt, seed=420) if dt != BOOL else I.booleans(shape, 0.5, seed=420)
            for p in (0.0, 0.03, 0.5, 1.0):
                m = I.bernoulli_mask(shape, p, seed=421)
                assert check_masked_select(x, m, what="p=%g" % p) == ("select" if x.numel() % 4 == 0 and x.numel() else "select-slab")
        x = I.typed((6, 50, 7), dt, seed=422) if dt != BOOL else I.booleans((6, 50, 7), 0.5, seed=422)
        m = I.bernoulli_mask((6, 50, 7), 0.3, seed=423)
        assert check_masked_select(x.permute(2, 0, 1), m.permute(2, 0, 1), what="permuted") == "select-strided"
        check_masked_select(x, m[:, :, :1], what="mask broadcast")
        check_masked_select(x[:, :1], m, what="x broadcast")
        check_masked_select(x, I.bernoulli_mask((7,), 0.5, seed=424), what="row mask")
        check_masked_select(x, m, capacity=10, what="small buffer")            # count still exact, 10 results written
        check_masked_select(x[:0], m[:0], what="empty")
    d = lambda *s, dt=F32: torch.zeros(s, dtype=dt, device="cuda")
    cnt, ws = d(1, dt=I64), B.workspace(4096)
    for args, kind in (((d(5), cnt, d(5), d(5)), "DTYPE"), ((d(5, dt=I32), cnt, d(5), d(5, dt=BOOL)), "DTYPE"),
                       ((d(5), d(1, dt=I32), d(5), d(5, dt=BOOL)), "DTYPE"), ((d(5), d(2, dt=I64), d(5), d(5, dt=BOOL)), "SHAPE"),
                       ((d(5, 1), cnt, d(5), d(5, dt=BOOL)), "SHAPE"), ((d(5), cnt, d(5), d(4, dt=BOOL)), "SHAPE")):
        with pytest.raises(B.TxError) as e:
            B.tx_masked_select(*args, ws)
        assert e.value.kind == kind, (kind, e.value.kind)
    with pytest.raises(B.TxError) as e:
        B.tx_masked_select(d(5), cnt, d(5), d(5, dt=BOOL), None)
    assert e.value.kind == "WORKSPACE"


def test_nonzero_sweep():
    for dt in ALL:
        for shape in [(7, 13, 5), (4096,), (4097,), (3, 5000), (1,), (), (2, 3, 4, 5, 6)]:
            for p in (0.0, 0.05, 0.7):
                keep = I.bernoulli_mask(shape, p, seed=430)
                x = (I.typed(shape, dt, seed=431) if dt != BOOL else torch.ones(shape, dtype=BOOL))
                x = torch.where(keep, x, torch.zeros((), dtype=dt))
                # whole vectors of 4 elements: the single pass; anything else: one element per lane, three passes
                assert check_nonzero(x, what="p=%g" % p) == ("nonzero-fused" if x.numel() % 4 == 0 else "select-slab")
                if x.numel() % 4 == 0:
                    B.tx_force_path("select-3pass")
                    try:
                        assert check_nonzero(x, what="three passes, p=%g" % p) == "select"
                    finally:
                        B.tx_force_path(None)
        x = torch.where(I.bernoulli_mask((6, 50, 7), 0.3, seed=432), I.typed((6, 50, 7), dt, seed=433) if dt != BOOL
                        else torch.ones((6, 50, 7), dtype=BOOL), torch.zeros((), dtype=dt))
        assert check_nonzero(x.permute(2, 0, 1), what="permuted") == "select-strided"
        check_nonzero(x[:, ::2], what="sliced")
        check_nonzero(x, capacity=17, what="small buffer")
        check_nonzero(x[:0], what="empty")
    sp = torch.tensor([0.0, -0.0, 1.0, float("nan"), 0.0, float("-inf"), 1e-45])
    for dt in (F32, BF16, F16):
        check_nonzero(sp.to(dt), what="signed zero, nan")
    d = lambda *s, dt=F32: torch.zeros(s, dtype=dt, device="cuda")
    cnt, ws = d(1, dt=I64), B.workspace(4096)
    for args, kind in (((d(5, 1), cnt, d(5)), "DTYPE"), ((d(5, 2, dt=I64), cnt, d(5)), "SHAPE"), ((d(5, dt=I64), cnt, d(5)), "SHAPE")):
        with pytest.raises(B.TxError) as e:
            B.tx_nonzero(*args, ws)
        assert e.value.kind == kind, (kind, e.value.kind)


def test_compaction_both_contiguous_forms_agree_with_oracle():
    for dt in ALL:
        x = I.typed((300, 1024), dt, seed=445) if dt != BOOL else I.booleans((300, 1024), 0.5, seed=445)
        m = I.bernoulli_mask((300, 1024), 0.3, seed=446)
        xs = torch.where(m, x, torch.zeros((), dtype=dt))
        assert check_masked_select(x, m) == "select" and check_nonzero(xs) == "nonzero-fused"
        B.tx_force_path("select-fused")
        try:
            assert check_masked_select(x, m) == "select-fused"
        finally:
            B.tx_force_path(None)
        B.tx_force_path("select-slab")
        try:
            assert check_masked_select(x, m) == "select-slab" and check_nonzero(xs) == "select-slab"
        finally:
            B.tx_force_path(None)
        # unaligned bases fall back to the element-per-lane form
        assert check_masked_select(x.view(-1)[1:-3], m.view(-1)[1:-3], what="offset base") in ("select", "select-fused", "select-slab")


def test_compaction_full_size():
    x = I.typed((8192, 8192), F32, seed=440)
    m = I.bernoulli_mask((8192, 8192), 0.25, seed=441)
    assert check_masked_select(x, m) == "select"
    B.tx_force_path("select-fused")                                     # the single-pass alternative on the same inputs
    try:
        assert check_masked_select(x, m) == "select-fused"
        for p in (0.0, 1.0):                                            # nothing / everything selected, many tiles
            assert check_masked_select(x[:2048], I.bernoulli_mask((2048, 8192), p, seed=443)) == "select-fused"
        xb = I.typed((4096, 8192), BF16, seed=444)
        assert check_masked_select(xb, I.bernoulli_mask((4096, 8192), 0.6, seed=445)) == "select-fused"
        assert check_masked_select(x[:1025, :8188].contiguous(), m[:1025, :8188].contiguous(), what="ragged last tile") == "select-fused"
    finally:
        B.tx_force_path(None)
    xs = torch.where(I.bernoulli_mask((8192, 4096), 0.1, seed=442), x[:, :4096], torch.zeros(()))
    assert check_nonzero(xs) == "nonzero-fused"
    assert check_nonzero(xs, capacity=1000003, what="small buffer") == "nonzero-fused"
    assert check_nonzero(xs.view(64, 128, 4096), what="three coordinates") == "nonzero-fused"
    for p in (0.0, 1.0):                                                # nothing / everything non-zero, many tiles
        assert check_nonzero(torch.full((1024, 4100), p), what="all %g" % p) == "nonzero-fused"
    assert check_nonzero(xs.to(I64)[:3000], what="8-byte elements") == "nonzero-fused"
    B.tx_force_path("select-3pass")
    try:
        assert check_nonzero(xs) == "select"
    finally:
        B.tx_force_path(None)


# --------------------------------------------------------------------------- scatter_reduce_, index_put_
def check_scatter_reduce(self_cpu, dim, idx_cpu, src_cpu, reduce, include_self, what=""):
    want = O.scatter_reduce_(self_cpu.clone(), dim, idx_cpu, src_cpu, reduce, include_self)
    dst = to_device_view(self_cpu).clone() if self_cpu.is_contiguous() else to_device_view(self_cpu)
    idx, src = to_device_view(idx_cpu), to_device_view(src_cpu)
    ws = B.workspace(B.tx_scatter_reduce_workspace_bytes(dst, dim, idx, src, reduce, include_self))
    B.tx_scatter_reduce_(dst, dim, idx, src, reduce, include_self, ws)
    used = B.tx_last_path()
    torch.cuda.synchronize()
    what = "scatter_reduce %s %s self%s idx%s dim=%d include_self=%s %s [%s]" % (reduce, self_cpu.dtype, tuple(self_cpu.shape),
                                                                              tuple(idx_cpu.shape), dim, include_self, what, used)
    if not self_cpu.dtype.is_floating_point:
        assert_exact(dst, want, what)
    else:
        # what lands on an element, in magnitude: sums and means are judged against it, products and extrema have no cancellation
        s2 = self_cpu.double() ** 2
        window = tuple(slice(0, n) for n in idx_cpu.shape)
        s2.scatter_add_(dim, idx_cpu.long().contiguous(), (src_cpu.double() ** 2)[window].contiguous())
        scale = s2.sqrt() if reduce in ("sum", "mean") else torch.zeros_like(s2)
        assert_rel(dst, want, 1e-5 if self_cpu.dtype == F32 else 1e-2, scale, what)
    return used


@pytest.mark.parametrize("reduce", ["sum", "prod", "mean", "amax", "amin"])
def test_scatter_reduce_sweep(reduce):
    g = torch.Generator().manual_seed(450)
    for dt, inc in itertools.product((F32, BF16, F16, I32, I64), (True, False)):
        for shape, dim, ishape in [((50, 64), 0, (300, 64)), ((50, 64), 1, (50, 20)), ((6, 20, 48), 1, (6, 77, 48)), ((33,), 0, (200,)),
                                   ((40, 7), 0, (5, 3))]:
            small = reduce == "prod"
            s = (I.typed(shape, dt, seed=451) if not small else (torch.randint(-2, 3, shape, generator=g).to(dt)))
            sshape = tuple(max(a, b) for a, b in zip(ishape, shape)) if dim is None else ishape
            src = (I.typed(sshape, dt, seed=452) if not small else torch.randint(-2, 3, sshape, generator=g).to(dt))
            if reduce == "prod" and dt.is_floating_point:
                s, src = s * 0.5 + 1, src * 0.25 + 1                      # products of many terms stay finite
            idx = torch.randint(0, shape[dim], ishape, generator=g)
            used = check_scatter_reduce(s, dim, idx, src, reduce, inc)
            assert used == ("scatter-reduce-sort" if not (reduce == "sum" and inc) else used)
        # NaN / inf in the values, strided views, int32 index
        if dt.is_floating_point:
            s, src = I.typed((30, 16), dt, seed=453, specials=0.05), I.typed((90, 16), dt, seed=454, specials=0.05)
            idx = torch.randint(0, 30, (90, 16), generator=g)
            if reduce in ("amax", "amin"):
                check_scatter_reduce(s, 0, idx, src, reduce, inc, what="specials")
        s, src = I.typed((30, 32), dt, seed=455), I.typed((90, 32), dt, seed=456)
        if reduce == "prod":
            s, src = (s.abs().clamp(max=1) if dt.is_floating_point else s.clamp(-1, 1)), (src.abs().clamp(max=1) if dt.is_floating_point else src.clamp(-1, 1))
        idx = torch.randint(0, 15, (90, 16), generator=g)
        check_scatter_reduce(s[::2, ::2], 0, idx.to(I32), src[:, ::2], reduce, inc, what="views")
    d = lambda *s, dt=F32: torch.zeros(s, dtype=dt, device="cuda")
    ws = B.workspace(1 << 16)
    if reduce == "mean":
        with pytest.raises(B.TxError) as e:
            B.tx_scatter_reduce_(d(4, 3, dt=BOOL), 0, d(2, 3, dt=I64), d(2, 3, dt=BOOL), reduce, True, ws)
        assert e.value.kind == "DTYPE"
    else:
        for inc in (True, False):
            check_scatter_reduce(I.booleans((30, 16), 0.4, seed=457), 0, torch.randint(0, 30, (90, 16), generator=g),
                                 I.booleans((90, 16), 0.6, seed=458), reduce, inc, what="bool")
    with pytest.raises(B.TxError) as e:
        B.tx_scatter_reduce_(d(4, 3), 0, d(2, 3, dt=I64), d(2, 3), "median", True, ws)
    assert e.value.kind == "SCALAR"
    with pytest.raises(B.TxError) as e:
        B.tx_scatter_reduce_(d(4, 3), 0, d(2, 3, dt=I64), d(2, 3), reduce, False, None)
    assert e.value.kind == "WORKSPACE"


def check_index_put(self_cpu, indices_cpu, values_cpu, accumulate, unique=True, what=""):
    want = O.index_put_(self_cpu.clone(), indices_cpu, values_cpu, accumulate)
    dst = to_device_view(self_cpu).clone() if self_cpu.is_contiguous() else to_device_view(self_cpu)
    ind, val = [to_device_view(i) for i in indices_cpu], to_device_view(values_cpu)
    nbytes = B.tx_index_put_workspace_bytes(dst, ind, val, accumulate)
    B.tx_index_put_(dst, ind, val, accumulate, B.workspace(nbytes) if nbytes else None)
    used = B.tx_last_path()
    torch.cuda.synchronize()
    what = "index_put %s self%s values%s accumulate=%s %s [%s]" % (self_cpu.dtype, tuple(self_cpu.shape), tuple(values_cpu.shape),
                                                                accumulate, what, used)
    if accumulate and self_cpu.dtype.is_floating_point:
        s2 = self_cpu.double() ** 2
        s2.index_put_(tuple(i.long() for i in indices_cpu), values_cpu.double() ** 2, accumulate=True)
        assert_rel(dst, want, 1e-5 if self_cpu.dtype == F32 else 1e-2, s2.sqrt(), what)
    else:
        assert unique or accumulate, "assignment with duplicates has no unique answer"
        assert_exact(dst, want, what)
    return used


def test_index_put_sweep():
    g = torch.Generator().manual_seed(460)
    for dt in ALL:
        mk = (lambda shape, seed: I.typed(shape, dt, seed=seed)) if dt != BOOL else (lambda shape, seed: I.booleans(shape, 0.3, seed=seed))
        s = mk((12, 9, 16), 461)
        # accumulate, duplicates allowed: one, two and three index tensors, negative indices, broadcast values
        i0, i1, i2 = torch.randint(-12, 12, (40,), generator=g), torch.randint(-9, 9, (40,), generator=g), torch.randint(-16, 16, (40,), generator=g)
        used = check_index_put(s, [i0], mk((40, 9, 16), 462), True)              # whole rows: the scatter_add_ row path
        assert used == ("scatter-sort-rows" if dt.is_floating_point else "index-put-atomic" if dt == BOOL else "scatter-atomic")
        used = check_index_put(s, [i0, i1], mk((40, 16), 463), True)
        assert used == ("index-put-sort" if dt.is_floating_point else "index-put-atomic")
        check_index_put(s, [i0, i1.to(I32), i2], mk((40,), 464), True)
        check_index_put(s, [i0, i1], mk((16,), 465), True, what="values broadcast over positions")
        check_index_put(s, [i0, i1], mk((), 466), True, what="0-dim values")
        check_index_put(s, [i0.view(40, 1)[:5], i1.view(1, 40)[:, :7]], mk((5, 7, 16), 467), True, what="broadcast indices")
        check_index_put(s.permute(1, 0, 2), [i1, i0], mk((40, 16), 468), True, what="permuted self")
        check_index_put(s, [i0[::2], i1[::2]], mk((40, 16), 469)[::2], True, what="strided index and values")
        # assignment: distinct destinations
        perm = torch.randperm(12 * 9, generator=g)[:50]
        u0, u1 = perm // 9, perm % 9 - 9                                       # second index given as negatives
        assert check_index_put(s, [u0, u1], mk((50, 16), 470), False) == "index-put"
        # whole dense rows over dim 0: the row-copy kernel (negative indices wrap); by name, sliced or shifted: one lane per element
        rp = torch.randperm(12, generator=g)[:7]
        rp[::2] -= 12
        used = check_index_put(s, [rp], mk((7, 9, 16), 471), False, what="rows")
        assert used == ("index-put" if dt == BOOL else "index-put-rows"), (dt, used)
        B.tx_force_path("index-put")
        try:
            assert check_index_put(s, [rp], mk((7, 9, 16), 471), False, what="rows, by name") == "index-put"
        finally:
            B.tx_force_path(None)
        assert check_index_put(s[:, :, 1:], [rp], mk((7, 9, 15), 474), False, what="rows of a slice") == "index-put"
        assert check_index_put(s, [rp[:5].to(I32)], mk((9, 9, 16), 475)[::2], False, what="strided values rows") == (
            "index-put" if dt == BOOL else "index-put-rows")
        check_index_put(s, [u0, u1], mk((1, 16), 472), False, what="broadcast values")
        check_index_put(s, [u0[:0], u1[:0]], mk((0, 16), 473), True, what="no positions")
    d = lambda *s, dt=F32: torch.zeros(s, dtype=dt, device="cuda")
    ix = lambda *v: torch.tensor(v, device="cuda")
    for args, kind in (((d(4, 3), [ix(0, 1)], d(2, 4)), "SHAPE"), ((d(4, 3), [ix(0, 1), ix(0, 1, 2)], d(2)), "SHAPE"),
                       ((d(4, 3), [ix(0.0, 1.0)], d(2, 3)), "DTYPE"), ((d(4, 3), [ix(0, 1)], d(2, 3, dt=BF16)), "DTYPE"),
                       ((d(4, 3), [], d(2, 3)), "DIM"), ((d(4, 3), [ix(0), ix(0), ix(0)], d(1)), "DIM")):
        with pytest.raises(B.TxError) as e:
            B.tx_index_put_(args[0], args[1], args[2], True, B.workspace(1 << 16))
        assert e.value.kind == kind, (kind, e.value.kind)
    with pytest.raises(B.TxError) as e:
        B.tx_index_put_(d(4, 3), [ix(0, 1)], d(2, 3), True, None)
    assert e.value.kind == "WORKSPACE"


def test_scatter_reduce_whole_rows():
    # a row id broadcast over the trailing dims: sum, amax and amin take the sorted whole-row kernels
    g = torch.Generator().manual_seed(470)
    cases = [(37, 1000, 256, "uniform"), (37, 1000, 99, "uniform"), (9, 1500, 64, "hot"), (300, 130, 24, "uniform"),
             (5, 700, 16, "one")]
    for dt, (nrow, n, width, kind) in itertools.product((F32, BF16, F16, I32, I64), cases):
        s, src = I.typed((nrow, width), dt, seed=471), I.typed((n, width), dt, seed=472)
        if kind == "uniform":
            rows = torch.randint(0, nrow, (n,), generator=g)
        elif kind == "hot":                           # one destination takes most rows: runs that pass through whole chunks
            rows = torch.where(torch.rand(n, generator=g) < 0.9, torch.tensor(4), torch.randint(0, nrow, (n,), generator=g))
        else:
            rows = torch.full((n,), 2)
        idx = rows.unsqueeze(1).expand(n, width)
        for reduce, inc in (("sum", False), ("amax", True), ("amax", False), ("amin", True), ("amin", False)):
            used = check_scatter_reduce(s, 0, idx, src, reduce, inc, what=kind)
            assert used == ("scatter-reduce-rows" if width % 4 == 0 else "scatter-reduce-rows-scalar"), used
        assert check_scatter_reduce(s, 0, idx, src, "mean", True, what=kind) == "scatter-reduce-sort"
    # NaN in src, int32 index, a strided destination whose rows stay contiguous, and the same input forced onto the element path
    s, src = I.typed((64, 128), F32, seed=473), I.typed((900, 128), F32, seed=474, specials=0.02)
    rows = torch.randint(0, 32, (900,), generator=g)
    idx = rows.to(I32).unsqueeze(1).expand(900, 128)
    for reduce, inc in (("amax", True), ("amin", False), ("sum", False)):
        assert check_scatter_reduce(s[::2], 0, idx, src, reduce, inc, what="views").startswith("scatter-reduce-rows")
        B.tx_force_path("scatter-reduce-sort")
        try:
            assert check_scatter_reduce(s[::2], 0, idx, src, reduce, inc, what="forced") == "scatter-reduce-sort"
        finally:
            B.tx_force_path(None)


def test_scatter_reduce_and_index_put_larger():
    g = torch.Generator().manual_seed(480)
    s, src = I.typed((4096, 256), F32, seed=481), I.typed((65536, 256), F32, seed=482)
    rows = I.zipf_rows(65536, 4096, 1.1, seed=4)
    idx = rows.unsqueeze(1).expand(65536, 256)
    for reduce, inc in (("amax", True), ("mean", False), ("sum", False)):
        check_scatter_reduce(s, 0, idx, src, reduce, inc, what="zipf rows")
    check_index_put(s, [rows], src, True, what="zipf rows")
    si = I.typed((4096, 256), I64, seed=483)
    check_index_put(si, [rows, torch.randint(0, 256, (65536,), generator=g)], I.typed((65536,), I64, seed=484), True)
    perm = torch.randperm(4096, generator=g)
    assert check_index_put(s, [perm], I.typed((4096, 256), F32, seed=485), False) == "index-put-rows"
    assert check_index_put(s, [perm[:4095] - 4096], I.typed((4095, 256), F32, seed=486), False, what="odd row count") == "index-put-rows"
