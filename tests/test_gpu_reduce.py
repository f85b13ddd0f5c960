"""GPU parity: dimension reductions (HIP library through the C ABI) vs. the CPU oracle.

sum / mean / amax / argmax / prod / var over dim 0, dim -1, dims (0,2) and all
dims, keepdim both ways, fp32 / bf16 / fp16 / int dtypes, on small and
multi-tile ragged shapes, strided views, and the full [64,4096,1024] workload.
"""
import itertools

import pytest
import torch

from oracle import oracle as O
from paper_2512_10977_amd import binding as B
from paper_2512_10977_amd import inputs as I
from tests.parity import assert_exact, assert_exact_fp, assert_rel, to_device_view

pytestmark = pytest.mark.gpu

F32, BF16, F16, I32, I64, BOOL = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool
OPS = ["sum", "mean", "amax", "argmax", "prod", "var", "amin", "argmin", "std", "any", "all", "logsumexp", "nansum", "nanmean",
       "count_nonzero", "norm"]
FLT_MIN = 1.1754943508222875e-38


def natural_scale(op, x, dims, keepdim):
    """Magnitude of what a result was made of (binary64): sqrt(sum x^2) for sum, that / n for mean."""
    if op in ("sum", "mean", "nansum", "nanmean") and x.dtype.is_floating_point:
        xd = x.double()
        xd = torch.where(xd.isfinite(), xd, torch.zeros_like(xd))
        d = list(range(x.dim())) if dims is None else dims
        if x.dim() == 0:
            s = xd.abs()
            n = 1
        else:
            s = (xd * xd).sum(dim=d, keepdim=keepdim).sqrt()
            n = 1
            for k in ([d] if isinstance(d, int) else d):
                n *= x.shape[k]
        return s / max(n, 1) if op in ("mean", "nanmean") else s
    if op == "prod":
        return FLT_MIN
    if op == "logsumexp":
        return 1.0             # max + log(sum): the absolute error scales with |max|, floor one
    return 0.0


def check_reduce(op, x_cpu, dims=None, keepdim=False, correction=1.0, out_dtype=None, what=""):
    try:
        want = O.reduce(op, x_cpu, dims, keepdim, correction, out_dtype=out_dtype)
    except O.OracleError as e:
        x = to_device_view(x_cpu)
        with pytest.raises(B.TxError) as g:
            dt, shape = B.tx_infer_reduce(op, x, dims, keepdim)      # may already be the expected error
            B.tx_reduce(op, torch.empty(shape, dtype=dt, device="cuda"), x, dims, keepdim, correction)
        assert g.value.kind.lower() == e.kind, (g.value.kind, e.kind)
        return None
    x = to_device_view(x_cpu)
    out = torch.empty(want.shape, dtype=want.dtype, device="cuda")
    nbytes = B.tx_reduce_workspace_bytes(op, out, x, dims, keepdim)
    ws = B.workspace(nbytes) if nbytes else None
    B.tx_reduce(op, out, x, dims, keepdim, correction, ws)
    used = B.tx_last_path()
    torch.cuda.synchronize()
    what = "%s %s %s dims=%s keepdim=%s %s [%s]" % (op, x_cpu.dtype, tuple(x_cpu.shape), dims, keepdim, what, used)
    if op in ("argmax", "argmin") or not want.dtype.is_floating_point:
        assert_exact(out, want, what)
    elif op in ("amax", "amin"):
        assert_exact_fp(out, want, what)
    else:
        rel = 1e-5 if want.dtype == F32 and x_cpu.dtype == F32 else (1e-5 if want.dtype == F32 else 1e-2)
        assert_rel(out, want, rel, natural_scale(op, x_cpu, dims, keepdim), what)
    return used


def check_reduce_keepdim_form(op, x_cpu, dims):
    """keepdim=True at a size where the oracle takes seconds per call: the library's keepdim=True result must be its
    own keepdim=False result, bit for bit, in the shape the oracle's inference gives (the values were just checked
    against the oracle by the keepdim=False call; the two forms run the same kernels on the same plan)."""
    x = to_device_view(x_cpu)
    dt, flat_shape = B.tx_infer_reduce(op, x, dims, False)
    dt_k, keep_shape = B.tx_infer_reduce(op, x, dims, True)
    want_dt, want_shape = O.infer_reduce(op, x_cpu, dims, True)
    assert (dt_k, tuple(keep_shape)) == (want_dt, tuple(want_shape)) and dt == dt_k
    outs = []
    for keepdim, shape in ((False, flat_shape), (True, keep_shape)):
        out = torch.empty(shape, dtype=dt, device="cuda")
        nbytes = B.tx_reduce_workspace_bytes(op, out, x, dims, keepdim)
        B.tx_reduce(op, out, x, dims, keepdim, 1.0, B.workspace(nbytes) if nbytes else None)
        outs.append(out)
    torch.cuda.synchronize()
    a, b = outs[0].reshape(-1), outs[1].reshape(-1)
    same = (a == b) | ((a != a) & (b != b)) if dt.is_floating_point else (a == b)
    assert bool(same.all()), "%s dims=%s: keepdim=True differs from keepdim=False" % (op, dims)


DIMSETS = [0, -1, 1, (0, 2), None]


@pytest.mark.parametrize("op", ["sum", "argmax", "var", "amin", "logsumexp"])
def test_reduce_short_rows_half_a_wave_per_row(op):
    """Many rows of 1 to 2 KiB: half a wave per row; the same rows with a wave each, by name."""
    for dt, shape in ((BF16, (70000, 1024)), (F32, (66000, 512)), (F32, (65536, 260)), (BF16, (2, 33000, 520))):
        x = I.reduction_input(shape, dt, seed=77)
        assert check_reduce(op, x, -1) == "rows-half", (dt, shape)
        B.tx_force_path("rows-wave")
        try:
            assert check_reduce(op, x, -1, what="a wave per row") == "rows-wave"
        finally:
            B.tx_force_path(None)
    assert check_reduce(op, I.reduction_input((66000, 256), F32, seed=78), -1) == "rows-wave"        # 1 KiB: a wave
    assert check_reduce(op, I.reduction_input((1000, 512), F32, seed=79), -1) == "rows-wave"         # too few rows


@pytest.mark.parametrize("op", OPS)
def test_reduce_small_sweep(op):
    for dt, dims, keepdim in itertools.product([F32, BF16, F16, I32, I64, BOOL], DIMSETS, [False, True]):
        x = I.typed((7, 13, 5), dt, seed=201, std=1.0)
        check_reduce(op, x, dims, keepdim)
    for kind in I.VIEW_KINDS:
        for dims in DIMSETS:
            check_reduce(op, I.make_view((7, 13, 5), F32, kind, seed=202, std=1.0), dims, what=kind)
            check_reduce(op, I.make_view((7, 13, 5), I64, kind, seed=203), dims, what=kind)


@pytest.mark.parametrize("op", OPS)
def test_reduce_edge_cases(op):
    check_reduce(op, torch.tensor(3.5), None)
    check_reduce(op, torch.tensor(3.5), 0)
    check_reduce(op, torch.tensor(3.5), -1, keepdim=True)
    check_reduce(op, torch.zeros((3, 0)), 1)                 # empty reduced extent (error for amax / argmax)
    check_reduce(op, torch.zeros((0, 3)), 1)                 # empty kept extent: empty result
    check_reduce(op, torch.zeros((0,)), None)
    check_reduce(op, I.typed((5, 1, 7), F32, seed=204), 1)   # reducing a size-1 dim
    check_reduce(op, I.typed((1, 1), F32, seed=205), None)
    x = I.typed((6, 9), F32, seed=206, specials=0.08)        # NaN / inf inside
    for dims in (0, 1, None):
        check_reduce(op, x, dims, what="specials")
    ties = I.typed((40, 33), BF16, seed=207, std=1.0)        # few distinct values: real ties for argmax
    for dims in (0, 1, None):
        check_reduce(op, ties, dims, what="ties")


def test_reduce_error_codes():
    d = lambda *s, dt=F32: torch.zeros(s, dtype=dt, device="cuda")
    for bad in ((0, 0), (1, -2), 3, -4):
        with pytest.raises(B.TxError) as e:
            B.tx_reduce("sum", d(), d(2, 3, 4), bad)
        assert e.value.kind == "DIM"
    for op in ("prod", "argmax", "argmin"):
        with pytest.raises(B.TxError) as e:
            B.tx_reduce(op, d(3, dt=I64 if op != "prod" else F32), d(2, 3, 4), (0, 2))
        assert e.value.kind == "DIM"
    for op in ("std", "logsumexp"):
        with pytest.raises(B.TxError) as e:
            B.tx_reduce(op, d(dt=I64), d(4, dt=I64))
        assert e.value.kind == "DTYPE"
    with pytest.raises(B.TxError) as e:
        B.tx_reduce("any", d(3), d(3, 4), 1)                 # any / all return bool
    assert e.value.kind == "DTYPE"
    with pytest.raises(B.TxError) as e:
        B.tx_reduce("amin", d(3), d(3, 0), 1)
    assert e.value.kind == "EMPTY_REDUCTION"
    with pytest.raises(B.TxError) as e:
        B.tx_reduce("mean", d(dt=I64), d(4, dt=I64))
    assert e.value.kind == "DTYPE"
    with pytest.raises(B.TxError) as e:
        B.tx_reduce("argmax", d(dt=I64), d(4, dt=BOOL))
    assert e.value.kind == "DTYPE"
    with pytest.raises(B.TxError) as e:
        B.tx_reduce("amax", d(3), d(3, 0), 1)
    assert e.value.kind == "EMPTY_REDUCTION"
    with pytest.raises(B.TxError) as e:
        B.tx_reduce("sum", d(4), d(3, 4), 1)
    assert e.value.kind == "SHAPE"
    big = d(1, 1 << 22)
    with pytest.raises(B.TxError) as e:
        B.tx_reduce("sum", d(), big, None, ws=None)          # split reduction without workspace
    assert e.value.kind == "WORKSPACE"


@pytest.mark.parametrize("op", OPS)
def test_reduce_multi_tile_ragged(op):
    # rows path (wave and block groups), cols path, split paths, ragged tails, misaligned bases
    paths = set()
    for dt in (F32, BF16, I64):
        x = I.typed((37, 50, 1027), dt, seed=210, std=1.0)
        for dims in (0, -1, (0, 2), None, 1):
            paths.add(check_reduce(op, x, dims))
        y = I.typed((3, 70001), dt, seed=211, std=1.0)
        paths.add(check_reduce(op, y, 1))                    # few long rows -> split rows
        paths.add(check_reduce(op, y[:, 1:], 1))             # misaligned
        z = I.typed((5000, 96), dt, seed=212, std=1.0)
        paths.add(check_reduce(op, z, 0))                    # cols with split
        paths.add(check_reduce(op, z.t(), 1))                # transposed view: reduced dim strided, kept contiguous
        paths.add(check_reduce(op, z, 1))
        paths.add(check_reduce(op, I.typed((600, 9001), dt, seed=215, std=1.0), 1))   # long rows, enough of them: block per row
    paths.discard(None)
    assert {"rows-wave", "rows-block", "rows-split", "cols"} <= paths, paths
    if op in ("sum", "mean", "prod", "var", "std", "logsumexp", "nansum", "nanmean", "norm"):
        check_reduce(op, I.typed((64, 300), BF16, seed=213, std=1.0), 1, out_dtype=F32, what="fp32 out")


def test_var_correction_and_shift():
    x = I.typed((33, 257), F32, seed=214, std=1.0)
    for c in (0.0, 1.0, 2.5, 300.0):
        check_reduce("var", x, 1, correction=c)
    check_reduce("var", x + 1024.0, 1)
    check_reduce("var", x[:, :1], 1)                         # n = 1 -> NaN


# --------------------------------------------------------------------------- full workload [64,4096,1024]
FULL = (64, 4096, 1024)


@pytest.fixture(scope="module")
def full_inputs():
    return {F32: I.reduction_input(FULL, F32), BF16: I.reduction_input(FULL, BF16), I64: I.reduction_input(FULL, I64)}


@pytest.mark.parametrize("dims", [0, -1, (0, 2), None])
@pytest.mark.parametrize("dt", [F32, BF16, I64])
def test_reduce_full_size(full_inputs, dt, dims):
    x = full_inputs[dt]
    ops = ["sum", "amax", "argmax"] if dt == I64 else OPS[:6]
    if dims is None:        # the oracle walks all 2.7e8 elements on one core per op: keep the all-dims list short
        ops = {F32: ["sum", "argmax", "var"], BF16: ["mean", "amax", "prod"], I64: ["sum", "argmax"]}[dt]
    for op in ops:
        if dims == (0, 2) and op in ("prod", "argmax"):
            continue
        check_reduce(op, x, dims, keepdim=False)
        check_reduce_keepdim_form(op, x, dims)


@pytest.mark.parametrize("dims", [0, -1])
def test_new_reductions_full_size(full_inputs, dims):
    for op in ("amin", "argmin", "std", "logsumexp"):
        check_reduce(op, full_inputs[F32], dims)
    for op in ("logsumexp", "amin"):
        check_reduce(op, full_inputs[BF16], dims)
    x = full_inputs[I64]
    check_reduce("argmin", x, dims)
    z = (x % 7 != 0).to(torch.int32)                         # mostly non-zero: "all" has to see every zero
    z[:, 5, 9] = 1
    z[3, :, 11] = 1
    check_reduce("all", z, dims)
    check_reduce("any", (x % 1000003 == 0), dims)


def test_std_and_logsumexp_details():
    x = I.typed((33, 257), F32, seed=216, std=1.0)
    for c in (0.0, 1.0, 2.5, 300.0):
        check_reduce("std", x, 1, correction=c)
    check_reduce("std", x + 1024.0, 1)
    big = I.typed((40, 3000), F32, seed=217, std=30.0)       # spread of 100+ in the exponent: rescaling matters
    check_reduce("logsumexp", big, 1)
    check_reduce("logsumexp", big - 20000.0, 1)
    check_reduce("logsumexp", big + 20000.0, None)
    inf = float("inf")
    sp = torch.tensor([[1.0, -inf, 2.0], [-inf, -inf, -inf], [inf, 1.0, 2.0], [float("nan"), inf, 0.0], [inf, -inf, inf]])
    check_reduce("logsumexp", sp, 1)
    check_reduce("logsumexp", sp, 0)
    check_reduce("logsumexp", sp.repeat(1, 500), 1)          # across lanes and waves


@pytest.mark.parametrize("p", [0.0, 2.0, float("inf"), -float("inf"), 3.0, 0.5, -1.0])
def test_norm_orders(p):
    paths = set()
    for dt in (F32, BF16, F16):
        x = I.typed((37, 50, 259), dt, seed=220, std=1.0)
        for dims in (0, -1, (0, 2), None, 1):
            paths.add(check_reduce("norm", x, dims, correction=p))
        paths.add(check_reduce("norm", I.typed((3, 70001), dt, seed=221, std=1.0), 1, correction=p))
        paths.add(check_reduce("norm", I.typed((5000, 96), dt, seed=222, std=1.0), 0, correction=p))
        check_reduce("norm", I.typed((6, 9), dt, seed=223, specials=0.08), 1, correction=p, what="specials")
        check_reduce("norm", torch.zeros((3, 0), dtype=dt), 1, correction=p)         # empty extent: 0, or an error for inf / negative p
        check_reduce("norm", torch.zeros((0, 3), dtype=dt), 1, correction=p)
    assert {"rows-wave", "rows-split", "cols"} <= paths, paths
    # squares beyond fp32's range inside, a result within it
    big = torch.tensor([[1e20, -1e20, 3e19], [1e-30, 1e-30, 0.0]], dtype=F32)
    check_reduce("norm", big, 1, correction=p, what="large and tiny")
    check_reduce("norm", torch.tensor([1, 2]), None, correction=p)                    # integers: refused
    check_reduce("norm", torch.ones(3), None, correction=float("nan"))               # NaN exponent: refused


def test_nan_reductions_and_count_full_size(full_inputs):
    x = full_inputs[F32].clone()
    x.view(-1)[::7] = float("nan")
    for dims in (0, -1, None):
        check_reduce("nansum", x, dims)
        check_reduce("nanmean", x, dims)
    x[:, 3, :] = float("nan")                                                        # whole slices of NaN: nansum 0, nanmean NaN
    check_reduce("nanmean", x, 0)
    check_reduce("nansum", x, -1)
    z = full_inputs[F32].clone()
    z.view(-1)[::3] = 0.0
    z.view(-1)[1::5] = -0.0
    for dims in (0, -1, None):
        check_reduce("count_nonzero", z, dims)
        check_reduce("norm", full_inputs[F32], dims, correction=2.0)
    check_reduce("count_nonzero", full_inputs[BF16], -1)
    check_reduce("count_nonzero", full_inputs[I64] % 3, 0)
    check_reduce("norm", full_inputs[BF16], -1, correction=2.0)
    check_reduce("norm", full_inputs[F32], 0, correction=float("inf"))
