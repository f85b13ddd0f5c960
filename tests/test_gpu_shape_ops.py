"""GPU parity: copy with conversion, flip, roll, tril, triu (HIP library through the C ABI) vs. the CPU oracle.
Everything here moves or converts values without arithmetic, so every comparison is bit-exact."""
import itertools

import pytest
import torch

from oracle import oracle as O
from paper_2512_10977_amd import binding as B
from paper_2512_10977_amd import inputs as I
from tests.parity import assert_exact, assert_exact_fp, to_device_view

pytestmark = pytest.mark.gpu

F32, BF16, F16, I32, I64, BOOL = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool
ALL = [F32, BF16, F16, I32, I64, BOOL]


def same(out, want, what):
    (assert_exact_fp if want.dtype.is_floating_point else assert_exact)(out, want, what)


def in_range(x, dst):
    """Values a float -> integer conversion is defined for: finite and inside the target's range."""
    if x.dtype.is_floating_point and not dst.is_floating_point and dst != BOOL:
        return torch.where(x.isfinite() & (x.abs() < 1e9), x, torch.zeros_like(x))
    return x


def check_copy(x_cpu, dst, shape=None, out_layout=None, what=""):
    x_cpu = in_range(x_cpu, dst)
    want = O.copy(x_cpu, dtype=dst, shape=shape)
    x = to_device_view(x_cpu)
    out = torch.empty(want.shape, dtype=dst, device="cuda")
    if out_layout == "transposed" and out.dim() >= 2:
        out = torch.empty(want.shape[::-1], dtype=dst, device="cuda").permute(*range(out.dim() - 1, -1, -1))
    B.tx_copy(out, x)
    used = B.tx_last_path()
    torch.cuda.synchronize()
    same(out, want, "copy %s -> %s %s %s [%s]" % (x_cpu.dtype, dst, tuple(want.shape), what, used))
    return used


def test_copy_every_dtype_pair_and_layout():
    for da, db in itertools.product(ALL, ALL):
        for kind in I.VIEW_KINDS:
            check_copy(I.make_view((7, 13, 5), da, kind, seed=401, specials=0.02), db, what=kind)
        check_copy(I.typed((33, 40), da, seed=402), db, out_layout="transposed", what="transposed out")
        check_copy(I.typed((), da, seed=403), db)
        check_copy(I.typed((0, 3), da, seed=404), db)
        check_copy(I.typed((5,), da, seed=405), db, shape=(4, 3, 5), what="broadcast")
        check_copy(I.typed((), da, seed=406), db, shape=(6, 2), what="broadcast 0-dim")
    # halves of ties, subnormals, values beyond fp16's range: one rounding
    edge = torch.tensor([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -11, 65520.0, 65519.0, 1e-41, -6e-8, 3.3e38, 2 ** 24 + 1.0], dtype=F32)
    for dt in (BF16, F16):
        check_copy(edge, dt, what="ties")
    big = torch.tensor([2 ** 24 + 1, 2 ** 24 + 3, -(2 ** 53) - 1, 2 ** 40 + 5, 2 ** 62, -2 ** 63])
    for dt in (F32, BF16, F16, I32, BOOL):
        check_copy(big, dt, what="large integers")
    with pytest.raises(B.TxError) as e:
        B.tx_copy(torch.zeros(3, device="cuda"), torch.zeros(4, 3, device="cuda"))
    assert e.value.kind == "SHAPE"


@pytest.mark.parametrize("da,db", [(F32, F32), (F32, BF16), (BF16, F32), (I64, F32), (F32, I32), (F16, BOOL), (I64, I64)])
def test_copy_full_size(da, db):
    x = I.typed((8192, 8192), da, seed=407, specials=0.0 if not db.is_floating_point else 0.01)
    assert check_copy(x, db) == "vec"
    assert check_copy(x.t(), db, what="transposed") in ("tile", "tile-scalar")


def check_remap(op, x_cpu, *args, what=""):
    fn = {"flip": O.flip, "roll": O.roll, "tril": O.tril, "triu": O.triu}[op]
    call = {"flip": B.tx_flip, "roll": B.tx_roll, "tril": lambda o, x, k: B.tx_tri(o, x, k, False), "triu": lambda o, x, k: B.tx_tri(o, x, k, True)}[op]
    try:
        want = fn(x_cpu, *args)
    except O.OracleError as e:
        with pytest.raises(B.TxError) as g:
            call(torch.empty(x_cpu.shape, dtype=x_cpu.dtype, device="cuda"), to_device_view(x_cpu), *args)
        assert g.value.kind.lower() == e.kind, (op, args, g.value.kind, e.kind)
        return None
    x = to_device_view(x_cpu)
    out = torch.empty(want.shape, dtype=want.dtype, device="cuda")
    call(out, x, *args)
    used = B.tx_last_path()
    torch.cuda.synchronize()
    same(out, want, "%s%s %s %s %s [%s]" % (op, args, x_cpu.dtype, tuple(x_cpu.shape), what, used))
    return used


def test_flip_roll_sweep():
    paths = set()
    for dt in ALL:
        for kind in ("contig", "transposed", "step2_inner", "expand_col"):
            x = I.make_view((6, 12, 16), dt, kind, seed=410, specials=0.02)
            for dims in ([0], [1, 2], [0, 1, 2], [-1], [], [-2]):
                paths.add(check_remap("flip", x, dims, what=kind))
            for shifts, dims in (([1], [0]), ([-2, 3], [1, 2]), ([7, 0, -13], [0, 1, 2]), ([2], [-1]), ([1, 2], [1, 1]), ([12], [1])):
                paths.add(check_remap("roll", x, shifts, dims, what=kind))
        for shape in ((), (1,), (0, 3), (5, 0), (257,), (3, 1000)):
            x = I.typed(shape, dt, seed=411)
            check_remap("flip", x, [0] if len(shape) else [0])
            check_remap("roll", x, [3], [-1])
    assert {"remap", "remap-vec"} <= paths, paths
    x = I.typed((2, 3, 4), F32, seed=412)
    for args in (("flip", [3]), ("flip", [0, 0]), ("flip", [1, -2]), ("roll", [1], [-4])):
        check_remap(args[0], x, *args[1:])
    with pytest.raises(B.TxError) as e:
        B.tx_flip(torch.zeros(2, 3, device="cuda", dtype=BF16), torch.zeros(2, 3, device="cuda"), [0])
    assert e.value.kind == "DTYPE"
    d = torch.zeros(4, 4, device="cuda")
    with pytest.raises(B.TxError) as e:
        B.tx_flip(d, d, [0])
    assert e.value.kind == "OVERLAP"


def test_tril_triu_sweep():
    for dt in ALL:
        for kind in ("contig", "transposed", "step2_inner"):
            x = I.make_view((3, 9, 16), dt, kind, seed=413, specials=0.02)
            for k in (0, 1, -2, 4, -9, 17):
                check_remap("tril", x, k, what=kind)
                check_remap("triu", x, k, what=kind)
        t = I.typed((2, 3, 7, 5), dt, seed=414)
        for k in (0, 2, -3):
            check_remap("tril", t, k)
            check_remap("triu", t.transpose(2, 3), k)
        check_remap("tril", I.typed((0, 3), dt, seed=415), 0)
        check_remap("triu", I.typed((5,), dt, seed=416), 0)                       # fewer than two dims: refused
    nan = torch.full((4, 4), float("nan"))
    check_remap("tril", nan, 0, what="zeros are written, not multiplied in")


@pytest.mark.parametrize("op", ["flip_outer", "flip_inner", "roll_outer", "roll_inner", "tril", "triu"])
def test_remap_full_size(op):
    x = I.typed((8192, 8192), F32, seed=417, specials=0.01)
    if op == "flip_outer":
        assert check_remap("flip", x, [0]) == "remap-vec"
    elif op == "flip_inner":
        assert check_remap("flip", x, [1]) == "remap-vec"
    elif op == "roll_outer":
        assert check_remap("roll", x, [1234], [0]) == "remap-vec"
    elif op == "roll_inner":
        assert check_remap("roll", x, [-777], [1]) == "remap"
    else:
        assert check_remap(op, x, 5) == "remap-vec"
        check_remap(op, I.typed((4, 2048, 2048), BF16, seed=418), -3)
