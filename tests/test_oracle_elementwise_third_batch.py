"""Pins for the oracle's third batch of elementwise operators: sin cos exp2 log2 log10 rsqrt reciprocal silu square
sign floor ceil trunc round isnan isinf isfinite bitwise_not, and the binary bitwise_and / or / xor and atan2.

More of the paper's largest category (Table 1, "Elementwise", 161 operators).  Expected values: mpmath at 50 digits,
exact integers, truth tables over the special values, and the ATen CPU operators for the dtype rules (Section 3.2) -
nothing comes from the oracle or the HIP library.
"""
import math
import random
import struct

import mpmath
import pytest
import torch

from oracle import oracle as O

F32, BF16, F16, I32, I64, B = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool
ALL = (B, I32, I64, F16, BF16, F32)
NAN, INF = float("nan"), float("inf")


def f32(x):
    return struct.unpack("<f", struct.pack("<f", x))[0]


MP = {
    "sin": mpmath.sin, "cos": mpmath.cos, "exp2": lambda v: mpmath.power(2, v), "log2": lambda v: mpmath.log(v, 2),
    "log10": mpmath.log10, "rsqrt": lambda v: 1 / mpmath.sqrt(v), "reciprocal": lambda v: 1 / v,
    "silu": lambda v: v / (1 + mpmath.exp(-v)),
}


@pytest.mark.parametrize("op", sorted(MP))
def test_float_functions_match_mpmath_within_half_ulp(op):
    mpmath.mp.dps = 50
    rng = random.Random(31)
    positive = op in ("log2", "log10", "rsqrt")
    xs = [f32(rng.uniform(0.001, 50.0) if positive else rng.uniform(-30.0, 30.0)) for _ in range(300)]
    xs += [f32(v) for v in (1e-30, 1e30, 0.5, 1.0, 2.0)] if positive else [f32(v) for v in (1e-30, -1e-30, 1e4, -87.0, 88.0)]
    got = O.unary(op, torch.tensor(xs, dtype=F32)).tolist()
    for x, g in zip(xs, got):
        exact = MP[op](mpmath.mpf(x))
        if abs(exact) > mpmath.mpf(3.4e38):
            assert math.isinf(g)
            continue
        assert abs(mpmath.mpf(g) - exact) <= abs(exact) * mpmath.mpf(2) ** -23 * mpmath.mpf("0.5001") + mpmath.mpf(2) ** -150, (op, x, g)


def test_float_function_special_values():
    t = lambda *v: torch.tensor(v, dtype=F32)
    assert O.unary("sin", t(0.0, -0.0)).tolist() == [0.0, -0.0] and math.isnan(O.unary("sin", t(INF)).item())
    assert O.unary("cos", t(0.0)).item() == 1.0 and math.isnan(O.unary("cos", t(-INF)).item())
    assert O.unary("exp2", t(10.0, -1.0, -INF, 128.0, -150.0)).tolist() == [1024.0, 0.5, 0.0, INF, 0.0]
    assert O.unary("log2", t(8.0, 0.0, INF)).tolist() == [3.0, -INF, INF] and math.isnan(O.unary("log2", t(-1.0)).item())
    assert O.unary("log10", t(1000.0, 0.0)).tolist() == [3.0, -INF]
    assert O.unary("rsqrt", t(4.0, 0.0, INF)).tolist() == [0.5, INF, 0.0] and math.isnan(O.unary("rsqrt", t(-1.0)).item())
    assert O.unary("reciprocal", t(4.0, -0.0, INF)).tolist() == [0.25, -INF, 0.0]
    assert O.unary("silu", t(0.0, -INF)).tolist()[0] == 0.0 and math.isnan(O.unary("silu", t(-INF)).item())   # -inf * 0
    assert O.unary("silu", t(INF, 100.0)).tolist() == [INF, 100.0]
    for op in MP:
        assert math.isnan(O.unary(op, t(NAN)).item()), op
    # integers and bools compute in fp32; silu refuses them
    assert O.unary("exp2", torch.tensor([3, 0])).dtype == F32 and O.unary("exp2", torch.tensor([3, 0])).tolist() == [8.0, 1.0]
    assert O.unary("reciprocal", torch.tensor([True, False])).tolist() == [1.0, INF]
    with pytest.raises(O.OracleError):
        O.unary("silu", torch.tensor([1, 2]))
    # half types: one rounding from the exact value of the rounded input
    x = torch.tensor([0.3, 1.7, -2.2], dtype=BF16)
    want = torch.tensor([math.sin(v) for v in x.tolist()], dtype=torch.float64).to(BF16)
    assert torch.equal(O.unary("sin", x), want)


def test_square_sign_rounding_family_tables():
    x = torch.tensor([NAN, -0.0, 0.0, 2.5, -2.5, 0.5, 1.5, -0.5, -INF, INF, 3.999, -3.001], dtype=F32)
    got = {op: O.unary(op, x).tolist() for op in ("sign", "floor", "ceil", "trunc", "round")}
    assert got["sign"][1:] == [0.0, 0.0, 1.0, -1.0, 1.0, 1.0, -1.0, -1.0, 1.0, 1.0, -1.0] and got["sign"][0] == 0.0
    assert math.copysign(1, got["sign"][1]) == 1.0                                   # (0 < x) - (x < 0) of -0.0 is +0.0
    assert got["floor"][1:] == [-0.0, 0.0, 2.0, -3.0, 0.0, 1.0, -1.0, -INF, INF, 3.0, -4.0]
    assert got["ceil"][1:] == [-0.0, 0.0, 3.0, -2.0, 1.0, 2.0, -0.0, -INF, INF, 4.0, -3.0]
    assert got["trunc"][1:] == [-0.0, 0.0, 2.0, -2.0, 0.0, 1.0, -0.0, -INF, INF, 3.0, -3.0]
    assert got["round"][1:] == [-0.0, 0.0, 2.0, -2.0, 0.0, 2.0, -0.0, -INF, INF, 4.0, -3.0]   # halves to even
    for op in ("floor", "ceil", "trunc", "round"):
        assert math.isnan(got[op][0]) and math.copysign(1, got[op][1]) == -1.0, op       # the sign of zero is kept
    assert math.copysign(1, got["ceil"][7]) == -1.0 and math.copysign(1, got["round"][7]) == -1.0
    # squares: exact product rounded once; integers wrap; a bool becomes the int64 0 / 1
    v = [f32(1.0 + 2.0 ** -12), f32(3.1), f32(-1e20), f32(1e-30)]
    from fractions import Fraction
    sq = O.unary("square", torch.tensor(v, dtype=F32)).tolist()
    for a, g in zip(v, sq):
        exact = Fraction(a) * Fraction(a)
        assert g == (torch.tensor(float(exact), dtype=torch.float64).float().item() if exact < Fraction(3.5e38) else INF)
    assert O.unary("square", torch.tensor([70000, -3], dtype=I32)).tolist() == [(70000 * 70000 + 2 ** 31) % 2 ** 32 - 2 ** 31, 9]
    assert O.unary("square", torch.tensor([3037000500], dtype=I64)).item() == (3037000500 ** 2 + 2 ** 63) % 2 ** 64 - 2 ** 63
    r = O.unary("square", torch.tensor([True, False]))
    assert r.dtype == I64 and r.tolist() == [1, 0]
    assert O.unary("sign", torch.tensor([-7, 0, 9], dtype=I32)).tolist() == [-1, 0, 1]
    assert O.unary("sign", torch.tensor([True, False])).tolist() == [True, False]
    for op in ("floor", "ceil", "trunc", "round"):
        assert O.unary(op, torch.tensor([-7, 0, 9])).tolist() == [-7, 0, 9]
        with pytest.raises(O.OracleError):
            O.unary(op, torch.tensor([True]))


def test_classification_and_bitwise():
    x = torch.tensor([NAN, INF, -INF, 0.0, -1.5, 3e38], dtype=F32)
    assert O.unary("isnan", x).tolist() == [True, False, False, False, False, False]
    assert O.unary("isinf", x).tolist() == [False, True, True, False, False, False]
    assert O.unary("isfinite", x).tolist() == [False, False, False, True, True, True]
    for dt in (I32, I64, B):
        v = torch.tensor([0, 1], dtype=dt)
        assert O.unary("isnan", v).tolist() == [False, False] and O.unary("isfinite", v).tolist() == [True, True]
    rng = random.Random(32)
    for dt, bits in ((I32, 32), (I64, 64)):
        a = [rng.randrange(-2 ** (bits - 1), 2 ** (bits - 1)) for _ in range(200)]
        b = [rng.randrange(-2 ** (bits - 1), 2 ** (bits - 1)) for _ in range(200)]
        ta, tb = torch.tensor(a, dtype=dt), torch.tensor(b, dtype=dt)
        assert O.binary("bitwise_and", ta, tb).tolist() == [x & y for x, y in zip(a, b)]
        assert O.binary("bitwise_or", ta, tb).tolist() == [x | y for x, y in zip(a, b)]
        assert O.binary("bitwise_xor", ta, tb).tolist() == [x ^ y for x, y in zip(a, b)]
        assert O.unary("bitwise_not", ta).tolist() == [~x for x in a]
    p, q = torch.tensor([True, True, False, False]), torch.tensor([True, False, True, False])
    assert O.binary("bitwise_and", p, q).tolist() == [True, False, False, False]
    assert O.binary("bitwise_xor", p, q).tolist() == [False, True, True, False]
    assert O.unary("bitwise_not", p).tolist() == [False, False, True, True]
    r = O.binary("bitwise_or", p, torch.tensor([4, 4, 4, 4], dtype=I32))           # bool promotes to the integer dtype
    assert r.dtype == I32 and r.tolist() == [5, 5, 4, 4]
    for args in (("bitwise_and", torch.ones(2), torch.ones(2)), ("bitwise_or", torch.ones(2, dtype=I32), torch.ones(2))):
        with pytest.raises(O.OracleError) as e:
            O.binary(*args)
        assert e.value.kind == "dtype"
    with pytest.raises(O.OracleError):
        O.unary("bitwise_not", torch.ones(2))


def test_atan2_quadrants_special_values_and_mpmath():
    mpmath.mp.dps = 50
    pi = math.pi
    y = torch.tensor([0.0, -0.0, 1.0, -1.0, 0.0, -0.0, INF, -INF, INF, 1.0, NAN], dtype=F32)
    x = torch.tensor([-1.0, -1.0, 0.0, 0.0, 1.0, 1.0, INF, -INF, 1.0, INF, 1.0], dtype=F32)
    got = O.binary("atan2", y, x).tolist()
    want = [pi, -pi, pi / 2, -pi / 2, 0.0, -0.0, pi / 4, -3 * pi / 4, pi / 2, 0.0]
    for g, w in zip(got, want):
        assert g == f32(w) and math.copysign(1, g) == math.copysign(1, w)
    assert math.isnan(got[-1])
    rng = random.Random(33)
    ys, xs = [f32(rng.uniform(-9, 9)) for _ in range(300)], [f32(rng.uniform(-9, 9)) for _ in range(300)]
    for a, b, g in zip(ys, xs, O.binary("atan2", torch.tensor(ys), torch.tensor(xs)).tolist()):
        exact = mpmath.atan2(mpmath.mpf(a), mpmath.mpf(b))
        assert abs(mpmath.mpf(g) - exact) <= abs(exact) * mpmath.mpf(2) ** -23 * mpmath.mpf("0.5001")
    r = O.binary("atan2", torch.tensor([1, 0]), torch.tensor([0, -1]))
    assert r.dtype == F32 and r.tolist() == [f32(pi / 2), f32(pi)]


def test_dtype_rules_agree_with_the_aten_cpu_operators():
    fns = {"sin": torch.sin, "cos": torch.cos, "exp2": torch.exp2, "log2": torch.log2, "log10": torch.log10, "rsqrt": torch.rsqrt,
           "reciprocal": torch.reciprocal, "silu": torch.nn.functional.silu, "square": torch.square, "sign": torch.sign,
           "floor": torch.floor, "ceil": torch.ceil, "trunc": torch.trunc, "round": torch.round, "isnan": torch.isnan,
           "isinf": torch.isinf, "isfinite": torch.isfinite, "bitwise_not": torch.bitwise_not}
    for op, fn in fns.items():
        for dt in ALL:
            x = torch.ones(3, dtype=dt)
            try:
                want = fn(x).dtype
            except RuntimeError:
                want = None
            try:
                got = O.unary(op, x).dtype
            except O.OracleError:
                got = None
            assert got == want, (op, dt, got, want)
    for op, fn in (("bitwise_and", torch.bitwise_and), ("bitwise_or", torch.bitwise_or), ("bitwise_xor", torch.bitwise_xor),
                   ("atan2", torch.atan2)):
        for da in ALL:
            for db in ALL:
                a, b = torch.ones(3, dtype=da), torch.ones(3, dtype=db)
                try:
                    want = fn(a, b).dtype
                except RuntimeError:
                    want = None
                try:
                    got = O.binary(op, a, b).dtype
                except O.OracleError:
                    got = None
                assert got == want, (op, da, db, got, want)
