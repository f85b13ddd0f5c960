"""Pins for the oracle's fourth batch of elementwise operators: tan asin acos atan sinh cosh asinh acosh atanh erf
erfc relu frac signbit hardswish hardsigmoid mish, and the binary fmod remainder hypot copysign logaddexp logaddexp2
xlogy heaviside fmax fmin nextafter gcd lcm bitwise_left_shift bitwise_right_shift.

More of the paper's largest category (Table 1, "Elementwise", 161 operators).  Expected values: mpmath at 50 digits,
exact integer and rational arithmetic in Python, truth tables over the special values, struct-level bit stepping,
and the ATen CPU operators for the dtype rules (Section 3.2) - nothing comes from the oracle or the HIP library.
"""
import math
import random
import struct
from fractions import Fraction

import mpmath
import pytest
import torch

from oracle import oracle as O

F32, BF16, F16, I32, I64, B = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool
ALL = (B, I32, I64, F16, BF16, F32)
NAN, INF = float("nan"), float("inf")


def f32(x):
    return struct.unpack("<f", struct.pack("<f", x))[0]


def close_half_ulp(g, exact, what):
    if abs(exact) > mpmath.mpf(3.4028235e38):
        assert math.isinf(g), what
        return
    assert abs(mpmath.mpf(g) - exact) <= abs(exact) * mpmath.mpf(2) ** -23 * mpmath.mpf("0.5001") + mpmath.mpf(2) ** -150, what


MP = {
    "tan": (mpmath.tan, (-1.5, 1.5)), "asin": (mpmath.asin, (-1.0, 1.0)), "acos": (mpmath.acos, (-1.0, 1.0)),
    "atan": (mpmath.atan, (-50.0, 50.0)), "sinh": (mpmath.sinh, (-20.0, 20.0)), "cosh": (mpmath.cosh, (-20.0, 20.0)),
    "asinh": (mpmath.asinh, (-1e4, 1e4)), "acosh": (mpmath.acosh, (1.0, 1e4)), "atanh": (mpmath.atanh, (-0.999, 0.999)),
    "erf": (mpmath.erf, (-4.0, 4.0)), "erfc": (mpmath.erfc, (-3.0, 9.0)),
    "mish": (lambda v: v * mpmath.tanh(mpmath.log(1 + mpmath.exp(v))), (-30.0, 30.0)),
    "hardsigmoid": (lambda v: min(max(v + 3, 0), 6) / 6, (-5.0, 5.0)),
    "hardswish": (lambda v: v * min(max(v + 3, 0), 6) / 6, (-5.0, 5.0)),
}


@pytest.mark.parametrize("op", sorted(MP))
def test_float_functions_match_mpmath_within_half_ulp(op):
    mpmath.mp.dps = 50
    rng = random.Random(41)
    fn, (lo, hi) = MP[op]
    xs = [f32(rng.uniform(lo, hi)) for _ in range(300)] + [f32(v) for v in (lo * 0.5, hi * 0.5, hi * 1e-3, hi * 1e-20)]
    xs = [x for x in xs if lo <= x <= hi]
    got = O.unary(op, torch.tensor(xs, dtype=F32)).tolist()
    for x, g in zip(xs, got):
        close_half_ulp(g, fn(mpmath.mpf(x)), (op, x, g))


def test_unary_special_values_and_dtype_rules():
    t = lambda *v: torch.tensor(v, dtype=F32)
    pi = math.pi
    assert O.unary("tan", t(0.0, -0.0)).tolist() == [0.0, -0.0] and math.isnan(O.unary("tan", t(INF)).item())
    assert O.unary("asin", t(1.0, -1.0, 0.0)).tolist() == [f32(pi / 2), f32(-pi / 2), 0.0] and math.isnan(O.unary("asin", t(1.5)).item())
    assert O.unary("acos", t(1.0, -1.0)).tolist() == [0.0, f32(pi)] and math.isnan(O.unary("acos", t(-1.5)).item())
    assert O.unary("atan", t(INF, -INF, 0.0)).tolist() == [f32(pi / 2), f32(-pi / 2), 0.0]
    assert O.unary("sinh", t(0.0, INF, -INF, 100.0)).tolist() == [0.0, INF, -INF, INF]
    assert O.unary("cosh", t(0.0, INF, -INF)).tolist() == [1.0, INF, INF]
    assert O.unary("asinh", t(0.0, INF, -INF)).tolist() == [0.0, INF, -INF]
    assert O.unary("acosh", t(1.0, INF)).tolist() == [0.0, INF] and math.isnan(O.unary("acosh", t(0.5)).item())
    assert O.unary("atanh", t(0.0, 1.0, -1.0)).tolist() == [0.0, INF, -INF] and math.isnan(O.unary("atanh", t(1.5)).item())
    assert O.unary("erf", t(0.0, INF, -INF, 10.0)).tolist() == [0.0, 1.0, -1.0, 1.0]
    assert O.unary("erfc", t(0.0, INF, -INF, 30.0)).tolist() == [1.0, 0.0, 2.0, 0.0]
    assert O.unary("mish", t(0.0, INF, 100.0)).tolist() == [0.0, INF, 100.0] and math.isnan(O.unary("mish", t(-INF)).item())  # -inf * 0
    assert O.unary("hardsigmoid", t(-3.0, 3.0, 0.0, -INF, INF, 9.0)).tolist() == [0.0, 1.0, 0.5, 0.0, 1.0, 1.0]
    hs = O.unary("hardswish", t(-3.0, 3.0, 0.0, -4.0, 7.0, INF)).tolist()
    assert hs == [-0.0, 3.0, 0.0, -0.0, 7.0, INF] and math.copysign(1, hs[0]) == -1.0                                    # -3 * 0 / 6
    assert math.isnan(O.unary("hardswish", t(-INF)).item())                                                            # -inf * 0
    for op in sorted(MP) + ["relu", "frac"]:
        assert math.isnan(O.unary(op, t(NAN)).item()), op
    # relu keeps -0.0 and NaN, zeroes the negatives; integers too; bool refused
    r = O.unary("relu", t(-0.0, -1.0, 2.5, -INF, INF)).tolist()
    assert r == [-0.0, 0.0, 2.5, 0.0, INF] and math.copysign(1, r[0]) == -1.0 and math.copysign(1, r[1]) == 1.0
    assert O.unary("relu", torch.tensor([-5, 0, 7], dtype=I32)).tolist() == [0, 0, 7]
    assert O.unary("relu", torch.tensor([-2 ** 63, 2 ** 63 - 1])).tolist() == [0, 2 ** 63 - 1]
    # frac: x - trunc(x), sign of x, exact
    fr = O.unary("frac", t(2.75, -2.75, 5.0, -0.0, 1e10, f32(0.1))).tolist()
    assert fr == [0.75, -0.75, 0.0, 0.0, 0.0, f32(0.1)]
    assert math.isnan(O.unary("frac", t(INF)).item()) and math.isnan(O.unary("frac", t(-INF)).item())
    # signbit: the bit itself
    neg_nan = struct.unpack("<f", struct.pack("<I", 0xFFC00000))[0]
    assert O.unary("signbit", t(-0.0, 0.0, -1.0, 1.0, -INF, NAN, neg_nan)).tolist() == [True, False, True, False, True, False, True]
    assert O.unary("signbit", torch.tensor([-1, 0, 1], dtype=I32)).tolist() == [True, False, False]
    assert O.unary("signbit", torch.tensor([True, False])).tolist() == [False, False]
    assert O.unary("signbit", torch.tensor([-0.0, 2.0], dtype=BF16)).tolist() == [True, False]
    # dtype rules against the ATen CPU operators
    import torch.nn.functional as NF
    aten = {"tan": torch.tan, "asin": torch.asin, "acos": torch.acos, "atan": torch.atan, "sinh": torch.sinh, "cosh": torch.cosh,
            "asinh": torch.asinh, "acosh": torch.acosh, "atanh": torch.atanh, "erf": torch.erf, "erfc": torch.erfc,
            "relu": torch.relu, "frac": torch.frac, "signbit": torch.signbit, "hardswish": NF.hardswish,
            "hardsigmoid": NF.hardsigmoid, "mish": NF.mish}
    for op, fn in aten.items():
        for dt in ALL:
            x = torch.tensor([0, 1, 1, 0]).to(dt)
            try:
                want = fn(x)
            except RuntimeError:
                with pytest.raises(O.OracleError) as e:
                    O.unary(op, x)
                assert e.value.kind == "dtype", (op, dt)
                continue
            got = O.unary(op, x)
            assert got.dtype == want.dtype, (op, dt)
            assert torch.allclose(got.double(), want.double(), rtol=1e-2 if dt in (F16, BF16) else 1e-6, equal_nan=True), (op, dt)
    # half types: one rounding from the exact value of the rounded input
    x = torch.tensor([0.3, 1.7, -2.2], dtype=F16)
    want = torch.tensor([math.erf(v) for v in x.tolist()], dtype=torch.float64).to(F16)
    assert torch.equal(O.unary("erf", x), want)


def py_fmod(a, b):
    r = abs(a) % abs(b)
    return -r if a < 0 else r


def py_gcd_wrapped(a, b, bits):
    g = math.gcd(a, b)
    return (g + 2 ** (bits - 1)) % 2 ** bits - 2 ** (bits - 1)


def test_fmod_remainder_exact():
    rng = random.Random(42)
    for dt, bits in ((I32, 32), (I64, 64)):
        a = [rng.randrange(-2 ** (bits - 1), 2 ** (bits - 1)) for _ in range(300)] + [-2 ** (bits - 1), 5, -5, 5, -5, 0]
        b = [rng.choice([1, -1]) * rng.randrange(1, 2 ** rng.randrange(1, bits - 1)) for _ in range(300)] + [-1, 3, 3, -3, -3, 7]
        ta, tb = torch.tensor(a, dtype=dt), torch.tensor(b, dtype=dt)
        assert O.binary("fmod", ta, tb).tolist() == [py_fmod(x, y) for x, y in zip(a, b)]
        assert O.binary("remainder", ta, tb).tolist() == [x % y for x, y in zip(a, b)]          # Python's % has the divisor's sign
        with pytest.raises(O.OracleError) as e:
            O.binary("fmod", ta, torch.zeros(1, dtype=dt))
        assert e.value.kind == "scalar"
        with pytest.raises(O.OracleError):
            O.binary("remainder", ta[:3], torch.tensor([1, 0, 2], dtype=dt))
    # floats: exact rational remainder (always representable), then the divisor's sign for remainder
    a = [f32(rng.uniform(-1e4, 1e4)) for _ in range(300)] + [f32(1e30), 6.0, -6.0, 5.5]
    b = [f32(rng.choice([1, -1]) * rng.uniform(1e-3, 1e2)) for _ in range(300)] + [f32(3.3), -3.0, 3.0, -2.0]
    fm = O.binary("fmod", torch.tensor(a), torch.tensor(b)).tolist()
    rm = O.binary("remainder", torch.tensor(a), torch.tensor(b)).tolist()
    for x, y, g, h in zip(a, b, fm, rm):
        fx, fy = Fraction(x), Fraction(y)
        q = abs(fx) // abs(fy)
        r = abs(fx) - q * abs(fy)
        r = -r if fx < 0 else r
        assert Fraction(g) == r, (x, y, g)
        want = r + fy if (r != 0 and ((r < 0) != (fy < 0))) else r
        assert h == torch.tensor(float(want), dtype=torch.float64).float().item(), (x, y, h)
    t = lambda *v: torch.tensor(v, dtype=F32)
    got = O.binary("fmod", t(5.0, -5.0, INF, 5.0, -0.0, NAN), t(0.0, INF, 2.0, -INF, 2.0, 1.0)).tolist()
    assert math.isnan(got[0]) and got[1] == -5.0 and math.isnan(got[2]) and got[3] == 5.0 and math.isnan(got[5])
    assert got[4] == 0.0 and math.copysign(1, got[4]) == -1.0
    got = O.binary("remainder", t(5.0, -5.0, INF, 5.0, 6.0, -1.0), t(0.0, INF, 2.0, -INF, -3.0, 3.0)).tolist()
    assert math.isnan(got[0]) and got[1] == INF and math.isnan(got[2]) and got[3] == -INF and got[4] == 0.0 and got[5] == 2.0
    with pytest.raises(O.OracleError) as e:
        O.binary("fmod", torch.tensor([True]), torch.tensor([True]))
    assert e.value.kind == "dtype"
    r = O.binary("remainder", torch.tensor([True, False]), torch.tensor([-3, 5], dtype=I32))
    assert r.dtype == I32 and r.tolist() == [-2, 0]


BIN_MP = {
    "hypot": lambda a, b: mpmath.sqrt(a * a + b * b),
    "logaddexp": lambda a, b: mpmath.log(mpmath.exp(a) + mpmath.exp(b)),
    "logaddexp2": lambda a, b: mpmath.log(mpmath.power(2, a) + mpmath.power(2, b), 2),
    "xlogy": lambda a, b: a * mpmath.log(b),
}


@pytest.mark.parametrize("op", sorted(BIN_MP))
def test_binary_float_functions_match_mpmath(op):
    mpmath.mp.dps = 60
    rng = random.Random(43)
    if op == "xlogy":
        a = [f32(rng.uniform(-10, 10)) for _ in range(300)]
        b = [f32(rng.uniform(1e-3, 100)) for _ in range(300)]
    elif op == "hypot":
        a = [f32(rng.uniform(-1, 1) * 10.0 ** rng.randrange(-18, 19)) for _ in range(300)]
        b = [f32(rng.uniform(-1, 1) * 10.0 ** rng.randrange(-18, 19)) for _ in range(300)]
    else:
        a = [f32(rng.uniform(-80, 80)) for _ in range(300)] + [f32(-1000.0), f32(1000.0), f32(3.0)]
        b = [f32(rng.uniform(-80, 80)) for _ in range(300)] + [f32(-1001.0), f32(999.5), f32(3.0)]
    got = O.binary(op, torch.tensor(a), torch.tensor(b)).tolist()
    for x, y, g in zip(a, b, got):
        close_half_ulp(g, BIN_MP[op](mpmath.mpf(x), mpmath.mpf(y)), (op, x, y, g))


def test_binary_float_special_values():
    t = lambda *v: torch.tensor(v, dtype=F32)
    h = O.binary("hypot", t(INF, NAN, 3e38, 3.0, NAN), t(NAN, -INF, 3e38, 4.0, 1.0)).tolist()
    assert h[:4] == [INF, INF, INF, 5.0] and math.isnan(h[4])
    c = O.binary("copysign", t(1.0, -1.0, 2.0, 0.0, INF), t(-0.0, NAN, -3.0, -1.0, -1.0)).tolist()
    assert c == [-1.0, 1.0, -2.0, -0.0, -INF] and math.copysign(1, c[3]) == -1.0
    cn = O.binary("copysign", t(NAN), t(-1.0))
    assert math.isnan(cn.item()) and struct.unpack("<I", struct.pack("<f", cn.item()))[0] >> 31 == 1
    ci = O.binary("copysign", torch.tensor([3, -3], dtype=I32), torch.tensor([-1, 1], dtype=I64))
    assert ci.dtype == F32 and ci.tolist() == [-3.0, 3.0]
    for op in ("logaddexp", "logaddexp2"):
        g = O.binary(op, t(INF, -INF, INF, NAN, -INF, 5.0), t(INF, -INF, -INF, 1.0, 2.0, NAN)).tolist()
        assert g[:3] == [INF, -INF, INF] and math.isnan(g[3]) and g[4] == 2.0 and math.isnan(g[5]), op
        with pytest.raises(O.OracleError) as e:
            O.binary(op, torch.tensor([1]), torch.tensor([2]))
        assert e.value.kind == "dtype"
    assert O.binary("logaddexp2", t(3.0, 0.0), t(3.0, 0.0)).tolist() == [4.0, 1.0]
    x = O.binary("xlogy", t(0.0, 0.0, 1.0, 0.0, NAN, 2.0, 0.0), t(NAN, -1.0, -1.0, 0.0, 0.0, 0.0, INF)).tolist()
    assert math.isnan(x[0]) and x[1] == 0.0 and math.isnan(x[2]) and x[3] == 0.0 and math.isnan(x[4]) and x[5] == -INF and x[6] == 0.0
    xi = O.binary("xlogy", torch.tensor([0, 2]), torch.tensor([0, 1]))
    assert xi.dtype == F32 and xi.tolist() == [0.0, 0.0]
    hv = O.binary("heaviside", t(NAN, 0.0, -0.0, 2.0, -1.0, INF, -INF), t(7.0)).tolist()
    assert hv == [0.0, 7.0, 7.0, 1.0, 0.0, 1.0, 0.0]
    assert O.binary("heaviside", torch.tensor([-2, 0, 3], dtype=I32), torch.tensor([9, 9, 9], dtype=I32)).tolist() == [0, 9, 1]
    assert O.binary("heaviside", torch.tensor([True, False]), torch.tensor([False, False])).tolist() == [True, False]
    assert O.binary("heaviside", torch.tensor([True, False]), torch.tensor([True, True])).tolist() == [True, True]
    with pytest.raises(O.OracleError) as e:
        O.binary("heaviside", torch.tensor([1], dtype=I32), torch.tensor([1], dtype=I64))
    assert e.value.kind == "dtype"
    fm = O.binary("fmax", t(NAN, NAN, 1.0, -INF, 2.0), t(1.0, NAN, NAN, 3.0, -5.0)).tolist()
    assert fm[0] == 1.0 and math.isnan(fm[1]) and fm[2:] == [1.0, 3.0, 2.0]
    fn = O.binary("fmin", t(NAN, NAN, 1.0, -INF, 2.0), t(1.0, NAN, NAN, 3.0, -5.0)).tolist()
    assert fn[0] == 1.0 and math.isnan(fn[1]) and fn[2:] == [1.0, -INF, -5.0]
    assert O.binary("fmax", torch.tensor([3, -7], dtype=I32), torch.tensor([-4, 9])).tolist() == [3, 9]
    assert O.binary("fmin", torch.tensor([True, True]), torch.tensor([True, False])).tolist() == [True, False]


def step_bits(x, toward, fmt):
    """Python model of nextafter on an IEEE encoding: fmt = (struct code for the integer, pack, unpack)."""
    to_bits, from_bits, nbits = fmt
    if math.isnan(x) or math.isnan(toward):
        return NAN
    if x == toward:
        return toward
    if x == 0:
        return from_bits(1 | ((1 << (nbits - 1)) if toward < 0 else 0))
    u = to_bits(x)
    return from_bits(u + 1 if (x < toward) == (x > 0) else u - 1)


FMT32 = (lambda v: struct.unpack("<I", struct.pack("<f", v))[0], lambda u: struct.unpack("<f", struct.pack("<I", u))[0], 32)
FMT16 = (lambda v: struct.unpack("<H", struct.pack("<e", v))[0], lambda u: struct.unpack("<e", struct.pack("<H", u))[0], 16)


def test_nextafter_steps_one_encoding():
    rng = random.Random(44)
    a = [f32(rng.uniform(-1, 1) * 10.0 ** rng.randrange(-40, 38)) for _ in range(300)]
    b = [f32(rng.uniform(-1, 1) * 10.0 ** rng.randrange(-40, 38)) for _ in range(300)]
    a += [0.0, -0.0, 1.0, INF, f32(3.4028234663852886e38), 1.0, NAN, f32(1e-45), -INF, 2.0]
    b += [1.0, -1.0, 1.0, 0.0, INF, NAN, 1.0, 0.0, INF, 2.0]
    got = O.binary("nextafter", torch.tensor(a), torch.tensor(b)).tolist()
    for x, y, g in zip(a, b, got):
        want = step_bits(x, y, FMT32)
        assert (math.isnan(g) and math.isnan(want)) or (g == want and math.copysign(1, g) == math.copysign(1, want)), (x, y, g, want)
    # the C library's float routine agrees (through ATen's CPU operator)
    assert torch.equal(torch.tensor(got[:300]), torch.nextafter(torch.tensor(a[:300]), torch.tensor(b[:300])))
    # fp16: the same stepping on the 16-bit encoding
    a16 = [0.0, 1.0, 65504.0, -65504.0, 6e-8, -1.0, 1.0, 0.5]
    b16 = [1.0, 2.0, INF, -INF, 0.0, 0.0, 1.0, -3.0]
    got = O.binary("nextafter", torch.tensor(a16, dtype=F16), torch.tensor(b16, dtype=F16)).tolist()
    assert got == [step_bits(torch.tensor(x, dtype=F16).item(), y, FMT16) for x, y in zip(a16, b16)]
    # bf16: one step is 2^-7 relative above 1, 2^-8 below
    g = O.binary("nextafter", torch.tensor([1.0, 1.0, 0.0], dtype=BF16), torch.tensor([2.0, 0.0, -1.0], dtype=BF16))
    assert g.dtype == BF16 and g.double().tolist() == [1.0 + 2.0 ** -7, 1.0 - 2.0 ** -8, -(2.0 ** -133)]
    with pytest.raises(O.OracleError):
        O.binary("nextafter", torch.tensor([1]), torch.tensor([2]))


def test_gcd_lcm_shifts_exact():
    rng = random.Random(45)
    for dt, bits in ((I32, 32), (I64, 64)):
        wrap = lambda v: (v + 2 ** (bits - 1)) % 2 ** bits - 2 ** (bits - 1)
        a = [rng.randrange(-2 ** rng.randrange(1, bits - 1), 2 ** rng.randrange(1, bits - 1)) for _ in range(300)] + [0, 0, -12, 7, -2 ** (bits - 1)]
        b = [rng.randrange(-2 ** rng.randrange(1, bits - 1), 2 ** rng.randrange(1, bits - 1)) for _ in range(300)] + [0, 9, 18, 0, 6]
        ta, tb = torch.tensor(a, dtype=dt), torch.tensor(b, dtype=dt)
        assert O.binary("gcd", ta, tb).tolist() == [wrap(math.gcd(x, y)) for x, y in zip(a, b)]
        assert O.binary("lcm", ta, tb).tolist() == [wrap(math.lcm(x, y)) for x, y in zip(a, b)]
        assert O.binary("gcd", torch.tensor([-2 ** (bits - 1)], dtype=dt), torch.tensor([0], dtype=dt)).item() == -2 ** (bits - 1)
        s = [rng.randrange(0, bits) for _ in range(300)] + [bits - 1, bits, -1, bits + 8, 0]
        v = [rng.randrange(-2 ** (bits - 1), 2 ** (bits - 1)) for _ in range(300)] + [1, 1, -1, -8, -8]
        tv, ts = torch.tensor(v, dtype=dt), torch.tensor(s, dtype=dt)
        assert O.binary("bitwise_left_shift", tv, ts).tolist() == [wrap(x << k) if 0 <= k < bits else 0 for x, k in zip(v, s)]
        assert O.binary("bitwise_right_shift", tv, ts).tolist() == [(x >> k) if 0 <= k < bits else (-1 if x < 0 else 0) for x, k in zip(v, s)]
        # ATen's CPU operators on in-range operands (the out-of-range rows as well: same rule)
        assert torch.equal(O.binary("bitwise_left_shift", tv, ts), torch.bitwise_left_shift(tv, ts))
        assert torch.equal(O.binary("bitwise_right_shift", tv, ts), torch.bitwise_right_shift(tv, ts))
        assert torch.equal(O.binary("gcd", ta[:300], tb[:300]), torch.gcd(ta[:300], tb[:300]))
        assert torch.equal(O.binary("lcm", ta[:300], tb[:300]).abs(), torch.lcm(ta[:300], tb[:300]).abs())
    for op in ("gcd", "lcm", "bitwise_left_shift", "bitwise_right_shift"):
        for args in ((torch.ones(2), torch.ones(2)), (torch.tensor([True]), torch.tensor([True])), (torch.ones(2, dtype=I32), torch.ones(2))):
            with pytest.raises(O.OracleError) as e:
                O.binary(op, *args)
            assert e.value.kind == "dtype", op
    r = O.binary("gcd", torch.tensor([True, False]), torch.tensor([6, 4], dtype=I32))      # a bool promotes to the integer dtype
    assert r.dtype == I32 and r.tolist() == [1, 4]


def test_binary_dtype_rules_against_aten_and_out_casting():
    names = ["fmod", "remainder", "hypot", "copysign", "logaddexp", "logaddexp2", "xlogy", "heaviside", "fmax", "fmin", "nextafter",
             "gcd", "lcm", "bitwise_left_shift", "bitwise_right_shift"]
    for op in names:
        fn = getattr(torch, op)
        for da in ALL:
            for db in ALL:
                a, b = torch.tensor([3, 1, 2]).to(da), torch.tensor([2, 1, 1]).to(db)
                try:
                    want = fn(a, b)
                except RuntimeError:
                    with pytest.raises(O.OracleError) as e:
                        O.binary(op, a, b)
                    assert e.value.kind == "dtype", (op, da, db)
                    continue
                got = O.binary(op, a, b)
                assert got.dtype == want.dtype, (op, da, db)
                assert torch.allclose(got.double(), want.double(), rtol=1e-2 if want.dtype in (F16, BF16) else 1e-6), (op, da, db)
    # out= casting: the value in the result dtype, then converted
    a, b = torch.tensor([5.5, -5.5], dtype=BF16), torch.tensor([2.0, 2.0], dtype=BF16)
    out = torch.empty(2, dtype=F32)
    assert O.binary("remainder", a, b, out=out).tolist() == [1.5, 0.5]
    with pytest.raises(O.OracleError):
        O.binary("hypot", a, b, out=torch.empty(2, dtype=I32))
    assert O.binary("gcd", torch.tensor([12]), torch.tensor([18]), out=torch.empty(1, dtype=F32)).item() == 6.0
    assert O.unary("relu", torch.tensor([-2, 3], dtype=I32), out=torch.empty(2, dtype=F16)).tolist() == [0.0, 3.0]
    assert O.unary("signbit", torch.tensor([-2.0, 3.0]), out=torch.empty(2, dtype=I64)).tolist() == [1, 0]
