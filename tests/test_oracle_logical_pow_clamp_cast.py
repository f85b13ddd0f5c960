"""Pins for the oracle's logical family, pow, clamp and `out=` casting.

More members of the paper's "Elementwise" category (Table 1) and the two ways
an ATen operator can write into a tensor of another dtype (an explicit `out=`
tensor, an in-place variant).  The paper delegates the definitions to the ATen
CPU operators (Section 3.2); expected values here are truth tables, Python's
exact integers, the special-value table of C Annex F, mpmath at 50 digits and
hand-worked roundings - nothing comes from the oracle itself or from the HIP
library.
"""
import math
import random
import struct

import mpmath
import pytest
import torch

from oracle import oracle as O

F32, BF16, F16, I32, I64, B = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool
NAN, INF = float("nan"), float("inf")


def f32(x):
    return struct.unpack("<f", struct.pack("<f", x))[0]


def bits32(x):
    return struct.unpack("<I", struct.pack("<f", x))[0]


def ulps(a, b):
    def key(v):
        u = bits32(v)
        return (u & 0x7FFFFFFF) if u < 0x80000000 else -(u & 0x7FFFFFFF)
    return abs(key(a) - key(b))


def same(got, want):
    """Equal values, NaN == NaN, signed zeros distinguished."""
    if isinstance(want, float) and math.isnan(want):
        return math.isnan(got)
    return got == want and math.copysign(1, got) == math.copysign(1, want)


# --------------------------------------------------------------------------- logical family
@pytest.mark.parametrize("dt", [B, I32, I64, F16, BF16, F32])
def test_logical_truth_tables(dt):
    vals = [0, 1] if dt == B else [0, 3, -2] if not dt.is_floating_point else [0.0, -0.0, 2.5, NAN, -INF]
    truth = lambda v: not (v == 0)                      # a NaN is not zero
    a = torch.tensor([x for x in vals for _ in vals], dtype=dt)
    b = torch.tensor([y for _ in vals for y in vals], dtype=dt)
    pairs = [(x, y) for x in vals for y in vals]
    for name, fn in (("logical_and", lambda p, q: p and q), ("logical_or", lambda p, q: p or q),
                     ("logical_xor", lambda p, q: p != q)):
        got = O.binary(name, a, b)
        assert got.dtype == B
        assert got.tolist() == [fn(truth(x), truth(y)) for x, y in pairs], name
    got = O.unary("logical_not", torch.tensor(vals, dtype=dt))
    assert got.dtype == B and got.tolist() == [not truth(v) for v in vals]


def test_logical_mixed_dtypes_and_broadcast():
    a = torch.tensor([[0.0], [1e-30], [NAN]], dtype=F32)
    b = torch.tensor([0, 7], dtype=I64)
    assert O.binary("logical_or", a, b).tolist() == [[False, True], [True, True], [True, True]]
    assert O.binary("logical_and", a, b).tolist() == [[False, False], [False, True], [False, True]]
    # a tiny 0-dim fp32 operand is converted to the bf16 common dtype first, where it is zero
    tiny = torch.tensor(1e-45, dtype=F32)
    assert O.binary("logical_or", torch.zeros(2, dtype=BF16), tiny).tolist() == [False, False]


# --------------------------------------------------------------------------- pow
ANNEX_F = [
    (NAN, 0.0, 1.0), (NAN, -0.0, 1.0), (1.0, NAN, 1.0), (1.0, INF, 1.0), (-1.0, INF, 1.0), (-1.0, -INF, 1.0),
    (0.0, -1.0, INF), (-0.0, -3.0, -INF), (-0.0, -2.0, INF), (0.0, 2.0, 0.0), (-0.0, 3.0, -0.0), (-0.0, 2.0, 0.0),
    (-2.0, 3.0, -8.0), (-2.0, 2.0, 4.0), (-2.0, 0.5, NAN), (-8.0, 1.0 / 3.0, NAN), (0.5, INF, 0.0), (2.0, INF, INF),
    (0.5, -INF, INF), (2.0, -INF, 0.0), (INF, -1.0, 0.0), (INF, 2.0, INF), (-INF, 3.0, -INF), (-INF, 2.0, INF),
    (-INF, -3.0, -0.0), (NAN, 1.0, NAN), (2.0, NAN, NAN), (2.0, 10.0, 1024.0), (9.0, 0.5, 3.0), (2.0, -2.0, 0.25),
    (10.0, 38.0, f32(1e38)), (10.0, 39.0, INF), (2.0, -149.0, 2.0 ** -149), (2.0, -151.0, 0.0),
]


def test_pow_special_values():
    a = torch.tensor([r[0] for r in ANNEX_F], dtype=F32)
    b = torch.tensor([r[1] for r in ANNEX_F], dtype=F32)
    got = O.binary("pow", a, b).tolist()
    for (x, y, want), g in zip(ANNEX_F, got):
        if want == f32(1e38):
            assert ulps(g, want) <= 1, (x, y, g)
        else:
            assert same(g, want), (x, y, g, want)


def test_pow_fp32_matches_mpmath_within_half_ulp():
    mpmath.mp.dps = 50
    rng = random.Random(5)
    xs = [f32(rng.uniform(0.01, 30.0)) for _ in range(400)]
    ys = [f32(rng.uniform(-12.0, 12.0)) for _ in range(400)]
    got = O.binary("pow", torch.tensor(xs, dtype=F32), torch.tensor(ys, dtype=F32)).tolist()
    for x, y, g in zip(xs, ys, got):
        exact = mpmath.power(mpmath.mpf(x), mpmath.mpf(y))
        want = f32(float(exact))
        assert ulps(g, want) <= 1                       # the double rounding through binary64 can only move a tie
        assert abs(mpmath.mpf(g) - exact) <= abs(exact) * mpmath.mpf(2) ** -23 * mpmath.mpf("0.5001")


def test_pow_half_operands_round_once_from_the_exact_power():
    mpmath.mp.dps = 50
    x = torch.tensor([1.5, 2.25, 0.3, 7.0], dtype=BF16)
    y = torch.tensor([2.5, -1.5, 3.0, 0.5], dtype=BF16)
    got = O.binary("pow", x, y)
    assert got.dtype == BF16
    for xv, yv, g in zip(x.tolist(), y.tolist(), got.tolist()):
        exact = float(mpmath.power(mpmath.mpf(xv), mpmath.mpf(yv)))
        assert g == torch.tensor(exact, dtype=torch.float64).to(BF16).item()


def test_pow_integers_are_python_powers_modulo_two_to_the_width():
    rng = random.Random(9)
    base = [rng.randint(-9, 9) for _ in range(300)] + [2, 3, -3, 7]
    expo = [rng.randint(0, 40) for _ in range(300)] + [63, 41, 41, 0]
    for dt, bits in ((I32, 32), (I64, 64)):
        got = O.binary("pow", torch.tensor(base, dtype=dt), torch.tensor(expo, dtype=dt)).tolist()
        for bb, e, g in zip(base, expo, got):
            want = pow(bb, e) % (1 << bits)
            want -= (1 << bits) if want >= (1 << (bits - 1)) else 0
            assert g == want, (bb, e, dt)


def test_pow_integer_negative_exponent_and_dtype_rules():
    b = torch.tensor([1, -1, -1, 2, 0, -5], dtype=I64)
    e = torch.tensor([-7, -3, -4, -1, -2, -1], dtype=I64)
    assert O.binary("pow", b, e).tolist() == [1, -1, 1, 0, 0, 0]     # trunc(1 / b^|e|), and 0 for a zero base
    # integer with floating operand computes in the floating dtype; bool with bool is refused
    r = O.binary("pow", torch.tensor([2, 3], dtype=I32), torch.tensor([0.5, 2.0], dtype=F32))
    assert r.dtype == F32 and r.tolist() == [f32(math.sqrt(2.0)), 9.0]
    r = O.binary("pow", torch.tensor([True, False]), torch.tensor([2, 0], dtype=I32))
    assert r.dtype == I32 and r.tolist() == [1, 1]
    with pytest.raises(O.OracleError) as ei:
        O.binary("pow", torch.tensor([True]), torch.tensor([True]))
    assert ei.value.kind == "dtype"


# --------------------------------------------------------------------------- clamp
def py_clamp(v, lo, hi):
    if isinstance(v, float) and math.isnan(v):
        return v
    if lo is not None and v < lo:
        v = lo
    if hi is not None and v > hi:
        v = hi
    return v


@pytest.mark.parametrize("lo,hi", [(-1.5, 2.0), (None, 0.25), (0.5, None), (3.0, -3.0), (0.0, 0.0)])
def test_clamp_float_brute_force(lo, hi):
    vals = [-INF, -7.0, -1.5, -0.0, 0.0, 0.375, 2.0, 2.5, INF, NAN]
    got = O.clamp(torch.tensor(vals, dtype=F32), lo, hi).tolist()
    for v, g in zip(vals, got):
        assert same(g, py_clamp(v, lo, hi)), (v, lo, hi, g)


def test_clamp_integers_and_promotion():
    x = torch.tensor([-2 ** 31, -5, 0, 9, 2 ** 31 - 1], dtype=I32)
    assert O.clamp(x, -5, 9).tolist() == [-5, -5, 0, 9, 9]
    assert O.clamp(x, None, -6).tolist() == [-2 ** 31, -6, -6, -6, -6]
    assert O.clamp(x, 7, 3).tolist() == [3] * 5                      # lower above upper: the upper bound everywhere
    r = O.clamp(x, -0.5, 8.5)                                        # floating bound: fp32 result
    assert r.dtype == F32 and r.tolist() == [-0.5, -0.5, 0.0, 8.5, 8.5]
    big = torch.tensor([-2 ** 62, 2 ** 62], dtype=I64)
    assert O.clamp(big, -2 ** 40, 2 ** 41).tolist() == [-2 ** 40, 2 ** 41]


def test_clamp_bounds_are_converted_to_the_result_dtype():
    # 0.1 is not a bf16 value: the bound becomes bf16(0.1) = 0.10009765625 before it is applied
    x = torch.tensor([0.0, 0.1001, 0.5], dtype=BF16)
    got = O.clamp(x, 0.1, None)
    assert got.dtype == BF16 and got.tolist() == [0.10009765625, 0.10009765625, 0.5]
    # fp32: 0.1 becomes the binary32 value of 0.1
    assert O.clamp(torch.tensor([0.0], dtype=F32), 0.1, None).item() == f32(0.1)


def test_clamp_nan_bound_and_errors():
    x = torch.tensor([1.0, NAN, -3.0], dtype=F32)
    assert all(math.isnan(v) for v in O.clamp(x, NAN, 2.0).tolist())
    assert all(math.isnan(v) for v in O.clamp(x, None, NAN).tolist())
    for args, kind in (((torch.tensor([True]), 0, 1), "dtype"), ((x, None, None), "scalar"),
                       ((torch.tensor([1], dtype=I32), 2 ** 31, None), "scalar")):
        with pytest.raises(O.OracleError) as ei:
            O.clamp(*args)
        assert ei.value.kind == kind


# --------------------------------------------------------------------------- out= casting
def test_cast_rules_table():
    one = {dt: torch.ones(2, dtype=dt) for dt in (B, I32, I64, F16, BF16, F32)}
    order = {B: 0, I32: 1, I64: 1, F16: 2, BF16: 2, F32: 2}
    for src in (I32, I64, F16, BF16, F32):
        for dst in one:
            ok = not (order[src] == 2 and order[dst] < 2) and not (dst == B)
            try:
                O.binary("add", one[src], one[src], out_dtype=dst)
                assert ok, (src, dst)
            except O.OracleError as e:
                assert not ok and e.kind == "dtype", (src, dst)
    # a bool result (comparison, logical op, bool arithmetic) can go anywhere
    for dst in one:
        r = O.binary("lt", torch.tensor([1, 5], dtype=I32), torch.tensor([3, 3], dtype=I32), out_dtype=dst)
        assert r.tolist() == [1, 0] and r.dtype == dst
        r = O.unary("logical_not", torch.tensor([0.0, 2.0]), out_dtype=dst)
        assert r.tolist() == [1, 0]


def test_result_is_rounded_to_the_result_dtype_before_the_cast():
    # bf16: 1 + 2^-9 is not representable, the bf16 sum is 1; an fp32 out tensor must hold 1, not 1.001953125
    a = torch.tensor([1.0, 256.0], dtype=BF16)
    b = torch.tensor([2.0 ** -9, 1.0], dtype=BF16)
    r = O.binary("add", a, b, out_dtype=F32)
    assert r.dtype == F32 and r.tolist() == [1.0, 256.0]            # 257 is the bf16 tie 256 | 258 -> even 256
    # int32 wraps before it widens
    r = O.binary("add", torch.tensor([2 ** 31 - 1], dtype=I32), torch.tensor([1], dtype=I32), out_dtype=I64)
    assert r.tolist() == [-2 ** 31]
    # int64 result narrowed to int32 keeps the low 32 bits
    r = O.binary("mul", torch.tensor([2 ** 20 + 1], dtype=I64), torch.tensor([2 ** 20], dtype=I64), out_dtype=I32)
    assert r.tolist() == [2 ** 20]
    # fp32 result into a half tensor: one further rounding
    r = O.unary("exp", torch.tensor([1.0], dtype=F32), out_dtype=F16)
    assert r.item() == torch.tensor(f32(math.e), dtype=F32).to(F16).item()


def test_integer_to_half_goes_through_binary32():
    # 2^24 + 2^16 + 1 lies above the bf16 tie 2^24 + 2^16 and would round up if converted directly; binary32
    # first drops the final 1 (a tie, to even), which lands exactly on the bf16 tie, which then goes to even: 2^24
    v = 2 ** 24 + 2 ** 16 + 1
    r = O.binary("add", torch.tensor([v], dtype=I64), torch.tensor([0], dtype=I64), out_dtype=BF16)
    assert r.item() == float(2 ** 24)
    r = O.unary("neg", torch.tensor([-v], dtype=I64), out_dtype=BF16)
    assert r.item() == float(2 ** 24)


def test_out_casting_agrees_with_the_aten_cpu_operators():
    """The definition the paper points to (Section 3.2): the ATen CPU operator itself, called with out=."""
    g = torch.Generator().manual_seed(3)
    xb, yb = torch.randn(257, generator=g).to(BF16), torch.randn(257, generator=g).to(BF16)
    xi, yi = torch.randint(-2 ** 31, 2 ** 31, (257,), generator=g, dtype=I64).to(I32), \
        torch.randint(-2 ** 31, 2 ** 31, (257,), generator=g, dtype=I64).to(I32)
    for op, fn in (("add", torch.add), ("sub", torch.sub), ("mul", torch.mul), ("maximum", torch.maximum)):
        for a, b, dst in ((xb, yb, F32), (xb, yb, F16), (xi, yi, I64), (xi, yi, F32), (xi, yi, BF16)):
            want = torch.empty(257, dtype=dst)
            fn(a, b, out=want)
            assert torch.equal(O.binary(op, a, b, out_dtype=dst), want), (op, dst)
    # in-place variant: a.add_(b) with a wider b computes in fp32 and rounds into a
    xf = torch.randn(257, generator=g)
    want = xb.clone().add_(xf)
    assert torch.equal(O.binary("add", xb, xf, out_dtype=BF16), want)
    with pytest.raises(RuntimeError):
        xi.clone().add_(xf)                                           # a floating result cannot go into an integer tensor
    with pytest.raises(O.OracleError):
        O.binary("add", xi, xf, out_dtype=I32)


def test_logical_pow_clamp_agree_with_the_aten_cpu_operators():
    g = torch.Generator().manual_seed(4)
    x, y = torch.randn(300, generator=g), torch.randn(300, generator=g)
    x[::7] = 0.0
    y[::5] = 0.0
    for name, fn in (("logical_and", torch.logical_and), ("logical_or", torch.logical_or),
                     ("logical_xor", torch.logical_xor)):
        assert torch.equal(O.binary(name, x, y), fn(x, y))
    assert torch.equal(O.unary("logical_not", x), torch.logical_not(x))
    assert torch.equal(O.clamp(x, -0.3, 0.8), torch.clamp(x, -0.3, 0.8))
    assert torch.equal(O.clamp(x.to(BF16), -0.3, 0.8), torch.clamp(x.to(BF16), -0.3, 0.8))
    xi = torch.randint(-50, 50, (300,), generator=g)
    assert torch.equal(O.clamp(xi, -7, 9), torch.clamp(xi, -7, 9))
    r = O.clamp(xi, -7.5, 9)
    assert r.dtype == torch.clamp(xi, -7.5, 9).dtype and torch.equal(r, torch.clamp(xi, -7.5, 9))
    bi, ei = torch.randint(-6, 7, (300,), generator=g), torch.randint(-3, 12, (300,), generator=g)
    assert torch.equal(O.binary("pow", bi, ei), torch.pow(bi, ei))
    p, q = x.abs() + 0.1, y * 3
    got, lib = O.binary("pow", p, q), torch.pow(p, q)
    assert max(ulps(a, b) for a, b in zip(got.tolist(), lib.tolist())) <= 1
