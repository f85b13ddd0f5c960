"""Pins for the oracle's unary operators with scalar parameters (leaky_relu elu celu selu softplus threshold hardshrink
softshrink logit nan_to_num) and the ternary addcmul / addcdiv / lerp.

More of the paper's "Deep Learning" and "Elementwise" categories (Table 1).  Expected values: mpmath at 40 digits, exact
rational arithmetic, truth tables over the special values, and the ATen CPU operators (Section 3.2) - nothing comes
from the oracle or the HIP library.
"""
import math
import random
import struct
from fractions import Fraction

import mpmath
import pytest
import torch
import torch.nn.functional as NF

from oracle import oracle as O

F32, BF16, F16, I32, I64, B = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool
ALL = (B, I32, I64, F16, BF16, F32)
NAN, INF = float("nan"), float("inf")
SELU_SCALE, SELU_ALPHA = mpmath.mpf("1.0507009873554804934193349852946"), mpmath.mpf("1.6732632423543772848170429916717")


def f32(x):
    return struct.unpack("<f", struct.pack("<f", x))[0]


def round_f32(fr):
    return torch.tensor(float(fr), dtype=torch.float64).float().item()


def close_half_ulp(g, exact, what):
    assert abs(mpmath.mpf(g) - exact) <= abs(exact) * mpmath.mpf(2) ** -23 * mpmath.mpf("0.5001") + mpmath.mpf(2) ** -150, what


MP = {
    "elu": (lambda x, p: x if x > 0 else p[0] * mpmath.expm1(x), (1.5,)),
    "celu": (lambda x, p: x if x > 0 else p[0] * mpmath.expm1(x / p[0]), (2.5,)),
    "selu": (lambda x, p: SELU_SCALE * (x if x > 0 else SELU_ALPHA * mpmath.expm1(x)), ()),
    "softplus": (lambda x, p: x if x * p[0] > p[1] else mpmath.log(1 + mpmath.exp(x * p[0])) / p[0], (2.0, 15.0)),
    "logit": (lambda x, p: mpmath.log(x / (1 - x)), ()),
    "leaky_relu": (lambda x, p: x if x > 0 else x * mpmath.mpf(p[0]), (0.01,)),
}


@pytest.mark.parametrize("op", sorted(MP))
def test_parametrised_functions_match_mpmath(op):
    mpmath.mp.dps = 40
    rng = random.Random(81)
    fn, params = MP[op]
    lo, hi = (0.0001, 0.9999) if op == "logit" else (-20.0, 20.0)
    xs = [f32(rng.uniform(lo, hi)) for _ in range(300)] + ([f32(1e-6), f32(-1e-6), f32(-80.0)] if op != "logit" else [f32(1e-30)])
    got = O.unary_param(op, torch.tensor(xs, dtype=F32), *params).tolist()
    for x, g in zip(xs, got):
        close_half_ulp(g, fn(mpmath.mpf(x), params), (op, x, g))


def test_piecewise_tables_and_special_values():
    x = torch.tensor([-3.0, -0.0, 0.0, 0.4, 5.0, NAN, INF, -INF], dtype=F32)
    lr = O.unary_param("leaky_relu", x, 0.5).tolist()
    assert lr[:5] == [-1.5, -0.0, 0.0, f32(0.4), 5.0] and math.isnan(lr[5]) and lr[6:] == [INF, -INF] and math.copysign(1, lr[1]) == -1
    assert O.unary_param("leaky_relu", x, -2.0).tolist()[0] == 6.0 and O.unary_param("leaky_relu", x, -2.0).tolist()[7] == INF
    th = O.unary_param("threshold", x, 0.3, 9.0).tolist()
    assert th[:5] == [9.0, 9.0, 9.0, f32(0.4), 5.0] and math.isnan(th[5]) and th[6:] == [INF, 9.0]   # a NaN is not at or below the threshold: it stays
    hs = O.unary_param("hardshrink", x, 0.5).tolist()
    assert hs[:5] == [-3.0, 0.0, 0.0, 0.0, 5.0] and math.isnan(hs[5]) and hs[6:] == [INF, -INF] and math.copysign(1, hs[1]) == 1
    assert O.unary_param("hardshrink", x, -1.0).tolist()[3] == f32(0.4)                          # an empty interval
    ss = O.unary_param("softshrink", x, 0.5).tolist()
    assert ss[:5] == [-2.5, -0.0, 0.0, 0.0, 4.5] and math.isnan(ss[5]) and ss[6:] == [INF, -INF] and math.copysign(1, ss[1]) == -1
    assert O.unary_param("softshrink", x, 0.0).tolist()[3] == f32(0.4)
    e = O.unary_param("elu", x, 1.5).tolist()
    assert e[1:5] == [-0.0, 0.0, f32(0.4), 5.0] and math.isnan(e[5]) and e[6:] == [INF, -1.5] and math.copysign(1, e[1]) == -1
    assert O.unary_param("celu", x, 2.0).tolist()[7] == -2.0 and O.unary_param("celu", x, -1.0).tolist()[7] == -INF
    sp = O.unary_param("softplus", x, 1.0, 20.0).tolist()
    assert sp[6] == INF and sp[7] == 0.0 and math.isnan(sp[5]) and sp[2] == f32(math.log(2))
    assert O.unary_param("softplus", torch.tensor([25.0, 19.0]), 1.0, 20.0).tolist() == [25.0, round_f32(Fraction(19) + Fraction(math.log1p(math.exp(-19.0))))]
    lg = O.unary_param("logit", torch.tensor([0.0, 0.25, 1.0, 1.5, NAN, -0.5])).tolist()
    assert lg[0] == -INF and lg[2] == INF and all(math.isnan(v) for v in lg[3:]) and lg[1] == f32(math.log(1 / 3))
    lge = O.unary_param("logit", torch.tensor([0.0, 0.25, 1.0, 1.5, NAN, -0.5]), 0.125, 1).tolist()
    assert lge[0] == lge[5] == f32(math.log(0.125 / 0.875)) and lge[2] == lge[3] == f32(math.log(0.875 / 0.125)) and math.isnan(lge[4])
    assert O.unary_param("logit", torch.tensor([0.25]), 0.75, 1).item() == f32(math.log(3.0))     # eps > 1/2: the lower bound wins
    n2n = O.unary_param("nan_to_num", x, 0.0, 3.4028234663852886e38, -3.4028234663852886e38).tolist()
    assert n2n == [-3.0, -0.0, 0.0, f32(0.4), 5.0, 0.0, 3.4028234663852886e38, -3.4028234663852886e38]
    assert O.unary_param("nan_to_num", x, 1.0, 2.0, -3.0).tolist()[5:] == [1.0, 2.0, -3.0]
    assert O.unary_param("nan_to_num", torch.tensor([NAN, INF], dtype=F16), 0.0, 1e9, -1e9).tolist() == [0.0, INF]   # rounded to the dtype
    # integers
    assert O.unary_param("threshold", torch.tensor([-3, 0, 5], dtype=I32), 1, 7).tolist() == [7, 7, 5]
    assert O.unary_param("threshold", torch.tensor([-3, 0, 5]), 0.5, 2.5).tolist() == [2, 2, 5]               # parameters truncated
    assert O.unary_param("nan_to_num", torch.tensor([-3, 5], dtype=I32)).tolist() == [-3, 5]
    assert O.unary_param("nan_to_num", torch.tensor([True, False])).tolist() == [True, False]
    r = O.unary_param("logit", torch.tensor([0, 1]))
    assert r.dtype == F32 and r.tolist() == [-INF, INF]
    for op, p in (("celu", (0.0,)), ("softshrink", (-1.0,)), ("softshrink", (NAN,))):
        with pytest.raises(O.OracleError) as e:
            O.unary_param(op, torch.ones(3), *p)
        assert e.value.kind == "scalar"
    with pytest.raises(O.OracleError):
        O.unary_param("prelu", torch.ones(3))


def test_unary_param_dtype_rules_against_aten():
    aten = {"leaky_relu": (lambda t: NF.leaky_relu(t, 0.1), (0.1,)), "elu": (lambda t: NF.elu(t, 1.5), (1.5,)),
            "celu": (lambda t: NF.celu(t, 2.0), (2.0,)), "selu": (NF.selu, ()), "softplus": (lambda t: NF.softplus(t, 2.0, 5.0), (2.0, 5.0)),
            "threshold": (lambda t: NF.threshold(t, 1, 7), (1, 7)), "hardshrink": (lambda t: NF.hardshrink(t, 0.5), (0.5,)),
            "softshrink": (lambda t: NF.softshrink(t, 0.5), (0.5,)), "logit": (lambda t: torch.logit(t, 0.1), (0.1, 1)),
            "nan_to_num": (lambda t: torch.nan_to_num(t, 1.0, 2.0, -3.0), (1.0, 2.0, -3.0))}
    g = torch.Generator().manual_seed(82)
    for op, (fn, params) in aten.items():
        for dt in ALL:
            x = (torch.randn(64, generator=g) * 2).to(dt) if dt.is_floating_point else torch.randint(-3, 4, (64,), generator=g).to(dt)
            try:
                want = fn(x)
            except RuntimeError:
                with pytest.raises(O.OracleError) as e:
                    O.unary_param(op, x, *params)
                assert e.value.kind == "dtype", (op, dt)
                continue
            got = O.unary_param(op, x, *params)
            assert got.dtype == want.dtype, (op, dt)
            tol = 1e-2 if dt in (F16, BF16) else 2e-6
            assert torch.allclose(got.double(), want.double(), rtol=tol, atol=tol, equal_nan=True), (op, dt)
    sp = torch.tensor([NAN, INF, -INF, 0.0, -0.0, 0.3, -0.3, 100.0, -100.0])
    for op, (fn, params) in aten.items():
        assert torch.allclose(O.unary_param(op, sp, *params), fn(sp), rtol=2e-6, atol=1e-30, equal_nan=True), op


def test_ternary_exact_and_against_aten():
    rng = random.Random(83)
    a = [f32(rng.uniform(-3, 3)) for _ in range(200)]
    b = [f32(rng.uniform(-3, 3)) for _ in range(200)]
    c = [f32(rng.uniform(0.1, 3) * rng.choice([1, -1])) for _ in range(200)]
    ta, tb, tc = torch.tensor(a), torch.tensor(b), torch.tensor(c)
    v = 0.375
    got = O.ternary("addcmul", ta, tb, tc, v).tolist()
    for x, y, z, g in zip(a, b, c, got):
        assert g == round_f32(Fraction(x) + Fraction(v) * Fraction(y) * Fraction(z))
    got = O.ternary("addcdiv", ta, tb, tc, v).tolist()
    for x, y, z, g in zip(a, b, c, got):
        exact = Fraction(x) + Fraction(v) * Fraction(y) / Fraction(z)
        assert abs(Fraction(g) - exact) <= abs(exact) * Fraction(1, 2 ** 23) * Fraction(51, 100) + Fraction(1, 2 ** 140)
    w = [f32(rng.uniform(-0.5, 1.5)) for _ in range(200)]
    got = O.ternary("lerp", ta, tb, torch.tensor(w)).tolist()
    for x, y, z, g in zip(a, b, w, got):
        fx, fy, fz = Fraction(x), Fraction(y), Fraction(z)
        exact = fx + fz * (fy - fx)                                       # the two branches are the same polynomial
        assert abs(Fraction(g) - exact) <= (abs(fx) + abs(fy)) * Fraction(1, 2 ** 23), (x, y, z, g)
    assert O.ternary("lerp", ta, tb, None, 0.0).tolist() == a and O.ternary("lerp", ta, tb, None, 1.0).tolist() == b    # exact at both ends
    assert torch.allclose(O.ternary("lerp", ta, tb, None, 0.3), torch.lerp(ta, tb, 0.3), rtol=2e-6, atol=1e-6)
    # integers wrap, the scalar is truncated; broadcasting; promotion; errors
    i = torch.tensor([-3, 0, 5, 2 ** 31 - 1], dtype=I32)
    assert O.ternary("addcmul", i, i, i, 2).tolist() == [15, 0, 55, ((2 ** 31 - 1) + 2 * (2 ** 31 - 1) ** 2 + 2 ** 31) % 2 ** 32 - 2 ** 31]
    assert O.ternary("addcmul", i, i, i, 0.5).tolist() == i.tolist()
    g = torch.Generator().manual_seed(84)
    x, y, z = torch.randn(4, 1, 6, generator=g), torch.randn(5, 1, generator=g), torch.randn(6, generator=g) + 3
    for op, fn in (("addcmul", torch.addcmul), ("addcdiv", torch.addcdiv)):
        want = fn(x, y, z, value=-1.25)
        got = O.ternary(op, x, y, z, -1.25)
        assert got.shape == want.shape and torch.allclose(got, want, rtol=2e-6, atol=1e-6)
        mixed = fn(x, torch.tensor([2, 3, 4, 5, 6]).view(5, 1), z.to(BF16))
        gm = O.ternary(op, x, torch.tensor([2, 3, 4, 5, 6]).view(5, 1), z.to(BF16))
        assert gm.dtype == mixed.dtype == F32 and torch.allclose(gm, mixed, rtol=2e-6, atol=1e-6)
        hb = fn(x.to(BF16), y.to(BF16), z.to(BF16))
        assert torch.allclose(O.ternary(op, x.to(BF16), y.to(BF16), z.to(BF16)).double(), hb.double(), rtol=2e-2, atol=2e-2)
    want = torch.lerp(x.expand(4, 5, 6), y.expand(4, 5, 6), z.expand(4, 5, 6).contiguous() / 6)
    assert torch.allclose(O.ternary("lerp", x, y, z / 6), want, rtol=2e-6, atol=1e-6)
    for args in (("addcmul", torch.tensor([True]), torch.tensor([True]), torch.tensor([True])), ("addcdiv", i, i, i),
                 ("lerp", i, i, None), ("lerp", x, y.to(BF16), None), ("lerp", x, y, z.to(F16))):
        with pytest.raises(O.OracleError) as e:
            O.ternary(*args)
        assert e.value.kind == "dtype", args[0]
    with pytest.raises(O.OracleError) as e:
        O.ternary("addcmul", torch.ones(3), torch.ones(4), torch.ones(3))
    assert e.value.kind == "shape"
    sp = O.ternary("lerp", torch.tensor([1.0, 1.0, NAN]), torch.tensor([3.0, INF, 1.0]), torch.tensor([1.0, 0.0, 0.5])).tolist()
    assert sp[0] == 3.0 and math.isnan(sp[1]) and math.isnan(sp[2])                               # 0 * inf


def test_round_decimals_and_gelu_tanh():
    mpmath.mp.dps = 40
    rng = random.Random(85)
    # round(x, decimals): binary32 arithmetic is the definition; ATen's CPU operator follows the same steps
    x = torch.tensor([f32(rng.uniform(-3000, 3000)) for _ in range(400)] + [1.2345, -2.5, 1250.0, 0.5, 15.0, 25.0, 0.125, -0.0, NAN, INF], dtype=F32)
    for d in (0, 1, 2, 3, -1, -2, -3):
        got = O.unary_param("round_decimals", x, d)
        want = torch.round(x, decimals=d)
        assert torch.equal(got.nan_to_num(7.0), want.nan_to_num(7.0)), d
        assert torch.equal(O.unary_param("round_decimals", x.to(BF16), d).float().nan_to_num(7.0), torch.round(x.to(BF16), decimals=d).float().nan_to_num(7.0)), d
    t = O.unary_param("round_decimals", torch.tensor([1.2345, -2.5, 1250.0, 0.125, 15.0, 25.0]), 2).tolist()
    assert t == [f32(1.23), -2.5, 1250.0, f32(0.12), 15.0, 25.0]                                  # 12.5 -> 12: halves to even
    assert O.unary_param("round_decimals", torch.tensor([15.0, 25.0, 35.0, -15.0]), -1).tolist() == [20.0, 20.0, 40.0, -20.0]
    assert torch.equal(O.unary_param("round_decimals", x[:400], 0), O.unary("round", x[:400]))
    for bad in (0.5, 39.0, NAN):
        with pytest.raises(O.OracleError) as e:
            O.unary_param("round_decimals", torch.ones(3), bad)
        assert e.value.kind == "scalar"
    with pytest.raises(O.OracleError) as e:
        O.unary_param("round_decimals", torch.tensor([1, 2]), 1)
    assert e.value.kind == "dtype"
    # tanh gelu: x (1 + tanh u) / 2 at 40 digits; relative accuracy also deep in the negative tail
    xs = [f32(rng.uniform(-9, 9)) for _ in range(300)] + [f32(-12.0), f32(-6.5), f32(1e-6), f32(-1e-6), f32(30.0)]
    got = O.unary_param("gelu_tanh", torch.tensor(xs, dtype=F32)).tolist()
    c = mpmath.sqrt(2 / mpmath.pi)
    for v, g in zip(xs, got):
        u = c * (mpmath.mpf(v) + mpmath.mpf("0.044715") * mpmath.mpf(v) ** 3)
        close_half_ulp(g, mpmath.mpf(v) * (1 + mpmath.tanh(u)) / 2, (v, g))
    sp = O.unary_param("gelu_tanh", torch.tensor([0.0, -0.0, INF, -INF, NAN, -100.0])).tolist()
    assert sp[0] == 0.0 and sp[2] == INF and math.isnan(sp[3]) and math.isnan(sp[4]) and sp[5] == 0.0 and math.copysign(1, sp[5]) == -1
    g = torch.Generator().manual_seed(86)
    for dt in (F32, BF16, F16):
        t = (torch.randn(500, generator=g) * 3).to(dt)
        tol = 2e-6 if dt == F32 else 1e-2
        assert torch.allclose(O.unary_param("gelu_tanh", t).double(), NF.gelu(t, approximate="tanh").double(), rtol=tol, atol=tol)
