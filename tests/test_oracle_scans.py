"""Pins for the oracle's further scans: cumprod and logcumsumexp along one dim.

The scan family of the hot path (cumsum with decoupled look-back) with two more combining operations.  Expected values:
exact integer and rational products in Python, mpmath logarithms of exact sums, shift invariance, special-value tables,
and the ATen CPU operators (Section 3.2) - nothing comes from the oracle or the HIP library.
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
NAN, INF = float("nan"), float("inf")


def f32(x):
    return struct.unpack("<f", struct.pack("<f", x))[0]


def test_cumprod_exact_integers_and_rationals():
    rng = random.Random(71)
    wrap = lambda v: (v + 2 ** 63) % 2 ** 64 - 2 ** 63
    for dt in (I32, I64):
        rows = [[rng.randrange(-9, 10) for _ in range(40)] for _ in range(5)]
        rows[2] = [rng.randrange(-2 ** 30, 2 ** 30) for _ in range(40)]          # wraps after a few factors
        got = O.scan("cumprod", torch.tensor(rows, dtype=dt), 1)
        assert got.dtype == I64
        for r, g in zip(rows, got.tolist()):
            p, want = 1, []
            for v in r:
                p *= v
                want.append(wrap(p))
            assert g == want
    assert O.scan("cumprod", torch.tensor([True, True, False, True])).tolist() == [1, 1, 0, 0]
    # floats: the exact rational product, rounded once per prefix
    r = [f32(rng.uniform(0.5, 1.5)) * rng.choice([1, -1]) for _ in range(60)]
    got = O.scan("cumprod", torch.tensor(r, dtype=F32)).tolist()
    p = Fraction(1)
    for v, g in zip(r, got):
        p *= Fraction(v)
        assert abs(Fraction(g) - p) <= abs(p) * Fraction(1, 2 ** 23) * Fraction(501, 1000), (g, float(p))
    # along other dims, through views, half types with an fp32 out
    g = torch.Generator().manual_seed(72)
    x = torch.rand(6, 7, 5, generator=g) + 0.5
    for dim in (0, 1, 2, -1, -3):
        assert torch.allclose(O.scan("cumprod", x, dim), torch.cumprod(x, dim), rtol=2e-6)
        assert torch.allclose(O.scan("cumprod", x.transpose(0, 2)[::2], dim), torch.cumprod(x.transpose(0, 2)[::2], dim), rtol=2e-6)
    h = (torch.rand(4, 9, generator=g) + 0.5).to(BF16)
    assert torch.equal(O.scan("cumprod", h, 1, out_dtype=F32), torch.cumprod(h.double(), 1).float())
    assert torch.equal(O.scan("cumprod", h, 1), torch.cumprod(h.double(), 1).to(BF16))
    sp = O.scan("cumprod", torch.tensor([2.0, INF, 0.0, 3.0, NAN])).tolist()
    assert sp[:2] == [2.0, INF] and all(math.isnan(v) for v in sp[2:])               # inf * 0
    assert O.scan("cumprod", torch.tensor(3.5)).item() == 3.5 and O.scan("cumprod", torch.empty(0, 3), 0).shape == (0, 3)


def test_logcumsumexp_against_mpmath_and_invariances():
    mpmath.mp.dps = 40
    rng = random.Random(73)
    r = [f32(rng.uniform(-30, 30)) for _ in range(80)]
    got = O.scan("logcumsumexp", torch.tensor(r, dtype=F32)).tolist()
    s = mpmath.mpf(0)
    for v, g in zip(r, got):
        s += mpmath.exp(mpmath.mpf(v))
        exact = mpmath.log(s)
        assert abs(mpmath.mpf(g) - exact) <= abs(exact) * mpmath.mpf(2) ** -23 * mpmath.mpf("0.51") + mpmath.mpf(2) ** -140, (v, g)
    # adding a constant that keeps every element exact shifts the result by it: no overflow at +-1000
    x = torch.tensor([f32(rng.uniform(-4, 4)) for _ in range(50)], dtype=F32)
    base = O.scan("logcumsumexp", x).double()
    for c in (1024.0, -1024.0):
        assert torch.allclose(O.scan("logcumsumexp", (x.double() + c).float()).double(), base + c, rtol=0, atol=2e-4)
    # monotone non-decreasing, at least the running maximum, at most that plus log(count)
    run_max = torch.cummax(x, 0).values.double()
    assert (base[1:] >= base[:-1]).all() and (base >= run_max - 1e-6).all()
    assert (base <= run_max + torch.log(torch.arange(1, 51, dtype=torch.float64)) + 1e-6).all()
    # equal elements: log(k) + v
    k = O.scan("logcumsumexp", torch.full((8,), 2.5)).double()
    assert torch.allclose(k, 2.5 + torch.log(torch.arange(1, 9, dtype=torch.float64)), rtol=0, atol=3e-7)


def test_logcumsumexp_special_values_dtypes_and_aten():
    t = lambda *v: torch.tensor(v, dtype=F32)
    assert O.scan("logcumsumexp", t(-INF, -INF, 1.0, -INF)).tolist() == [-INF, -INF, 1.0, 1.0]
    assert O.scan("logcumsumexp", t(0.0, INF, 1.0, -INF, INF)).tolist() == [0.0, INF, INF, INF, INF]
    g = O.scan("logcumsumexp", t(1.0, NAN, 2.0, INF)).tolist()
    assert g[0] == 1.0 and all(math.isnan(v) for v in g[1:])
    for bad in (torch.tensor([1, 2]), torch.tensor([True])):
        with pytest.raises(O.OracleError) as e:
            O.scan("logcumsumexp", bad)
        assert e.value.kind == "dtype"
    with pytest.raises(O.OracleError) as e:
        O.scan("logcumsumexp", torch.ones(3), 1)
    assert e.value.kind == "dim"
    with pytest.raises(O.OracleError):
        O.scan("cummax", torch.ones(3))
    gen = torch.Generator().manual_seed(74)
    x = torch.randn(6, 7, 5, generator=gen) * 3
    for dim in (0, 1, 2, -2):
        assert torch.allclose(O.scan("logcumsumexp", x, dim), torch.logcumsumexp(x, dim), rtol=2e-6, atol=2e-6)
        v = x.transpose(0, 1)[:, ::2]
        assert torch.allclose(O.scan("logcumsumexp", v, dim), torch.logcumsumexp(v, dim), rtol=2e-6, atol=2e-6)
    for dt in (BF16, F16):
        h = x.to(dt)
        want = torch.logcumsumexp(h.double(), 1)
        assert torch.equal(O.scan("logcumsumexp", h, 1), want.to(dt)) and torch.equal(O.scan("logcumsumexp", h, 1, out_dtype=F32), want.float())
    assert O.scan("logcumsumexp", torch.tensor(-2.0)).item() == -2.0 and O.scan("logcumsumexp", torch.empty(3, 0), 1).shape == (3, 0)
    # cumsum through the same entry is the cumsum
    assert torch.equal(O.scan("cumsum", x, 1), O.cumsum(x, 1))
