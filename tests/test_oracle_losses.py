"""Pins for the oracle's regression losses: mse_loss, l1_loss, smooth_l1_loss, huber_loss with none / mean / sum.

The paper's weakest category is "Deep Learning" (Table 1); its binary_cross_entropy listing (Appendix B.1) is one member
of the family "elementwise term, then an optional sum or mean", and these four are the same shape.  Expected values:
exact rational arithmetic, identities between the four, closed forms, and the ATen CPU operators (Section 3.2) -
nothing comes from the oracle or the HIP library.
"""
import math
import random
import struct
from fractions import Fraction

import pytest
import torch
import torch.nn.functional as NF

from oracle import oracle as O

F32, BF16, F16, I64 = torch.float32, torch.bfloat16, torch.float16, torch.int64
NAN, INF = float("nan"), float("inf")


def f32(x):
    return struct.unpack("<f", struct.pack("<f", x))[0]


def exact_term(kind, x, t, p):
    d = Fraction(x) - Fraction(t)
    ad = abs(d)
    if kind == "mse":
        return d * d
    if kind == "l1":
        return ad
    if kind == "smooth_l1":
        return d * d / (2 * Fraction(p)) if ad < Fraction(p) else ad - Fraction(p) / 2
    return d * d / 2 if ad <= Fraction(p) else Fraction(p) * (ad - Fraction(p) / 2)


def round_f32(fr):
    return torch.tensor(float(fr), dtype=torch.float64).float().item()


@pytest.mark.parametrize("kind,param", [("mse", 1.0), ("l1", 1.0), ("smooth_l1", 0.75), ("smooth_l1", 0.0), ("huber", 1.5), ("huber", 0.25)])
def test_terms_and_sums_against_exact_rationals(kind, param):
    rng = random.Random(51)
    x = [f32(rng.uniform(-3, 3)) for _ in range(200)] + [f32(1.0), f32(2.5), f32(-1.0)]
    t = [f32(rng.uniform(-3, 3)) for _ in range(200)] + [f32(1.0), f32(1.0), f32(0.5)]       # d = 0, |d| = 1.5 (huber's edge)
    tx, tt = torch.tensor(x), torch.tensor(t)
    terms = [exact_term(kind, a, b, param) for a, b in zip(x, t)]
    got = O.loss(kind, tx, tt, "none", param).tolist()
    # float(Fraction) is correctly rounded to binary64; the term is then rounded to fp32: at most a double rounding apart
    for g, e in zip(got, terms):
        assert abs(Fraction(g) - e) <= abs(e) * Fraction(1, 2 ** 23) * Fraction(501, 1000), (kind, g, float(e))
    total = sum(terms)
    assert O.loss(kind, tx, tt, "sum", param).item() == pytest.approx(float(total), rel=3e-7)
    assert O.loss(kind, tx, tt, "mean", param).item() == pytest.approx(float(total / len(x)), rel=3e-7)
    # the sum keeps binary64 until the end: fp32 terms of very different size do not swamp each other
    big = torch.tensor([1e4] + [1e-3] * 4096, dtype=F32)
    want = sum(exact_term(kind, v, 0.0, param) for v in big.tolist())
    assert O.loss(kind, big, torch.zeros_like(big), "sum", param).item() == round_f32(want)


def test_identities_between_the_losses():
    g = torch.Generator().manual_seed(52)
    x, t = torch.randn(37, 11, generator=g) * 2, torch.randn(37, 11, generator=g) * 2
    # beta = 0: smooth_l1 is l1
    assert torch.equal(O.loss("smooth_l1", x, t, "none", 0.0), O.loss("l1", x, t, "none"))
    # huber(delta) = delta * smooth_l1(beta = delta); with delta = 2^k the product is exact
    for delta in (0.5, 2.0):
        assert torch.equal(O.loss("huber", x, t, "none", delta), O.loss("smooth_l1", x, t, "none", delta) * delta)
    # a delta beyond every |d|: huber = mse / 2 exactly (a power of two)
    assert torch.equal(O.loss("huber", x, t, "none", 1e6), O.loss("mse", x, t, "none") * 0.5)
    # a beta below every |d|: smooth_l1 = l1 - beta / 2
    far = x + 5.0
    want = (far.double() - x.double()).abs() - 0.25
    assert torch.equal(O.loss("smooth_l1", far, x, "none", 0.5), want.float())
    # closed forms: a constant offset c gives c^2, |c|
    c = torch.full((5, 7), 1.5)
    z = torch.zeros(5, 7)
    assert O.loss("mse", c, z, "mean").item() == 2.25 and O.loss("l1", z, c, "sum").item() == 52.5
    assert O.loss("mse", c, z, "sum").item() == 2.25 * 35
    # symmetric in (x, t)
    for kind in ("mse", "l1", "smooth_l1", "huber"):
        assert torch.equal(O.loss(kind, x, t, "none", 0.7), O.loss(kind, t, x, "none", 0.7))


@pytest.mark.parametrize("dt", [F32, BF16, F16])
def test_against_aten_cpu_with_broadcasting_and_views(dt):
    g = torch.Generator().manual_seed(53)
    aten = {"mse": lambda x, t, r, p: NF.mse_loss(x, t, reduction=r), "l1": lambda x, t, r, p: NF.l1_loss(x, t, reduction=r),
            "smooth_l1": lambda x, t, r, p: NF.smooth_l1_loss(x, t, reduction=r, beta=p),
            "huber": lambda x, t, r, p: NF.huber_loss(x, t, reduction=r, delta=p)}
    tol = 2e-6 if dt == F32 else 2e-2
    shapes = [((19, 23), (19, 23)), ((19, 23), (23,)), ((4, 1, 6), (5, 1)), ((), ()), ((7,), ())]
    for kind, fn in aten.items():
        for (sx, st), red, p in [(s, r, p) for s in shapes for r in ("none", "mean", "sum") for p in (0.5, 2.0)]:
            x, t = (torch.randn(sx, generator=g) * 2).to(dt), (torch.randn(st, generator=g) * 2).to(dt)
            import warnings
            with warnings.catch_warnings():
                warnings.simplefilter("ignore")
                want = fn(x, t, red, p)
            got = O.loss(kind, x, t, red, p)
            assert got.dtype == want.dtype and got.shape == want.shape, (kind, sx, st, red)
            assert torch.allclose(got.double(), want.double(), rtol=tol, atol=tol), (kind, sx, st, red, p)
        xt = (torch.randn(12, 9, generator=g)).to(dt).t()
        tt = (torch.randn(9, 24, generator=g)).to(dt)[:, ::2]
        assert torch.allclose(O.loss(kind, xt, tt, "mean", 1.0).double(), fn(xt, tt, "mean", 1.0).double(), rtol=tol, atol=tol)


def test_special_values_empty_and_errors():
    x, t = torch.tensor([NAN, INF, 1.0, INF, -INF]), torch.tensor([0.0, 0.0, NAN, INF, INF])
    for kind in ("mse", "l1", "smooth_l1", "huber"):
        got = O.loss(kind, x, t, "none", 1.0).tolist()
        assert math.isnan(got[0]) and got[1] == INF and math.isnan(got[2]) and math.isnan(got[3]) and got[4] == INF, (kind, got)
        assert math.isnan(O.loss(kind, x, t, "sum", 1.0).item())
        e = torch.empty(0, 3)
        assert O.loss(kind, e, e, "none").shape == (0, 3) and O.loss(kind, e, e, "sum").item() == 0.0
        assert math.isnan(O.loss(kind, e, e, "mean").item())
        for args, what in (((torch.ones(3, dtype=I64), torch.ones(3, dtype=I64)), "dtype"), ((torch.ones(3), torch.ones(3, dtype=BF16)), "dtype"),
                           ((torch.ones(3), torch.ones(4)), "shape")):
            with pytest.raises(O.OracleError) as err:
                O.loss(kind, *args)
            assert err.value.kind == what
        with pytest.raises(O.OracleError) as err:
            O.loss(kind, torch.ones(3), torch.ones(3), "median")
        assert err.value.kind == "scalar"
        with pytest.raises(O.OracleError):
            O.loss(kind, torch.ones(3), torch.ones(3), "mean", out=torch.empty(3))
    for kind, bad in (("smooth_l1", -0.5), ("huber", 0.0), ("huber", -1.0), ("smooth_l1", NAN)):
        with pytest.raises(O.OracleError) as err:
            O.loss(kind, torch.ones(3), torch.ones(3), "mean", bad)
        assert err.value.kind == "scalar"
    with pytest.raises(O.OracleError):
        O.loss("hinge", torch.ones(3), torch.ones(3))
    # ATen refuses the same parameters
    with pytest.raises(RuntimeError):
        NF.smooth_l1_loss(torch.ones(3), torch.ones(3), beta=-0.5)
    with pytest.raises(RuntimeError):
        NF.huber_loss(torch.ones(3), torch.ones(3), delta=0.0)
    # half types: the term rounded once from the exact value
    xb, tb = torch.tensor([1.5, -0.25], dtype=BF16), torch.tensor([0.5, 0.75], dtype=BF16)
    assert O.loss("mse", xb, tb, "none").tolist() == [1.0, 1.0] and O.loss("mse", xb, tb, "mean").item() == 1.0
