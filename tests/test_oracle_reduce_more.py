"""Pins for the oracle's further reductions: nansum, nanmean, count_nonzero and the vector p-norm.

More of the paper's "Reduction" category (Table 1, 63 operators).  Expected values: exact rational sums and counts in
Python, mpmath roots, closed forms, and the ATen CPU operators (Section 3.2) - nothing comes from the oracle or the
HIP library.
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


def round_f32(fr):
    return torch.tensor(float(fr), dtype=torch.float64).float().item()


def test_nansum_nanmean_exact_and_against_aten():
    rng = random.Random(61)
    rows = [[f32(rng.uniform(-5, 5)) if rng.random() > 0.3 else NAN for _ in range(37)] for _ in range(11)]
    rows[3] = [NAN] * 37                                                  # nothing to add: sum 0, mean NaN
    x = torch.tensor(rows, dtype=F32)
    s, m = O.reduce("nansum", x, [1]).tolist(), O.reduce("nanmean", x, [1]).tolist()
    for r, gs, gm in zip(rows, s, m):
        vals = [Fraction(v) for v in r if not math.isnan(v)]
        assert gs == pytest.approx(float(sum(vals)), rel=2e-7, abs=1e-7)
        if vals:
            assert gm == pytest.approx(float(sum(vals) / len(vals)), rel=2e-7, abs=1e-7)
        else:
            assert gs == 0.0 and math.isnan(gm)
    for dims, keep in (([0], False), ([0, 1], False), (None, False), ([1], True), ([-2], True)):
        for op, fn in (("nansum", torch.nansum), ("nanmean", torch.nanmean)):
            want = fn(x, dim=dims, keepdim=keep) if dims is not None else fn(x)
            got = O.reduce(op, x, dims, keep)
            assert got.shape == want.shape and torch.allclose(got, want, rtol=1e-6, atol=1e-6, equal_nan=True), (op, dims, keep)
    # without NaNs they are sum and mean
    y = torch.tensor([[f32(rng.uniform(-5, 5)) for _ in range(20)] for _ in range(6)], dtype=F32)
    assert torch.equal(O.reduce("nansum", y, [0]), O.reduce("sum", y, [0])) and torch.equal(O.reduce("nanmean", y, [1]), O.reduce("mean", y, [1]))
    # infinities are kept; integers: the plain sum, nanmean refuses them; half input, fp32 out
    assert O.reduce("nansum", torch.tensor([INF, NAN, 1.0])).item() == INF and math.isnan(O.reduce("nanmean", torch.tensor([INF, NAN, -INF])).item())
    r = O.reduce("nansum", torch.tensor([[1, -2], [3, 4]], dtype=I32), [0])
    assert r.dtype == I64 and r.tolist() == [4, 2]
    assert O.reduce("nansum", torch.tensor([True, True, False])).item() == 2
    for bad in (torch.tensor([1, 2]), torch.tensor([True])):
        with pytest.raises(O.OracleError) as e:
            O.reduce("nanmean", bad)
        assert e.value.kind == "dtype"
    h = torch.tensor([1.5, NAN, 2.25], dtype=BF16)
    assert O.reduce("nansum", h).item() == 3.75 and O.reduce("nanmean", h, out_dtype=F32).item() == 1.875
    assert O.reduce("nansum", torch.empty(0, 3), [0]).tolist() == [0.0] * 3 and math.isnan(O.reduce("nanmean", torch.empty(0)).item())


def test_count_nonzero():
    rng = random.Random(62)
    vals = [[rng.choice([0.0, -0.0, 1.5, NAN, INF, -2.0]) for _ in range(23)] for _ in range(9)]
    x = torch.tensor(vals, dtype=F32)
    want_rows = [sum(1 for v in r if v != 0) for r in vals]              # NaN != 0 is true in Python as in IEEE
    assert O.reduce("count_nonzero", x, [1]).tolist() == want_rows
    assert O.reduce("count_nonzero", x).item() == sum(want_rows)
    assert O.reduce("count_nonzero", x, [1], True).shape == (9, 1)
    for dt in (B, I32, I64, F16, BF16):
        t = torch.tensor([[0, 3, 0, -1], [0, 0, 0, 0], [1, 1, 1, 1]]).to(dt)
        got = O.reduce("count_nonzero", t, [1])
        assert got.dtype == I64 and got.tolist() == [2 if dt != B else 2, 0, 4]
        assert torch.equal(got, torch.count_nonzero(t, dim=1))
        assert torch.equal(O.reduce("count_nonzero", t, [0, 1]), torch.count_nonzero(t, dim=(0, 1)))
    assert O.reduce("count_nonzero", torch.empty(0, 3), [0]).tolist() == [0, 0, 0]
    assert torch.equal(O.reduce("count_nonzero", x.t()[::2], [0]), torch.count_nonzero(x.t()[::2], dim=0))


def test_norm_closed_forms_special_orders_and_mpmath():
    mpmath.mp.dps = 40
    y = torch.tensor([3.0, -4.0, 0.0])
    assert O.reduce("norm", y, correction=2.0).item() == 5.0 and O.reduce("norm", y, correction=1.0).item() == 7.0
    assert O.reduce("norm", y, correction=INF).item() == 4.0 and O.reduce("norm", y, correction=-INF).item() == 0.0
    assert O.reduce("norm", y, correction=0.0).item() == 2.0
    assert O.reduce("norm", y, correction=-1.0).item() == 0.0          # 1 / (1/3 + 1/4 + 1/0)
    rng = random.Random(63)
    v = [f32(rng.uniform(-4, 4)) for _ in range(200)]
    x = torch.tensor(v)
    for p in (0.5, 1.0, 2.0, 3.0, -1.0, -2.0, 1.5):
        exact = mpmath.power(sum(mpmath.power(abs(mpmath.mpf(a)), p) for a in v), mpmath.mpf(1) / p)
        got = O.reduce("norm", x, correction=p).item()
        assert abs(mpmath.mpf(got) - exact) <= abs(exact) * mpmath.mpf(2) ** -23 * mpmath.mpf("0.51"), (p, got)
    assert O.reduce("norm", x, correction=INF).item() == max(abs(a) for a in v)
    assert O.reduce("norm", x, correction=-INF).item() == min(abs(a) for a in v)
    # nothing overflows or underflows that the result does not: sqrt(2) * 1e20, sqrt(2) * 1e-30
    big = O.reduce("norm", torch.tensor([1e20, 1e20]), correction=2.0).item()
    assert big == round_f32(Fraction(f32(1e20)) * Fraction(math.sqrt(2)))
    small = O.reduce("norm", torch.tensor([1e-30, 1e-30]), correction=2.0).item()
    assert small == pytest.approx(math.sqrt(2) * f32(1e-30), rel=2e-7)
    # NaN: sticky for every order but 0, where it counts as non-zero
    n = torch.tensor([3.0, NAN, 0.0])
    for p in (1.0, 2.0, 3.0, INF, -INF):
        assert math.isnan(O.reduce("norm", n, correction=p).item()), p
    assert O.reduce("norm", n, correction=0.0).item() == 2.0
    assert O.reduce("norm", torch.tensor([INF, 1.0]), correction=2.0).item() == INF
    # empty extents: 0 for p >= 0 (finite), an error for infinite and negative p
    for p in (0.0, 1.0, 2.0, 3.0):
        assert O.reduce("norm", torch.empty(0), correction=p).item() == 0.0
        assert O.reduce("norm", torch.empty(0, 3), [0], correction=p).tolist() == [0.0] * 3
    for p in (INF, -INF, -1.0):
        with pytest.raises(O.OracleError) as e:
            O.reduce("norm", torch.empty(0), correction=p)
        assert e.value.kind == "empty_reduction"
    with pytest.raises(O.OracleError) as e:
        O.reduce("norm", torch.tensor([1, 2]), correction=2.0)
    assert e.value.kind == "dtype"
    with pytest.raises(O.OracleError) as e:
        O.reduce("norm", y, correction=NAN)
    assert e.value.kind == "scalar"


@pytest.mark.parametrize("dt", [F32, BF16, F16])
def test_norm_against_aten_over_dims_and_views(dt):
    g = torch.Generator().manual_seed(64)
    x = (torch.randn(6, 9, 14, generator=g) * 2).to(dt)
    tol = 2e-6 if dt == F32 else 1e-2
    for p in (0.0, 1.0, 2.0, INF, -INF, 3.0, 0.5, -1.0):
        for dims, keep in (([2], False), ([0], True), ([0, 2], False), (None, False), ([1, 2], True)):
            want = torch.linalg.vector_norm(x, p, dim=dims, keepdim=keep)
            got = O.reduce("norm", x, dims, keep, correction=p)
            assert got.dtype == want.dtype and got.shape == want.shape
            assert torch.allclose(got.double(), want.double(), rtol=tol, atol=tol), (p, dims, keep)
        xv = x.transpose(0, 2)[::2]
        assert torch.allclose(O.reduce("norm", xv, [1], correction=p).double(), torch.linalg.vector_norm(xv, p, dim=1).double(), rtol=tol, atol=tol)
    # a half input with an fp32 result: the dtype= variant
    if dt != F32:
        want = torch.linalg.vector_norm(x, 2.0, dim=1, dtype=F32)
        assert torch.allclose(O.reduce("norm", x, [1], correction=2.0, out_dtype=F32), want, rtol=1e-6)
