"""Pins for the oracle's floor_divide and trunc_divide (ATen's div with rounding_mode "floor" / "trunc").

Two more of the paper's largest category (Table 1, "Elementwise").  Expected values: Python's exact integer and
rational arithmetic (// on ints, floor / trunc of a Fraction), IEEE special cases written out, and the ATen CPU
operators - nothing comes from the oracle or the HIP library.
"""
import math
import random
import struct
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import oracle as O

F32, BF16, F16, I32, I64, B = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool
NAN, INF = float("nan"), float("inf")


def wrap(v, bits):
    v &= (1 << bits) - 1
    return v - (1 << bits) if v >> (bits - 1) else v


def py_trunc_div(a, b):
    q = abs(a) // abs(b)
    return q if (a < 0) == (b < 0) else -q


@pytest.mark.parametrize("dt,bits", [(I32, 32), (I64, 64)])
def test_integers_match_exact_integer_division(dt, bits):
    rng = random.Random(5)
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    small = list(range(-9, 10))
    a = small * 19 + [lo, lo, hi, hi, lo + 1] + [rng.randint(lo, hi) for _ in range(400)]
    b = [d for d in small for _ in range(19)] + [-1, 1, -1, 2, -1] + [rng.choice([rng.randint(lo, hi), rng.randint(-50, 50)]) for _ in range(400)]
    pairs = [(x, y) for x, y in zip(a, b) if y != 0]
    ta, tb = torch.tensor([p[0] for p in pairs], dtype=dt), torch.tensor([p[1] for p in pairs], dtype=dt)
    fl, tr = O.binary("floor_divide", ta, tb), O.binary("trunc_divide", ta, tb)
    assert fl.dtype == dt and tr.dtype == dt
    for i, (x, y) in enumerate(pairs):
        assert fl[i].item() == wrap(x // y, bits), ("floor", x, y)
        assert tr[i].item() == wrap(py_trunc_div(x, y), bits), ("trunc", x, y)


def test_integer_zero_divisor_and_bool_are_errors():
    a, z = torch.tensor([1, 2, 3]), torch.tensor([1, 0, 1])
    for op in ("floor_divide", "trunc_divide"):
        with pytest.raises(O.OracleError):
            O.binary(op, a, z)
        with pytest.raises(O.OracleError):
            O.binary(op, torch.tensor([True]), torch.tensor([True]))
        # a float operand makes the division an IEEE one
        r = O.binary(op, a, z.to(F32))
        assert r.dtype == F32 and math.isinf(r[1].item())


def test_fp32_against_exact_rational_quotients():
    rng = np.random.default_rng(6)
    a = np.concatenate([rng.uniform(-1000, 1000, 3000), rng.integers(-60, 60, 1500)]).astype(np.float32)
    b = np.concatenate([rng.uniform(-30, 30, 3000), rng.integers(-12, 12, 1500)]).astype(np.float32)
    keep = b != 0
    a, b = a[keep], b[keep]
    fl = O.binary("floor_divide", torch.from_numpy(a), torch.from_numpy(b))
    tr = O.binary("trunc_divide", torch.from_numpy(a), torch.from_numpy(b))
    for i in range(len(a)):
        q = Fraction(float(a[i])) / Fraction(float(b[i]))
        assert fl[i].item() == math.floor(q), ("floor", a[i], b[i])      # |q| < 2^24: the floor is representable
        # trunc is defined on the rounded binary32 quotient (it differs from the exact one only when the division
        # rounds up to an integer)
        assert tr[i].item() == math.trunc(float(np.float32(a[i]) / np.float32(b[i]))), ("trunc", a[i], b[i])


def test_floor_does_not_round_a_quotient_up_to_the_next_integer():
    # 3 / nextbelow(1): the binary32 quotient rounds to 3.0000002 > 3 (fine), but 2.9999998 / 1 style cases where the
    # division would round *up* to an integer must still floor to the integer below
    below_three = struct.unpack("<f", struct.pack("<I", struct.unpack("<I", struct.pack("<f", 3.0))[0] - 1))[0]
    a = torch.tensor([below_three, 0.3 * 3, 1.0, -1.0, 6.0], dtype=F32)
    b = torch.tensor([1.0, 0.1, 0.1, 0.1, 0.1], dtype=F32)
    got = O.binary("floor_divide", a, b)
    want = [math.floor(Fraction(float(x)) / Fraction(float(y))) for x, y in zip(a.tolist(), b.tolist())]
    assert got.tolist() == [float(w) for w in want]


def test_special_values():
    a = torch.tensor([0.0, -0.0, 0.0, 1.0, -1.0, 0.0, 5.0, -5.0, INF, NAN, 1.0, 1.0, -1.0], dtype=F32)
    b = torch.tensor([3.0, 3.0, -3.0, 0.0, 0.0, 0.0, INF, INF, 2.0, 1.0, NAN, -3.0, 3.0], dtype=F32)
    fl = O.binary("floor_divide", a, b).tolist()
    tr = O.binary("trunc_divide", a, b).tolist()
    # zero results carry the sign of the quotient; x / 0 is the IEEE quotient
    for got, exp in ((fl[0], 0.0), (fl[1], -0.0), (fl[2], -0.0), (tr[0], 0.0), (tr[1], -0.0), (tr[2], -0.0)):
        assert got == 0.0 and math.copysign(1.0, got) == math.copysign(1.0, exp)
    assert fl[3] == INF and fl[4] == -INF and math.isnan(fl[5])
    assert tr[3] == INF and tr[4] == -INF and math.isnan(tr[5])
    # finite / infinity: fmod(a, inf) = a, so floor gives 0 for the same signs and -1 for different ones
    assert fl[6] == 0.0 and fl[7] == -1.0 and tr[6] == 0.0 and tr[7] == 0.0 and math.copysign(1.0, tr[7]) == -1.0
    assert math.isnan(fl[8]) and tr[8] == INF                  # fmod(inf, 2) is NaN; inf / 2 truncates to inf
    assert all(math.isnan(v) for v in (fl[9], fl[10], tr[9], tr[10]))
    assert fl[11] == -1.0 and fl[12] == -1.0 and tr[11] == 0.0 and tr[12] == 0.0


@pytest.mark.parametrize("dt", [F32, BF16, F16, I32, I64])
def test_against_aten_cpu_with_broadcasting_and_promotion(dt):
    g = torch.Generator().manual_seed(7)
    if dt.is_floating_point:
        a = (torch.randn((6, 1, 33), generator=g) * 40).to(dt)
        b = (torch.randn((5, 33), generator=g) * 6).to(dt)
        b[b == 0] = 1
    else:
        a = torch.randint(-500, 500, (6, 1, 33), generator=g).to(dt)
        b = torch.randint(1, 40, (5, 33), generator=g).to(dt) * (torch.randint(0, 2, (5, 33), generator=g) * 2 - 1).to(dt)
    for op, mode in (("floor_divide", "floor"), ("trunc_divide", "trunc")):
        want = torch.div(a, b, rounding_mode=mode)
        got = O.binary(op, a, b)
        assert got.dtype == want.dtype and got.shape == want.shape
        if dt in (BF16, F16) and mode == "floor":
            # ATen's kernel rounds every step of the floor algorithm to the half format, the oracle evaluates it in
            # binary32 and rounds once (2.15625 // -0.02685546875 is -81, the stepwise bf16 evaluation says -82):
            # quotients can differ by one, or in the last place
            assert ((got.float() - want.float()).abs() <= want.float().abs() * 2 ** -7 + 1).all()
            assert ((got.float() - want.float()).abs() == 0).float().mean() > 0.9
        else:
            assert torch.equal(got, want), op
    # mixed operands: int tensor with a float tensor gives the float dtype, int32 with int64 gives int64
    ai, bf = torch.tensor([7, -7, 9], dtype=I32), torch.tensor([2.0, 2.0, -4.0], dtype=F32)
    assert torch.equal(O.binary("floor_divide", ai, bf), torch.div(ai, bf, rounding_mode="floor"))
    assert O.binary("trunc_divide", ai, torch.tensor([2, 2, -4])).dtype == I64
