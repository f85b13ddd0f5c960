"""Pins for the oracle's softmax / log_softmax and cumsum.

Closed forms, invariants and 60-digit arithmetic for the operator definitions
the paper delegates to (Section 3.2 criterion; softmax belongs to Table 1's
"Deep Learning" category, cumsum to "Reduction").  No expected value comes
from the oracle or from the HIP library.
"""
import math

import mpmath
import pytest
import torch

from oracle import oracle as O
from paper_2512_10977_amd import inputs as I

F32, BF16, F16, I32, I64, B = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool


# --------------------------------------------------------------------------- softmax
def test_softmax_rows_sum_to_one_and_are_shift_invariant():
    x = I.softmax_logits((40, 257), F32, seed=3)
    y = O.softmax(x)
    assert ((y.double().sum(1) - 1).abs() <= 1e-6).all()
    assert (y >= 0).all()
    y2 = O.softmax(x + 8.0)                                   # the shift itself rounds, hence the slack
    assert ((y2.double() - y.double()).abs() <= 4e-6 * y.double() + 1e-12).all()


def test_softmax_uniform_and_two_element_closed_forms():
    for n in (1, 3, 64, 1000):
        y = O.softmax(torch.full((2, n), 1.75))
        assert ((y.double() - 1.0 / n).abs() <= 1e-7 / n).all()
        ly = O.softmax(torch.full((2, n), 1.75), log=True)
        assert ((ly.double() + math.log(n)).abs() <= 1e-6).all()
    # two entries: softmax = logistic(a - b)
    a, b = 0.3, -1.9
    y = O.softmax(torch.tensor([[a, b]]))
    fa, fb = float(torch.tensor(a)), float(torch.tensor(b))
    want = 1 / (1 + math.exp(fb - fa))
    assert abs(y[0, 0].item() - want) <= 1e-7 and abs(y[0, 1].item() - (1 - want)) <= 1e-7


def test_softmax_against_60_digit_arithmetic():
    mpmath.mp.dps = 60
    x = I.normal((3, 17), 4.0, seed=60)
    y, ly = O.softmax(x), O.softmax(x, log=True)
    for r in range(3):
        v = [mpmath.mpf(t) for t in x[r].tolist()]
        z = sum(mpmath.exp(t) for t in v)
        for c in range(17):
            assert abs(y[r, c].item() - float(mpmath.exp(v[c]) / z)) <= 1e-7 * float(mpmath.exp(v[c]) / z)
            assert abs(ly[r, c].item() - float(v[c] - mpmath.log(z))) <= 1e-6


def test_exp_of_log_softmax_is_softmax():
    x = I.softmax_logits((16, 100), F32, seed=61)
    y, ly = O.softmax(x).double(), O.softmax(x, log=True).double()
    assert ((ly.exp() - y).abs() <= 1e-6 * y + 1e-30).all()


def test_softmax_special_values():
    inf, nan = math.inf, math.nan
    x = torch.tensor([[0.0, -inf, 1.0], [-inf, -inf, -inf], [0.0, inf, 1.0], [0.0, nan, 1.0]])
    y, ly = O.softmax(x), O.softmax(x, log=True)
    assert y[0, 1].item() == 0.0 and ly[0, 1].item() == -inf
    assert abs(y[0, 0].item() + y[0, 2].item() - 1) < 1e-7
    for r in (1, 2, 3):
        assert y[r].isnan().all() and ly[r].isnan().all()
    assert O.softmax(torch.tensor(2.5), 0).item() == 1.0 and O.softmax(torch.tensor(2.5), 0, log=True).item() == 0.0
    assert O.softmax(torch.zeros((3, 0))).shape == (3, 0)
    with pytest.raises(O.OracleError):
        O.softmax(torch.ones(2, 2, dtype=I32))
    with pytest.raises(O.OracleError):
        O.softmax(torch.ones(2, 2), 2)


def test_softmax_other_dims_and_views():
    x = I.normal((5, 6, 7), 4.0, seed=62)
    for d in (0, 1, 2, -1, -3):
        dd = d % 3
        want = O.softmax(x.movedim(dd, -1).contiguous()).movedim(-1, dd)
        assert torch.equal(O.softmax(x, d), want)
    xt = I.make_view((5, 6, 7), F32, "transposed", seed=63)
    assert torch.equal(O.softmax(xt), O.softmax(xt.contiguous()))


def test_half_softmax_rounds_once_and_supports_fp32_out():
    x = I.normal((8, 50), 4.0, seed=64, dtype=BF16)
    y32 = O.softmax(x, out_dtype=F32)
    assert y32.dtype == F32 and torch.equal(y32, O.softmax(x.float()))
    assert torch.equal(O.softmax(x), y32.to(BF16)) or ((O.softmax(x).float() - y32).abs() <= 0.004 * y32).all()


# --------------------------------------------------------------------------- cumsum
def test_cumsum_closed_forms():
    n = 500
    assert O.cumsum(torch.ones(n, dtype=I64)).tolist() == list(range(1, n + 1))
    assert O.cumsum(torch.arange(n)).tolist() == [k * (k + 1) // 2 for k in range(n)]
    assert O.cumsum(torch.ones(n)).tolist() == [float(k) for k in range(1, n + 1)]
    r = O.cumsum(torch.tensor([True, False, True, True]))
    assert r.dtype == I64 and r.tolist() == [1, 1, 2, 3]
    assert O.cumsum(torch.tensor([5, -7], dtype=I32)).dtype == I64
    assert O.cumsum(torch.tensor([2 ** 62, 2 ** 62, 2 ** 62])).tolist() == [2 ** 62, -2 ** 63, -2 ** 62]


def test_cumsum_last_equals_sum_and_differences_recover_input():
    xi = I.cumsum_input((7, 300), I64, seed=3)
    c = O.cumsum(xi)
    assert torch.equal(c[:, -1], O.reduce("sum", xi, 1))
    assert torch.equal(c[:, 1:] - c[:, :-1], xi[:, 1:]) and torch.equal(c[:, 0], xi[:, 0])
    xf = I.cumsum_input((7, 300), F32, seed=3)
    cf = O.cumsum(xf)
    assert torch.equal(cf[:, -1], O.reduce("sum", xf, 1))            # both are the rounded binary64 sum
    for r in range(7):
        row = xf[r].tolist()
        for k in (0, 1, 17, 299):
            want = math.fsum(row[:k + 1])
            assert abs(cf[r, k].item() - want) <= 2.0 ** -23 * abs(want) + 1e-12


def test_cumsum_special_values_dims_and_views():
    inf = math.inf
    r = O.cumsum(torch.tensor([1.0, inf, 2.0, -inf, 5.0])).tolist()
    assert r[:3] == [1.0, inf, inf] and math.isnan(r[3]) and math.isnan(r[4])
    assert O.cumsum(torch.tensor(4.0), 0).item() == 4.0
    assert O.cumsum(torch.zeros((0, 4)), 1).shape == (0, 4)
    x = I.integers((4, 5, 6), -100, 100, seed=65)
    for d in (0, 1, 2, -2):
        dd = d % 3
        want = O.cumsum(x.movedim(dd, -1).contiguous()).movedim(-1, dd)
        assert torch.equal(O.cumsum(x, d), want)
        assert torch.equal(O.cumsum(x, d), torch.cumsum(x, d))        # library cross-check (exact for ints)
    xs = I.make_view((4, 5, 6), I64, "step2_inner", seed=66)
    assert torch.equal(O.cumsum(xs), O.cumsum(xs.contiguous()))
    with pytest.raises(O.OracleError):
        O.cumsum(x, 3)


def test_half_cumsum_accumulates_wide():
    x = torch.full((4096,), 1.0078125, dtype=BF16)
    c = O.cumsum(x)
    assert c[-1].item() == float(torch.tensor(4128.0).to(BF16))
    assert O.cumsum(x, out_dtype=F32)[-1].item() == 4128.0
