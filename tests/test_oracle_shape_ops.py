"""Pins for the oracle's data-moving shape operators: copy with conversion, flip, roll, tril, triu.

The paper's "Shape Manipulation" category (Table 1, 75 operators; its best-covered one).  Expected values: Python list
manipulation written out by hand, exact conversions through struct, and the ATen CPU operators (Section 3.2) -
nothing comes from the oracle or the HIP library.
"""
import itertools
import math
import random
import struct

import pytest
import torch

from oracle import oracle as O

F32, BF16, F16, I32, I64, B = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool
ALL = (B, I32, I64, F16, BF16, F32)
NAN, INF = float("nan"), float("inf")


def test_copy_conversions_exact():
    # float -> half: one rounding, ties to even; the ATen conversion is the same rule
    v = torch.tensor([1.0 + 2.0 ** -9, 1.0 + 3 * 2.0 ** -9, 65520.0, -1e-8, 3.3e38, NAN, -INF, 1.0 / 3], dtype=F32)
    for dt in (BF16, F16):
        got = O.copy(v, dtype=dt)
        assert got.dtype == dt and torch.equal(got.float().nan_to_num(7.0), v.to(dt).float().nan_to_num(7.0))
    assert O.copy(torch.tensor([1.0 + 2.0 ** -8]), dtype=BF16).item() == 1.0                      # a tie goes to the even neighbour
    assert O.copy(torch.tensor([1.0 + 3 * 2.0 ** -8]), dtype=BF16).item() == 1.0 + 2.0 ** -6
    # float -> integer truncates toward zero; -> bool is "not zero" (NaN and -0.5 are true)
    f = torch.tensor([2.9, -2.9, 0.0, -0.0, 1e9, -0.5, 123456.78], dtype=F32)
    assert O.copy(f, dtype=I32).tolist() == [2, -2, 0, 0, 1000000000, 0, 123456]
    assert O.copy(f, dtype=I64).tolist() == [2, -2, 0, 0, 1000000000, 0, 123456]
    assert O.copy(torch.tensor([0.0, -0.0, NAN, -0.5, 1e-40]), dtype=B).tolist() == [False, False, True, True, True]
    # integer -> floating through binary32, nearest-even; int64 -> int32 wraps; -> bool is "not zero"
    i = torch.tensor([2 ** 24 + 1, 2 ** 24 + 3, -(2 ** 53) - 1, 2 ** 40 + 5, -7, 0])
    assert O.copy(i, dtype=F32).tolist() == [float(2 ** 24), float(2 ** 24 + 4), -float(2 ** 53), float(2 ** 40), -7.0, 0.0]
    assert O.copy(i, dtype=I32).tolist() == [2 ** 24 + 1, 2 ** 24 + 3, -1, 5, -7, 0]
    assert O.copy(i, dtype=B).tolist() == [True, True, True, True, True, False]
    assert O.copy(torch.tensor([300, 2049]), dtype=F16).tolist() == [300.0, 2048.0] and O.copy(torch.tensor([257]), dtype=BF16).item() == 256.0
    assert O.copy(torch.tensor([True, False]), dtype=BF16).tolist() == [1.0, 0.0] and O.copy(torch.tensor([True, False]), dtype=I64).tolist() == [1, 0]
    # the same dtype keeps every bit (a NaN payload, -0.0)
    bits = torch.tensor([0x7FC12345, 0xFFC00001 - 2 ** 32, -2 ** 31], dtype=I32)
    assert torch.equal(O.copy(bits.view(F32)).view(I32), bits)
    # every pair of dtypes against ATen on values every dtype holds exactly
    src = torch.tensor([[0, 1, 2], [3, 0, 100]])
    for da, db in itertools.product(ALL, ALL):
        a = src.to(da)
        got = O.copy(a, dtype=db)
        assert got.dtype == db and torch.equal(got, a.to(db)), (da, db)


def test_copy_layouts_and_broadcast():
    g = torch.Generator().manual_seed(91)
    x = torch.randn(6, 7, 5, generator=g)
    for view in (x.transpose(0, 2), x[:, ::2], x[1], x.permute(1, 2, 0)[::3]):
        assert torch.equal(O.copy(view), view.contiguous())
        out = torch.empty(view.shape[::-1]).permute(*range(view.dim() - 1, -1, -1))          # a non-contiguous destination
        O.copy(view, out=out)
        assert torch.equal(out, view)
    row = torch.randn(5, generator=g)
    assert torch.equal(O.copy(row, shape=(4, 3, 5)), row.expand(4, 3, 5).contiguous())
    assert torch.equal(O.copy(torch.tensor(2.5), shape=(2, 2), dtype=I32), torch.full((2, 2), 2, dtype=I32))
    assert O.copy(torch.empty(0, 3)).shape == (0, 3)
    with pytest.raises(O.OracleError) as e:
        O.copy(torch.ones(4, 3), out=torch.empty(3))
    assert e.value.kind == "shape"
    with pytest.raises(O.OracleError):
        O.copy(torch.ones(4), out=torch.empty(3))


def nested(t):
    return t.tolist()


def test_flip_roll_by_hand_and_against_aten():
    x = torch.arange(24).view(2, 3, 4)
    l = nested(x)
    assert nested(O.flip(x, [0])) == l[::-1]
    assert nested(O.flip(x, [2])) == [[r[::-1] for r in m] for m in l]
    assert nested(O.flip(x, [0, 1])) == [m[::-1] for m in l[::-1]]
    assert nested(O.flip(x, [-1, -3])) == [[r[::-1] for r in m] for m in l[::-1]]
    assert nested(O.roll(x, [1], [2])) == [[r[-1:] + r[:-1] for r in m] for m in l]
    assert nested(O.roll(x, [-1], [1])) == [m[1:] + m[:1] for m in l]
    assert nested(O.roll(x, [5, -7], [2, 0])) == nested(O.roll(O.roll(x, [1], [2]), [1], [0]))          # 5 mod 4, -7 mod 2
    assert nested(O.roll(x, [1, 2], [2, 2])) == nested(O.roll(x, [3], [2]))                               # a dim listed twice: shifts add
    g = torch.Generator().manual_seed(92)
    for dt in ALL:
        t = (torch.randn(5, 4, 6, generator=g) * 4).to(dt)
        for dims in ([0], [1, 2], [0, 1, 2], [-1], []):
            assert torch.equal(O.flip(t, dims), torch.flip(t, dims)), (dt, dims)
            v = t.transpose(0, 1)[:, ::2]
            assert torch.equal(O.flip(v, dims), torch.flip(v, dims))
        for shifts, dims in (([1], [0]), ([-2, 3], [1, 2]), ([7, 0, -13], [0, 1, 2]), ([2], [-1])):
            assert torch.equal(O.roll(t, shifts, dims), torch.roll(t, shifts, dims)), (dt, shifts, dims)
            v = t.transpose(0, 2)
            assert torch.equal(O.roll(v, shifts, dims), torch.roll(v, shifts, dims))
    assert O.flip(torch.tensor(3.0), [0]).item() == 3.0 and O.roll(torch.tensor(3.0), [2], [0]).item() == 3.0
    assert O.flip(torch.empty(0, 3), [0, 1]).shape == (0, 3) and O.roll(torch.empty(3, 0), [1], [1]).shape == (3, 0)
    for call in (lambda: O.flip(x, [3]), lambda: O.flip(x, [0, 0]), lambda: O.flip(x, [1, -2]), lambda: O.roll(x, [1], [-4])):
        with pytest.raises(O.OracleError) as e:
            call()
        assert e.value.kind == "dim"
    with pytest.raises(O.OracleError) as e:
        O.flip(x, [0], out=torch.empty(2, 3, 4))
    assert e.value.kind == "dtype"


def test_tril_triu_by_hand_and_against_aten():
    x = torch.arange(1, 13).view(3, 4)
    assert O.tril(x).tolist() == [[1, 0, 0, 0], [5, 6, 0, 0], [9, 10, 11, 0]]
    assert O.triu(x).tolist() == [[1, 2, 3, 4], [0, 6, 7, 8], [0, 0, 11, 12]]
    assert O.tril(x, 1).tolist() == [[1, 2, 0, 0], [5, 6, 7, 0], [9, 10, 11, 12]]
    assert O.triu(x, -1).tolist() == [[1, 2, 3, 4], [5, 6, 7, 8], [0, 10, 11, 12]]
    assert O.tril(x, -5).tolist() == [[0] * 4] * 3 and O.triu(x, -5).tolist() == x.tolist()
    g = torch.Generator().manual_seed(93)
    for dt in ALL:
        t = (torch.randn(2, 3, 7, 5, generator=g) * 4).to(dt)
        for k in (0, 1, -2, 4, -6, 9):
            assert torch.equal(O.tril(t, k), torch.tril(t, k)) and torch.equal(O.triu(t, k), torch.triu(t, k)), (dt, k)
            v = t.transpose(2, 3)[:, :, ::2]
            assert torch.equal(O.tril(v, k), torch.tril(v, k)) and torch.equal(O.triu(v, k), torch.triu(v, k))
    # tril + triu - diagonal part = x
    f = torch.randn(6, 6, generator=g)
    assert torch.equal(O.tril(f, -1) + O.triu(f), f)
    n = torch.tensor([[NAN, NAN], [NAN, NAN]])
    assert O.tril(n).isnan().tolist() == [[True, False], [True, True]]                    # the zeros are written, not multiplied in
    assert O.tril(torch.empty(0, 3)).shape == (0, 3)
    with pytest.raises(O.OracleError) as e:
        O.tril(torch.ones(5))
    assert e.value.kind == "ndim"
