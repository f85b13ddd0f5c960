"""Pins for the oracle's dimension reductions (sum, mean, prod, amax, argmax, var).

Expected values are closed forms, exact big-integer / math.fsum arithmetic,
and structural invariants that hold for the operator definitions the paper
delegates to (Section 3.2: results must equal the ATen CPU operator's;
Table 1 "Reduction" category).  Nothing here is produced by the oracle or by
the HIP library.
"""
import itertools
import math

import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2512_10977_amd import inputs as I

F32, BF16, F16, I32, I64, B = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool


def close(a, b, rel=1e-6, abs_=0.0):
    return bool(((a.double() - b.double()).abs() <= rel * b.double().abs() + abs_).all())


# --------------------------------------------------------------------------- sum / mean
@pytest.mark.parametrize("n", [1, 7, 1024, 4096])
def test_sum_and_mean_of_arange_closed_form(n):
    assert O.reduce("sum", torch.arange(n)).item() == n * (n - 1) // 2
    xf = torch.arange(n, dtype=F32)
    assert O.reduce("sum", xf).item() == n * (n - 1) / 2          # exact in fp32 for n <= 4096
    assert O.reduce("mean", xf).item() == (n - 1) / 2
    assert O.reduce("sum", torch.arange(n, dtype=I32)).dtype == I64


def test_alternating_signs_cancel():
    x = torch.tensor([1.0, -1.0] * 500 + [1.0])
    assert O.reduce("sum", x).item() == 1.0 and O.reduce("sum", x[:-1]).item() == 0.0


def test_sum_matches_exactly_rounded_sum_on_small_inputs():
    x = I.normal((9, 37), 3.0, seed=40)
    got = O.reduce("sum", x, 1)
    for r in range(9):
        want = np.float32(math.fsum(x[r].tolist()))               # exactly rounded binary64 sum
        assert abs(got[r].item() - float(want)) <= abs(float(want)) * 2.0 ** -23
    got_all = O.reduce("sum", x).item()
    assert abs(got_all - math.fsum(x.flatten().tolist())) <= 1e-5


def test_int64_sum_wraps_and_equals_bigint_sum_mod_2_64():
    vals = [2 ** 62, 2 ** 62, 2 ** 62, 5, -7, 2 ** 62 + 11]
    want = sum(vals) % 2 ** 64
    want = want - 2 ** 64 if want >= 2 ** 63 else want
    assert O.reduce("sum", torch.tensor(vals)).item() == want
    x = I.integers((6, 50), -(2 ** 20), 2 ** 20, seed=41)
    assert O.reduce("sum", x, 0).tolist() == [sum(col) for col in zip(*x.tolist())]
    b = I.booleans((5, 9), 0.5, seed=42)
    s = O.reduce("sum", b, 1)
    assert s.dtype == I64 and s.tolist() == [sum(r) for r in b.tolist()]


def test_half_sum_accumulates_wide_and_rounds_once():
    # 4096 copies of 1 + 2^-7 (exact in bf16): a bf16-accumulated sum would stall; the true sum is 4128
    x = torch.full((4096,), 1.0078125, dtype=BF16)
    assert O.reduce("sum", x).item() == float(torch.tensor(4128.0).to(BF16))
    assert O.reduce("sum", x, out_dtype=F32).item() == 4128.0
    with pytest.raises(O.OracleError):
        O.reduce("mean", torch.arange(4))                         # mean of integers is an error


# --------------------------------------------------------------------------- prod
def test_prod_closed_forms():
    assert O.reduce("prod", torch.arange(1, 13)).item() == 479001600
    assert O.reduce("prod", torch.arange(1, 13, dtype=I32)).dtype == I64
    assert O.reduce("prod", torch.tensor([2.0, 0.5, 4.0, 8.0, 0.125])).item() == 4.0
    assert O.reduce("prod", torch.tensor([2 ** 40, 2 ** 30])).item() == 0                 # wraps mod 2^64
    assert O.reduce("prod", torch.zeros((0,))).item() == 1.0
    assert O.reduce("prod", torch.zeros((3, 0)), 1).tolist() == [1.0, 1.0, 1.0]
    x = torch.tensor([[1.5, -2.0, 3.0], [0.5, 0.5, -0.0]])
    r = O.reduce("prod", x, 1)
    assert r[0].item() == -9.0 and r[1].item() == 0.0 and math.copysign(1, r[1].item()) == -1
    with pytest.raises(O.OracleError) as e:
        O.reduce("prod", torch.ones(2, 3, 4), (0, 2))             # prod takes one dim or all
    assert e.value.kind == "dim"


def test_long_product_underflows_to_signed_zero():
    x = I.normal((1024,), 1.0, seed=43)
    r = O.reduce("prod", x).item()
    neg = int((x < 0).sum().item())
    assert r == 0.0 and math.copysign(1, r) == (-1 if neg % 2 else 1)


# --------------------------------------------------------------------------- amax / argmax
LAYOUTS = ["contig", "transposed", "step2_inner", "step2_outer"]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("dtype", [F32, BF16, I32])
def test_argmax_of_one_hot_is_the_hot_index(layout, dtype):
    shape = (4, 6, 5)
    for hot in [(0, 0, 0), (3, 5, 4), (2, 1, 3)]:
        x = I.make_view(shape, dtype, layout, seed=44)
        x = x.clone() if layout == "contig" else x          # views keep their layout below
        base = torch.zeros(shape, dtype=dtype)
        base[hot] = 1
        if layout != "contig":
            # rebuild the same logical values inside the strided layout
            store = I.make_view(shape, dtype, layout, seed=44)
            store.copy_(base)
            x = store
            assert x.stride() != base.stride()
        else:
            x = base
        flat = (hot[0] * 6 + hot[1]) * 5 + hot[2]
        assert O.reduce("argmax", x).item() == flat                      # logical row-major, not memory order
        for d in range(3):
            r = O.reduce("argmax", x, d)
            kept = tuple(h for i, h in enumerate(hot) if i != d)
            assert r[kept].item() == hot[d]
            r[kept] = 0
            assert int(r.abs().sum()) == 0                               # all-zero slices -> index 0 (first of ties)
            assert O.reduce("amax", x, d)[kept].item() == 1


def test_argmax_ties_and_nan_rules():
    inf, nan = math.inf, math.nan
    assert O.reduce("argmax", torch.tensor([3.0, 7.0, 7.0, 1.0])).item() == 1         # lowest index among ties
    assert O.reduce("argmax", torch.full((9,), 2.5)).item() == 0
    assert O.reduce("argmax", torch.tensor([inf, nan, 5.0])).item() == 1              # NaN outranks +inf
    assert O.reduce("argmax", torch.tensor([1.0, nan, 5.0, nan])).item() == 1         # first NaN wins
    assert O.reduce("argmax", torch.tensor([4, 9, 9, -3])).item() == 1
    assert math.isnan(O.reduce("amax", torch.tensor([1.0, nan, 5.0])).item())
    assert O.reduce("amax", torch.tensor([False, True, False])).item() is True
    with pytest.raises(O.OracleError):
        O.reduce("argmax", torch.tensor([True, False]))
    with pytest.raises(O.OracleError) as e:
        O.reduce("argmax", torch.ones(2, 3, 4), (0, 2))
    assert e.value.kind == "dim"


def test_amax_equals_x_at_argmax():
    x = I.normal((5, 7, 6), 1.0, seed=45, dtype=BF16)        # few distinct values -> real ties
    for d in range(3):
        idx = O.reduce("argmax", x, d, keepdim=True)
        assert torch.equal(torch.gather(x, d, idx), O.reduce("amax", x, d, keepdim=True))
    flat = O.reduce("argmax", x).item()
    assert x.flatten()[flat].item() == O.reduce("amax", x).item()
    assert O.reduce("argmax", x, keepdim=True).shape == (1, 1, 1)


def test_empty_extent_rules():
    with pytest.raises(O.OracleError) as e:
        O.reduce("amax", torch.zeros((3, 0)), 1)
    assert e.value.kind == "empty_reduction"
    with pytest.raises(O.OracleError):
        O.reduce("argmax", torch.zeros((0,)))
    assert O.reduce("amax", torch.zeros((0, 3)), 1).shape == (0,)     # only a kept dim is empty
    assert O.reduce("sum", torch.zeros((3, 0)), 1).tolist() == [0.0, 0.0, 0.0]
    assert all(math.isnan(v) for v in O.reduce("mean", torch.zeros((2, 0)), 1).tolist())
    assert all(math.isnan(v) for v in O.reduce("var", torch.zeros((2, 0)), 1).tolist())


# --------------------------------------------------------------------------- var
@pytest.mark.parametrize("n", [2, 10, 1000])
def test_var_of_arange_closed_form(n):
    x = torch.arange(n, dtype=F32)
    assert abs(O.reduce("var", x).item() - n * (n + 1) / 12) <= 1e-6 * n * n
    assert abs(O.reduce("var", x, correction=0).item() - (n * n - 1) / 12) <= 1e-6 * n * n


def test_var_edge_cases():
    assert O.reduce("var", torch.full((50,), 3.25)).item() == 0.0
    assert math.isnan(O.reduce("var", torch.tensor([2.0])).item())                 # 0/0
    assert O.reduce("var", torch.tensor([2.0]), correction=0).item() == 0.0
    assert O.reduce("var", torch.tensor([1.0, 2.0]), correction=2).item() == math.inf   # divisor clamps at 0
    assert O.reduce("var", torch.tensor([1.0, 2.0]), correction=3).item() == math.inf
    assert math.isnan(O.reduce("var", torch.tensor([1.0, 1.0]), correction=2).item())
    x = I.normal((300,), 1.0, seed=46)
    v0 = O.reduce("var", x).item()
    v1 = O.reduce("var", x + 1024.0).item()                          # shift invariance (x+1024 exact enough)
    assert abs(v0 - v1) <= 2e-3 * v0
    with pytest.raises(O.OracleError):
        O.reduce("var", torch.arange(5))


def test_var_matches_two_pass_definition_in_exact_arithmetic():
    from fractions import Fraction
    x = I.normal((4, 11), 2.0, seed=47)
    got = O.reduce("var", x, 1)
    for r in range(4):
        v = [Fraction(t) for t in x[r].tolist()]
        mu = sum(v) / len(v)
        want = float(sum((t - mu) ** 2 for t in v) / (len(v) - 1))
        assert abs(got[r].item() - want) <= 1e-6 * want


# --------------------------------------------------------------------------- multi-dim / keepdim / views
@pytest.mark.parametrize("op", ["sum", "amax", "mean", "var"])
def test_multi_dim_keepdim_and_flatten_invariants(op):
    x = I.normal((6, 5, 7), 1.0, seed=48)
    r02 = O.reduce(op, x, (0, 2))
    assert r02.shape == (5,)
    if op in ("sum", "amax"):
        step = O.reduce(op, O.reduce(op, x, 0), 1)                 # reduce 0, then old dim 2
        assert close(r02, step, 1e-6, 1e-6)
    # explicit definition on a materialised [5, 42] copy
    flat = x.permute(1, 0, 2).reshape(5, 42)
    assert close(r02, O.reduce(op, flat, 1), 1e-6, 1e-6)
    # keepdim equals the non-keepdim result reshaped
    for dims in (0, 1, -1, (0, 2), (2, 0), None):
        a = O.reduce(op, x, dims, keepdim=True)
        b = O.reduce(op, x, dims)
        assert a.dim() == 3 and torch.equal(a.reshape(b.shape), b)
    # all dims equals the reduction of the flattened copy
    assert close(O.reduce(op, x), O.reduce(op, x.reshape(-1), 0), 1e-6, 1e-6)
    # negative dims wrap; duplicates and out-of-range are errors
    assert torch.equal(O.reduce(op, x, -1), O.reduce(op, x, 2))
    for bad in ((0, 0), (1, -2), 3, -4):
        with pytest.raises(O.OracleError) as e:
            O.reduce(op, x, bad)
        assert e.value.kind == "dim"


@pytest.mark.parametrize("layout", LAYOUTS + ["expand_row", "expand_col"])
def test_reductions_on_views_equal_contiguous_copies(layout):
    x = I.make_view((6, 5, 8), F32, layout, seed=49)
    xi = I.make_view((6, 5, 8), I64, layout, seed=50)
    for op, dims in itertools.product(["sum", "mean", "amax", "argmax", "prod", "var"], [0, 2, None]):
        assert torch.equal(O.reduce(op, x, dims), O.reduce(op, x.contiguous(), dims))
    for op, dims in itertools.product(["sum", "amax", "argmax", "prod"], [1, None]):
        assert torch.equal(O.reduce(op, xi, dims), O.reduce(op, xi.contiguous(), dims))


def test_zero_dim_input():
    x = torch.tensor(3.5)
    for d in (0, -1, None):
        assert O.reduce("sum", x, d).item() == 3.5 and O.reduce("argmax", x, d).item() == 0
    with pytest.raises(O.OracleError):
        O.reduce("sum", x, 1)


def test_library_cross_check_tiny_shapes():
    # non-authoritative: torch CPU on tiny inputs
    x = I.normal((6, 5, 7), 1.0, seed=51)
    xi = I.integers((6, 5, 7), -1000, 1000, seed=52)
    for dims in (0, 1, 2):
        assert close(O.reduce("sum", x, dims), x.sum(dims), 1e-5, 1e-5)
        assert torch.equal(O.reduce("argmax", x, dims), x.argmax(dims))
        assert torch.equal(O.reduce("amax", x, dims), x.amax(dims))
        assert close(O.reduce("var", x, dims), x.var(dims), 1e-5)
        assert close(O.reduce("prod", x, dims), x.prod(dims), 1e-5)
        assert torch.equal(O.reduce("sum", xi, dims), xi.sum(dims))
        assert torch.equal(O.reduce("prod", xi, dims), xi.prod(dims))
    assert close(O.reduce("sum", x, (0, 2)), x.sum((0, 2)), 1e-5, 1e-5)
    assert O.reduce("argmax", x.permute(2, 0, 1)).item() == x.permute(2, 0, 1).argmax().item()
