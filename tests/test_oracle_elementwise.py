"""Pins for the oracle's format codecs, type promotion and elementwise operators.

The paper fixes only the criterion "match the ATen CPU operator on the same
inputs" (Section 3.2) and the operator / dtype set (Section 3.3); the values
below are what the operator definitions and IEEE-754 fix: exact rational
arithmetic, mpmath at 60 digits, closed forms, invariants, and literal
promotion tables.  None of the expected values comes from the oracle itself
or from the HIP library.
"""
import itertools
import math
import struct
from fractions import Fraction

import mpmath
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2512_10977_amd import inputs as I

F32, BF16, F16, I32, I64, B = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool


def bits32(x):
    return struct.unpack("<I", struct.pack("<f", x))[0]


def f32(x):
    return struct.unpack("<f", struct.pack("<f", x))[0]


# --------------------------------------------------------------------------- codecs
def test_f16_decode_all_patterns_matches_format_definition():
    # every binary16 pattern: (-1)^s * 2^(e-15) * (1 + m/1024), subnormals m * 2^-24
    for bits in range(0, 65536, 1):
        s, e, m = bits >> 15, (bits >> 10) & 31, bits & 1023
        got = O.decode(bits, F16)
        if e == 31:
            assert (math.isnan(got) if m else math.isinf(got))
            continue
        want = (m * 2.0 ** -24) if e == 0 else (1 + m / 1024.0) * 2.0 ** (e - 15)
        assert got == (-want if s else want), hex(bits)


def test_bf16_decode_is_top_half_of_f32():
    for bits in list(range(0, 65536, 7)) + [0x3F80, 0x7F7F, 0x0001, 0x8000]:
        got = O.decode(bits, BF16)
        want = struct.unpack("<f", struct.pack("<I", bits << 16))[0]
        assert (math.isnan(got) and math.isnan(want)) or got == want


def test_known_encodings():
    assert O.encode(1.0, F16) == 0x3C00 and O.encode(65504.0, F16) == 0x7BFF
    assert O.encode(2.0 ** -24, F16) == 0x0001 and O.encode(-0.0, F16) == 0x8000
    assert O.encode(1.0, BF16) == 0x3F80 and O.encode(-2.0, BF16) == 0xC000
    assert O.encode(float("inf"), F16) == 0x7C00 and O.encode(float("-inf"), BF16) == 0xFF80


def test_encode_ties_to_even_and_overflow():
    # binary16 has 10 fraction bits: 1 + 2^-11 is a tie between 1 and 1+2^-10
    assert O.encode(1 + 2.0 ** -11, F16) == 0x3C00           # tie -> even (down)
    assert O.encode(1 + 3 * 2.0 ** -11, F16) == 0x3C02       # tie -> even (up)
    assert O.encode(1 + 2.0 ** -11 + 2.0 ** -30, F16) == 0x3C01
    assert O.encode(65519.999, F16) == 0x7BFF and O.encode(65520.0, F16) == 0x7C00
    # subnormal: 2^-25 is a tie between 0 and 2^-24 -> 0; just above -> 2^-24
    assert O.encode(2.0 ** -25, F16) == 0 and O.encode(2.0 ** -25 * 1.0001, F16) == 1
    # largest subnormal rounds up into the smallest normal
    assert O.encode((1023.5 + 1e-9) * 2.0 ** -24, F16) == 0x0400
    # bfloat16 has 7 fraction bits
    assert O.encode(1 + 2.0 ** -8, BF16) == 0x3F80 and O.encode(1 + 3 * 2.0 ** -8, BF16) == 0x3F82


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_encode_matches_library_conversion_from_fp32(dtype):
    # fp32 -> half is a single rounding in torch; fp32 values are exact in binary64
    x = I.normal((20000,), 100.0, seed=11)
    x = torch.cat([x, x * 1e-6, x * 1e-9 if dtype == F16 else x * 1e30, torch.tensor([0.0, -0.0, 65504.0, 65520.0])])
    want = x.to(dtype).view(torch.int16).numpy().astype(np.uint16)
    got = np.array([O.encode(float(v), dtype) for v in x.tolist()], dtype=np.uint16)
    assert np.array_equal(got, want)


# --------------------------------------------------------------------------- promotion
DT = [B, I32, I64, F16, BF16, F32]
# result dtype for two dimensioned operands (row = a, column = b), written out by hand from the
# category rule: bool < integer < floating; wider wins inside a category; fp16 x bf16 -> fp32
SAME_RANK = [
    # bool  i32   i64   f16   bf16  f32
    [B,    I32,  I64,  F16,  BF16, F32],   # bool
    [I32,  I32,  I64,  F16,  BF16, F32],   # i32
    [I64,  I64,  I64,  F16,  BF16, F32],   # i64
    [F16,  F16,  F16,  F16,  F32,  F32],   # f16
    [BF16, BF16, BF16, F32,  BF16, F32],   # bf16
    [F32,  F32,  F32,  F32,  F32,  F32],   # f32
]
# a dimensioned (row), b 0-dim (column): b matters only if its category is strictly higher
DIM_VS_ZERODIM = [
    [B,    I32,  I64,  F16,  BF16, F32],   # bool[3] with ...
    [I32,  I32,  I32,  F16,  BF16, F32],   # i32[3]
    [I64,  I64,  I64,  F16,  BF16, F32],   # i64[3]
    [F16,  F16,  F16,  F16,  F16,  F16],   # f16[3]
    [BF16, BF16, BF16, BF16, BF16, BF16],  # bf16[3]
    [F32,  F32,  F32,  F32,  F32,  F32],   # f32[3]
]


@pytest.mark.parametrize("op", ["add", "mul", "maximum"])
def test_promotion_tables(op):
    for i, j in itertools.product(range(6), range(6)):
        a, b = torch.zeros(3, dtype=DT[i]), torch.zeros(3, dtype=DT[j])
        assert O.infer_binary(op, a, b)[0] == SAME_RANK[i][j], (DT[i], DT[j])
        z = torch.zeros((), dtype=DT[j])
        assert O.infer_binary(op, a, z)[0] == DIM_VS_ZERODIM[i][j], (DT[i], DT[j], "0-dim")
        assert O.infer_binary(op, z, a)[0] == DIM_VS_ZERODIM[i][j]
        # two 0-dim operands promote like same-rank operands
        assert O.infer_binary(op, torch.zeros((), dtype=DT[i]), z)[0] == SAME_RANK[i][j]


def test_promotion_tables_agree_with_library_on_this_machine():
    # non-authoritative cross-check of the hand-written tables against torch's own rule
    for i, j in itertools.product(range(6), range(6)):
        assert torch.result_type(torch.zeros(3, dtype=DT[i]), torch.zeros(3, dtype=DT[j])) == SAME_RANK[i][j]
        assert torch.result_type(torch.zeros(3, dtype=DT[i]), torch.zeros((), dtype=DT[j])) == DIM_VS_ZERODIM[i][j]


def test_div_and_eq_result_dtypes():
    for i, j in itertools.product(range(6), range(6)):
        a, b = torch.zeros(3, dtype=DT[i]), torch.zeros(3, dtype=DT[j])
        common = SAME_RANK[i][j]
        assert O.infer_binary("div", a, b)[0] == (common if common.is_floating_point else F32)
        assert O.infer_binary("eq", a, b)[0] == B


def test_broadcast_shape_rules():
    z = lambda *s: torch.zeros(s)
    assert O.infer_binary("add", z(4096, 1), z(1, 4096))[1] == (4096, 4096)
    assert O.infer_binary("add", z(0, 3), z(3))[1] == (0, 3)
    assert O.infer_binary("add", z(5, 1, 7), z(6, 1))[1] == (5, 6, 7)
    assert O.infer_binary("add", z(), z(2, 2))[1] == (2, 2)
    with pytest.raises(O.OracleError) as e:
        O.infer_binary("add", z(3, 2), z(3))
    assert e.value.kind == "shape"


# --------------------------------------------------------------------------- add / mul (exact class)
def nearest_f32_check(got, exact):
    """`got` (a finite float32 value) is a nearest binary32 to the rational `exact`."""
    g = Fraction(got)
    up = Fraction(float(np.nextafter(np.float32(got), np.float32(np.inf))))
    dn = Fraction(float(np.nextafter(np.float32(got), np.float32(-np.inf))))
    return abs(g - exact) <= abs(up - exact) and abs(g - exact) <= abs(dn - exact)


def test_add_fp32_is_one_ieee_rounding_of_the_exact_sum():
    a, b = I.broadcast_add_inputs(64, 48, seed=0)
    out = O.binary("add", a, b)
    assert out.shape == (64, 48) and out.dtype == F32
    for r in range(0, 64, 5):
        for c in range(0, 48, 7):
            exact = Fraction(a[r, 0].item()) + Fraction(b[0, c].item())
            assert nearest_f32_check(out[r, c].item(), exact)
    # and it is the machine's own binary32 addition
    want = (a.numpy().astype(np.float32) + b.numpy().astype(np.float32))
    assert np.array_equal(out.numpy().view(np.uint32), want.view(np.uint32))


def test_add_alpha_is_a_single_rounding_fma():
    a = I.normal((400,), 3.0, seed=1)
    b = I.normal((400,), 3.0, seed=2)
    for alpha in (0.1, -2.5, 3):
        out = O.binary("add", a, b, alpha=alpha)
        al = Fraction(f32(alpha))
        nfused_differs = 0
        for k in range(400):
            exact = Fraction(a[k].item()) + al * Fraction(b[k].item())
            assert nearest_f32_check(out[k].item(), exact), (alpha, k)
            unfused = np.float32(a[k].item()) + np.float32(f32(alpha)) * np.float32(b[k].item())
            nfused_differs += float(unfused) != out[k].item()
        if alpha == 0.1:
            assert nfused_differs > 0      # the test can tell fused from unfused


def test_mul_fp32_exact_and_integer_wrap():
    a = I.normal((300,), 3.0, seed=3)
    b = I.normal((300,), 3.0, seed=4)
    out = O.binary("mul", a, b)
    for k in range(300):
        assert nearest_f32_check(out[k].item(), Fraction(a[k].item()) * Fraction(b[k].item()))
    assert O.binary("mul", torch.tensor([2 ** 30], dtype=I32), torch.tensor([4], dtype=I32)).item() == 0
    assert O.binary("add", torch.tensor([2 ** 31 - 1], dtype=I32), torch.tensor([1], dtype=I32)).item() == -2 ** 31
    assert O.binary("add", torch.tensor([2 ** 63 - 1]), torch.tensor([1])).item() == -2 ** 63
    assert O.binary("add", torch.tensor([5], dtype=I32), torch.tensor([7], dtype=I32), alpha=-3).item() == -16
    x = I.integers((100,), -1000, 1000, 5, I64)
    y = I.integers((100,), -1000, 1000, 6, I32)
    out = O.binary("add", x, y, alpha=7)
    assert out.dtype == I64 and out.tolist() == [p + 7 * q for p, q in zip(x.tolist(), y.tolist())]


def test_bool_arithmetic():
    t, f = torch.tensor([True]), torch.tensor([False])
    assert O.binary("add", t, t, alpha=2).item() is True
    assert O.binary("add", f, t, alpha=0).item() is False
    assert O.binary("add", f, t).item() is True and O.binary("add", f, f).item() is False
    assert O.binary("mul", t, f).item() is False and O.binary("mul", t, t).item() is True
    assert O.binary("maximum", f, t).item() is True and O.binary("eq", f, f).item() is True


def test_float_alpha_with_integer_tensors_is_an_error():
    with pytest.raises(O.OracleError) as e:
        O.binary("add", torch.ones(3, dtype=I32), torch.ones(3, dtype=I32), alpha=0.5)
    assert e.value.kind == "scalar"


def test_half_add_is_fp32_add_then_one_rounding():
    for dt in (BF16, F16):
        a = I.normal((500,), 3.0, seed=7, dtype=dt)
        b = I.normal((500,), 3.0, seed=8, dtype=dt)
        out = O.binary("add", a, b)
        assert out.dtype == dt
        for k in range(0, 500, 3):
            s32 = f32(a[k].item() + b[k].item())                 # python double sum of two halves is exact
            assert out[k].view(torch.int16).item() & 0xFFFF == O.encode(s32, dt)


def test_conversion_to_common_dtype_happens_before_the_op():
    # 2^24+1 is not representable in fp32: it converts to 2^24 and compares equal
    assert O.binary("eq", torch.tensor([2 ** 24 + 1]), torch.tensor([2.0 ** 24])).item() is True
    assert O.binary("eq", torch.tensor([2 ** 24 + 2]), torch.tensor([2.0 ** 24])).item() is False
    # fp16[.] + fp32 0-dim stays fp16: the 0-dim value is rounded to fp16 first
    out = O.binary("add", torch.tensor([1.0], dtype=F16), torch.tensor(1e-4))
    assert out.dtype == F16
    h = O.decode(O.encode(1e-4, F16), F16)
    assert out.item() == O.decode(O.encode(1.0 + h, F16), F16)


def test_div_special_values_and_integer_division():
    out = O.binary("div", torch.tensor([1, 0, -1, 7], dtype=I32), torch.tensor([0, 0, 0, 2], dtype=I32))
    assert out.dtype == F32
    assert out[0].item() == math.inf and math.isnan(out[1].item()) and out[2].item() == -math.inf
    assert out[3].item() == 3.5
    a = I.normal((300,), 3.0, seed=9)
    b = I.normal((300,), 3.0, seed=10)
    out = O.binary("div", a, b)
    for k in range(300):
        assert nearest_f32_check(out[k].item(), Fraction(a[k].item()) / Fraction(b[k].item()))


def test_maximum_nan_and_eq_semantics():
    nan, inf = math.nan, math.inf
    a = torch.tensor([1.0, nan, 3.0, -inf, nan, -0.0, 5.0])
    b = torch.tensor([2.0, 1.0, nan, inf, nan, 0.0, -5.0])
    m = O.binary("maximum", a, b)
    assert m[0].item() == 2.0 and math.isnan(m[1].item()) and math.isnan(m[2].item())
    assert m[3].item() == inf and math.isnan(m[4].item()) and m[5].item() == 0.0 and m[6].item() == 5.0
    e = O.binary("eq", a, b)
    assert e.tolist() == [False, False, False, False, False, True, False]
    assert O.binary("maximum", torch.tensor([3, -7], dtype=I32), torch.tensor([-4, 9])).tolist() == [3, 9]


# --------------------------------------------------------------------------- where / masked_fill
def test_where_selects_converts_and_preserves_bits():
    c = torch.tensor([True, False, True, False])
    x = torch.tensor([1.5, 2.5, 3.5, 4.5])
    payload = struct.unpack("<f", struct.pack("<I", 0x7FC12345))[0]
    y = torch.tensor([payload, payload, -0.0, -0.0])
    out = O.where(c, x, y)
    assert out[0].item() == 1.5 and out[2].item() == 3.5
    assert out.view(torch.int32)[1].item() == 0x7FC12345            # NaN payload kept
    assert out.view(torch.int32)[3].item() == -2 ** 31               # -0.0 kept
    # promotion incl. the 0-dim rule, and broadcasting of all three operands
    out = O.where(torch.tensor([[True], [False]]), torch.tensor([1, 2, 3], dtype=I32), torch.tensor(2.5))
    assert out.dtype == F32 and out.tolist() == [[1.0, 2.0, 3.0], [2.5, 2.5, 2.5]]
    out = O.where(torch.tensor([True, False]), torch.tensor([7, 8], dtype=I32), torch.tensor(2 ** 40))
    assert out.dtype == I32 and out.tolist() == [7, 0]               # 2^40 wraps to 0 in int32
    with pytest.raises(O.OracleError):
        O.where(torch.tensor([1, 0]), x[:2], y[:2])                  # cond must be bool


def test_masked_fill_definition_and_value_cast():
    s = I.normal((6, 5), 1.0, seed=12)
    m = I.booleans((6, 5), 0.3, seed=13)
    out = O.masked_fill(s, m, -1.0)
    want = torch.where(m, torch.tensor(-1.0), s)
    assert torch.equal(out, want)
    assert torch.equal(O.masked_fill(s, torch.zeros(6, 5, dtype=B), 9.0), s)
    assert torch.equal(O.masked_fill(s, torch.ones(6, 5, dtype=B), 9.0), torch.full((6, 5), 9.0))
    # equals where(mask, full(value), self) computed by the oracle's own where
    assert torch.equal(out, O.where(m, torch.full((6, 5), -1.0), s))
    # broadcast masks [5] and [6,1]
    assert torch.equal(O.masked_fill(s, m[0], 2.0), torch.where(m[0].expand(6, 5), torch.tensor(2.0), s))
    assert torch.equal(O.masked_fill(s, m[:, :1], 2.0), torch.where(m[:, :1].expand(6, 5), torch.tensor(2.0), s))
    # value cast: 2.5 truncates to 2 in an integer tensor; rounds in bf16
    assert O.masked_fill(torch.zeros(2, dtype=I32), torch.tensor([True, False]), 2.5).tolist() == [2, 0]
    assert O.masked_fill(torch.zeros(2, dtype=I32), torch.tensor([True, False]), -2.5).tolist() == [-2, 0]
    o = O.masked_fill(torch.zeros(1, dtype=BF16), torch.tensor([True]), 1.00390625)   # 1 + 2^-8: tie -> 1.0
    assert o.item() == 1.0
    n = O.masked_fill(torch.zeros(2), torch.tensor([True, False]), math.nan)
    assert math.isnan(n[0].item()) and n[1].item() == 0.0


# --------------------------------------------------------------------------- unary, exact class
def test_neg_abs_exact():
    x = torch.tensor([1.5, -0.0, 0.0, math.inf, -math.inf])
    assert O.unary("neg", x).view(torch.int32).tolist() == [bits32(-1.5) - 2 ** 32, 0, -2 ** 31, bits32(-math.inf) - 2 ** 32, bits32(math.inf)]
    assert O.unary("abs", x).tolist() == [1.5, 0.0, 0.0, math.inf, math.inf]
    assert O.unary("abs", torch.tensor([-0.0])).view(torch.int32).item() == 0
    nanbits = torch.tensor([0x7FC00001], dtype=I32).view(F32)
    assert O.unary("neg", nanbits).view(torch.int32).item() == 0x7FC00001 - 2 ** 31
    assert O.unary("abs", O.unary("neg", nanbits)).view(torch.int32).item() == 0x7FC00001
    assert O.unary("neg", torch.tensor([-2 ** 63, 5])).tolist() == [-2 ** 63, -5]
    assert O.unary("abs", torch.tensor([-2 ** 31, -5], dtype=I32)).tolist() == [-2 ** 31, 5]
    for dt in (BF16, F16):
        h = torch.tensor([1.5, -2.0], dtype=dt)
        assert O.unary("neg", h).tolist() == [-1.5, 2.0] and O.unary("abs", h).tolist() == [1.5, 2.0]
    for op in ("neg", "abs"):
        with pytest.raises(O.OracleError):
            O.unary(op, torch.tensor([True]))


# --------------------------------------------------------------------------- unary, transcendental class
MP = {
    "exp": mpmath.exp, "log": mpmath.log, "sqrt": mpmath.sqrt, "tanh": mpmath.tanh,
    "sigmoid": lambda x: 1 / (1 + mpmath.exp(-x)),
    "gelu": lambda x: x * mpmath.ncdf(x),
}


def ulp_distance(a, b):
    """Distance in binary32 steps on the monotone integer mapping of floats."""
    def key(v):
        u = bits32(v)
        return (u & 0x7FFFFFFF) if u < 0x80000000 else -(u & 0x7FFFFFFF)
    return abs(key(a) - key(b))


@pytest.mark.parametrize("op", ["exp", "log", "sqrt", "sigmoid", "tanh", "gelu"])
def test_transcendentals_against_60_digit_arithmetic(op):
    mpmath.mp.dps = 60
    x = I.normal((1500,), 3.0, seed=20)
    if op in ("log", "sqrt"):
        x = x.abs() + 1e-3
    x = torch.cat([x, torch.tensor([-12.5, -9.0, -6.0, -1e-3, 1e-3, 1e-20, 0.5, 20.0, 80.0, -80.0])
                   if op not in ("log", "sqrt") else torch.tensor([1e-30, 1.0, 2.0, 1e30])])
    out = O.unary(op, x)
    worst = 0
    for xi, oi in zip(x.tolist(), out.tolist()):
        want = MP[op](mpmath.mpf(xi))
        wf = f32(float(want))                       # 60 digits -> binary64 -> binary32
        worst = max(worst, ulp_distance(oi, wf))
    assert worst <= 1, worst                        # at most a double-rounding slip


def test_transcendental_special_values():
    inf, nan = math.inf, math.nan
    t = lambda *v: torch.tensor(v, dtype=F32)
    assert O.unary("exp", t(-inf, inf, 0.0)).tolist() == [0.0, inf, 1.0]
    r = O.unary("log", t(0.0, -0.0, -1.0, inf, 1.0)).tolist()
    assert r[0] == -inf and r[1] == -inf and math.isnan(r[2]) and r[3] == inf and r[4] == 0.0
    r = O.unary("sqrt", t(-0.0, -1.0, 4.0, inf))
    assert r.view(torch.int32)[0].item() == -2 ** 31 and math.isnan(r[1].item()) and r[2].item() == 2.0 and r[3].item() == inf
    assert O.unary("sigmoid", t(-inf, inf, 0.0)).tolist() == [0.0, 1.0, 0.5]
    r = O.unary("tanh", t(-inf, inf, -0.0))
    assert r.tolist()[:2] == [-1.0, 1.0] and r.view(torch.int32)[2].item() == -2 ** 31
    r = O.unary("gelu", t(-0.0, nan, inf, -inf))
    assert r.view(torch.int32)[0].item() == -2 ** 31 and math.isnan(r[1].item())
    assert r[2].item() == inf and math.isnan(r[3].item())     # literal IEEE evaluation of x * Phi(x)
    for op in ("exp", "log", "sqrt", "sigmoid", "tanh", "gelu"):
        assert math.isnan(O.unary(op, t(nan)).item())


def test_transcendental_identities():
    x = I.normal((2000,), 3.0, seed=21).double()
    xf = x.float()
    d = lambda t: t.double()
    # tanh(x) = 2*sigmoid(2x) - 1
    lhs = d(O.unary("tanh", xf))
    rhs = 2 * d(O.unary("sigmoid", 2 * xf)) - 1
    assert (lhs - rhs).abs().max() < 3e-7
    # gelu(x) - gelu(-x) = x
    g = d(O.unary("gelu", xf)) - d(O.unary("gelu", -xf))
    assert ((g - d(xf)).abs() <= 2e-7 * d(xf).abs() + 1e-30).all()
    # exp(log x) ~ x, sqrt(x)^2 ~ x
    p = xf.abs() + 0.01
    assert ((d(O.unary("exp", O.unary("log", p))) - d(p)).abs() <= 1e-5 * d(p)).all()
    assert ((d(O.unary("sqrt", p)) ** 2 - d(p)).abs() <= 2e-7 * d(p)).all()


def test_integral_inputs_to_float_ops_and_dtype_errors():
    for dt in (B, I32, I64):
        x = torch.tensor([0, 1, 1], dtype=dt)
        out = O.unary("exp", x)
        assert out.dtype == F32 and out.tolist() == [1.0, f32(math.e), f32(math.e)]
        with pytest.raises(O.OracleError):
            O.unary("gelu", x)
    assert O.unary("sqrt", torch.tensor([16, 2], dtype=I64)).tolist() == [4.0, f32(math.sqrt(2))]


def test_half_transcendentals_round_once():
    mpmath.mp.dps = 40
    for dt in (BF16, F16):
        x = I.normal((300,), 2.0, seed=22, dtype=dt)
        out = O.unary("exp", x)
        for xi, oi in zip(x.tolist(), out.view(torch.int16).tolist()):
            want = O.encode(float(mpmath.exp(mpmath.mpf(xi))), dt)
            assert (oi & 0xFFFF) == want


# --------------------------------------------------------------------------- broadcasting and views
BIN_OPS = ["add", "mul", "div", "maximum", "eq"]


def same_bits(a, b):
    if a.dtype.is_floating_point:
        both_nan = a.isnan() & b.isnan()
        ia = a.contiguous().view(torch.int16 if a.element_size() == 2 else torch.int32)
        ib = b.contiguous().view(torch.int16 if b.element_size() == 2 else torch.int32)
        return bool(((ia == ib) | both_nan).all())
    return torch.equal(a, b)


@pytest.mark.parametrize("op", BIN_OPS)
@pytest.mark.parametrize("dtype", [F32, BF16, I32, B])
def test_broadcast_equals_explicit_expand(op, dtype):
    a = I.typed((7, 1, 5), dtype, seed=30, specials=0.05)
    b = I.typed((13, 1), dtype, seed=31, specials=0.05)
    out = O.binary(op, a, b)
    assert out.shape == (7, 13, 5)
    ea, eb = a.expand(7, 13, 5).contiguous(), b.expand(7, 13, 5).contiguous()
    assert same_bits(out, O.binary(op, ea, eb))
    # a 0-dim operand behaves like a shape-[1] operand numerically
    z = I.typed((), dtype, seed=32)
    assert same_bits(O.binary(op, a, z), O.binary(op, a, z.reshape(1)))


@pytest.mark.parametrize("kind", I.VIEW_KINDS)
@pytest.mark.parametrize("dtype", [F32, F16, I64])
def test_strided_views_equal_their_contiguous_copies(kind, dtype):
    a = I.make_view((7, 13, 5), dtype, kind, seed=33, specials=0.02)
    b = I.make_view((7, 13, 5), dtype, "contig", seed=34, specials=0.02)
    assert not (kind in ("transposed", "step2_inner", "expand_row") and a.is_contiguous())
    for op in BIN_OPS:
        assert same_bits(O.binary(op, a, b), O.binary(op, a.contiguous(), b))
        assert same_bits(O.binary(op, b, a), O.binary(op, b, a.contiguous()))
    uop = "exp" if dtype.is_floating_point else "neg"
    assert same_bits(O.unary(uop, a), O.unary(uop, a.contiguous()))
    # strided output: writing through a transposed out view gives the same values
    out_t = torch.empty((5, 7, 13), dtype=O.infer_binary("add", a, b)[0]).permute(1, 2, 0)
    O.binary("add", a, b, out=out_t)
    assert same_bits(out_t.contiguous(), O.binary("add", a, b))


def test_empty_and_zero_dim():
    for dt in DT:
        e = torch.zeros((0,), dtype=dt)
        assert O.binary("add", e, e).shape == (0,)
        z = I.typed((), dt, seed=35)
        r = O.binary("mul", z, z)
        assert r.shape == () and r.dtype == dt
    assert O.binary("add", torch.zeros((0, 3)), torch.ones(3)).shape == (0, 3)
    assert O.unary("exp", torch.tensor(0.0)).item() == 1.0


def test_library_cross_check_tiny_shapes():
    # non-authoritative: torch CPU on the same tiny inputs, for the ops whose semantics are not in question
    for dt in (F32, I32, I64):
        a = I.typed((7, 13, 5), dt, seed=36)
        b = I.typed((13, 1), dt, seed=37)
        assert torch.equal(O.binary("add", a, b), torch.add(a, b))
        assert torch.equal(O.binary("mul", a, b), torch.mul(a, b))
        assert torch.equal(O.binary("maximum", a, b), torch.maximum(a, b))
        assert torch.equal(O.binary("eq", a, b), torch.eq(a, b))
    a = I.typed((7, 13, 5), F32, seed=38)
    b = I.typed((13, 1), F32, seed=39)
    assert torch.equal(O.binary("div", a, b), torch.div(a, b))
    # alpha != 1: the library's vectorised same-shape path is a fused multiply-add like the oracle
    # (its scalar broadcast path is not, so only the same-shape case is compared)
    bb = b.expand(7, 13, 5).contiguous()
    assert torch.equal(O.binary("add", a, bb, alpha=0.3), torch.add(a, bb, alpha=0.3))
    for op, fn in (("exp", torch.exp), ("tanh", torch.tanh), ("sigmoid", torch.sigmoid)):
        got, want = O.unary(op, a), fn(a)
        assert ((got - want).abs() <= 4e-7 * want.abs() + 1e-37).all()
