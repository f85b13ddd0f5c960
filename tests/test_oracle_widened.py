"""Pins for the oracle's second batch of operators: sub, minimum, the comparison
family, log1p / expm1 / logsigmoid, amin / argmin, std, any / all, logsumexp.

These are further members of the two largest categories of the paper's
operator set (Table 1: "Elementwise", "Reduction"; logsigmoid and log1p are the
worked examples of Appendix D).  As for the first batch, the paper delegates
their definitions to the ATen CPU operators (Section 3.2); the expected values
here are exact rational arithmetic, mpmath at 60 digits, closed forms,
invariants and truth tables - nothing comes from the oracle itself or from the
HIP library.
"""
import itertools
import math
import struct
from fractions import Fraction

import mpmath
import pytest
import torch

from oracle import oracle as O
from paper_2512_10977_amd import inputs as I

F32, BF16, F16, I32, I64, B = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool


def f32(x):
    return struct.unpack("<f", struct.pack("<f", x))[0]


def bits32(x):
    return struct.unpack("<I", struct.pack("<f", x))[0]


def ulp_distance(a, b):
    def key(v):
        u = bits32(v)
        return (u & 0x7FFFFFFF) if u < 0x80000000 else -(u & 0x7FFFFFFF)
    return abs(key(a) - key(b))


def round_to_f32(q):
    """Nearest-even binary32 value of an exact Fraction (normal range)."""
    if q == 0:
        return 0.0
    return f32(float(q)) if abs(Fraction(float(q)) - q) == 0 else _round_fraction(q)


def _round_fraction(q):
    # binary64 conversion of a Fraction is correctly rounded in Python; a second rounding to binary32 can only go
    # wrong when the binary64 value lies exactly on a binary32 tie, which the two neighbours below rule out
    d = float(q)
    lo, hi = f32(d), f32(d)
    cands = {f32(d), f32(math.nextafter(d, math.inf)), f32(math.nextafter(d, -math.inf))}
    for c in list(cands):
        cands.add(struct.unpack("<f", struct.pack("<I", (bits32(c) + 1) & 0xFFFFFFFF))[0])
        cands.add(struct.unpack("<f", struct.pack("<I", (bits32(c) - 1) & 0xFFFFFFFF))[0])
    cands = [c for c in cands if math.isfinite(c)]
    best = min(cands, key=lambda c: (abs(Fraction(c) - q), bits32(c) & 1))
    return best


# --------------------------------------------------------------------------- sub
def test_sub_fp32_is_one_rounding_of_the_exact_difference():
    a = I.normal((400,), 100.0, seed=501)
    b = I.normal((400,), 100.0, seed=502) * 1e-3
    out = O.binary("sub", a, b)
    for x, y, o in zip(a.tolist(), b.tolist(), out.tolist()):
        assert o == round_to_f32(Fraction(x) - Fraction(y))


def test_sub_alpha_is_a_single_rounding_of_a_minus_alpha_b():
    a = I.normal((300,), 10.0, seed=503)
    b = I.normal((300,), 10.0, seed=504)
    for alpha in (2.5, -0.75, 3):
        out = O.binary("sub", a, b, alpha=alpha)
        al = Fraction(f32(float(alpha)))
        for x, y, o in zip(a.tolist(), b.tolist(), out.tolist()):
            assert o == round_to_f32(Fraction(x) - al * Fraction(y)), (x, y, alpha)


def test_sub_integers_wrap_and_bool_is_rejected():
    a = torch.tensor([-2 ** 31, 5, 7], dtype=I32)
    b = torch.tensor([1, -3, 7], dtype=I32)
    assert O.binary("sub", a, b).tolist() == [2 ** 31 - 1, 8, 0]                 # two's complement wrap
    assert O.binary("sub", a, b, alpha=3).tolist() == [((-2 ** 31 - 3 + 2 ** 31) % 2 ** 32) - 2 ** 31, 14, -14]
    big = torch.tensor([2 ** 63 - 1], dtype=I64)
    assert O.binary("sub", big, torch.tensor([-1])).tolist() == [-2 ** 63]
    assert O.binary("sub", torch.tensor([5], dtype=I32), torch.tensor([7])).dtype == I64
    assert O.binary("sub", torch.tensor([5]), torch.tensor([0.5])).tolist() == [4.5]
    for x, y in [(torch.tensor([True]), torch.tensor([True])), (torch.tensor([True]), torch.tensor([1])),
                 (torch.tensor([1.0]), torch.tensor([False]))]:
        with pytest.raises(O.OracleError) as e:
            O.binary("sub", x, y)
        assert e.value.kind == "dtype"
    with pytest.raises(O.OracleError) as e:
        O.binary("sub", torch.tensor([1]), torch.tensor([2]), alpha=0.5)
    assert e.value.kind == "scalar"


def test_sub_is_add_of_the_negated_operand():
    a = I.typed((7, 13, 5), F32, seed=505, specials=0.02)
    b = I.typed((13, 1), F32, seed=506, specials=0.02)
    s = O.binary("sub", a, b)
    t = O.binary("add", a, O.unary("neg", b))
    assert torch.equal(s.view(torch.int32)[~s.isnan()], t.view(torch.int32)[~t.isnan()]) and torch.equal(s.isnan(), t.isnan())
    h = I.typed((64,), BF16, seed=507)
    g = I.typed((64,), BF16, seed=508)
    assert torch.equal(O.binary("sub", h, g), (h.float() - g.float()).to(BF16))      # fp32 arithmetic, one rounding


# --------------------------------------------------------------------------- minimum / comparisons
def test_minimum_nan_zero_and_integer_rules():
    nan, inf = math.nan, math.inf
    a = torch.tensor([1.0, nan, 3.0, -inf, nan, -0.0, 0.0, 5.0])
    b = torch.tensor([2.0, 1.0, nan, inf, nan, 0.0, -0.0, -5.0])
    m = O.binary("minimum", a, b)
    assert m[0].item() == 1.0 and math.isnan(m[1].item()) and math.isnan(m[2].item())
    assert m[3].item() == -inf and math.isnan(m[4].item()) and m[7].item() == -5.0
    assert m.view(torch.int32)[5].item() == -2 ** 31 and m.view(torch.int32)[6].item() == 0    # equal operands: the first
    assert O.binary("minimum", torch.tensor([3, -7], dtype=I32), torch.tensor([-4, 9])).tolist() == [-4, -7]
    assert O.binary("minimum", torch.tensor([True, True, False]), torch.tensor([True, False, False])).tolist() == [True, False, False]
    x = I.typed((200,), F32, seed=510)
    y = I.typed((200,), F32, seed=511)
    lo, hi = O.binary("minimum", x, y), O.binary("maximum", x, y)
    assert torch.equal(O.binary("add", lo, hi), O.binary("add", x, y))            # {min, max} = {x, y}
    assert torch.equal(lo, O.unary("neg", O.binary("maximum", O.unary("neg", x), O.unary("neg", y))))


CMP = {"eq": lambda p, q: p == q, "ne": lambda p, q: p != q, "lt": lambda p, q: p < q, "le": lambda p, q: p <= q,
       "gt": lambda p, q: p > q, "ge": lambda p, q: p >= q}


@pytest.mark.parametrize("op", list(CMP))
def test_comparison_truth_tables(op):
    nan, inf = math.nan, math.inf
    vals = [-inf, -1.5, -0.0, 0.0, 1.5, inf, nan]
    a = torch.tensor([p for p in vals for _ in vals])
    b = torch.tensor([q for _ in vals for q in vals])
    got = O.binary(op, a, b)
    assert got.dtype == B
    assert got.tolist() == [CMP[op](p, q) for p in vals for q in vals]             # Python floats follow IEEE 754
    ints = [-2 ** 31, -1, 0, 1, 2 ** 31 - 1]
    ai = torch.tensor([p for p in ints for _ in ints], dtype=I32)
    bi = torch.tensor([q for _ in ints for q in ints], dtype=I32)
    assert O.binary(op, ai, bi).tolist() == [CMP[op](p, q) for p in ints for q in ints]
    bb = [False, True]
    assert O.binary(op, torch.tensor([p for p in bb for _ in bb]), torch.tensor([q for _ in bb for q in bb])).tolist() == \
        [CMP[op](p, q) for p in bb for q in bb]


def test_comparisons_happen_in_the_common_dtype():
    # int64 2^24 + 1 converted to fp32 is 2^24: equal to 16777216.0 after promotion, not before
    a = torch.tensor([2 ** 24 + 1, 5], dtype=I64)
    b = torch.tensor([16777216.0, 5.5], dtype=F32)
    assert O.binary("eq", a, b).tolist() == [True, False] and O.binary("lt", a, b).tolist() == [False, True]
    assert O.binary("ge", a, b).tolist() == [True, False] and O.binary("ne", a, b).tolist() == [False, True]
    # bf16 vs fp16 promote to fp32: no rounding of either operand
    x = torch.tensor([1.0078125], dtype=BF16)          # 1 + 2^-7, not representable in fp16 ... but exact in fp32
    y = torch.tensor([1.0078125], dtype=F16)           # fp16 has 10 fraction bits: exact too
    assert O.binary("eq", x, y).item() is True
    assert O.binary("gt", torch.tensor([3], dtype=I32), torch.tensor(2.5)).tolist() == [True]      # 0-dim float decides
    r = O.binary("le", torch.zeros(4, 1), torch.tensor([-1.0, 0.0, 1.0]))
    assert r.shape == (4, 3) and r[0].tolist() == [False, True, True]


def test_comparison_complements_and_library_cross_check():
    x = I.typed((7, 13, 5), F32, seed=512, specials=0.05)
    y = I.typed((7, 13, 5), F32, seed=513, specials=0.05)
    y[::2] = x[::2]
    ordered = ~(x.isnan() | y.isnan())
    assert torch.equal(O.binary("ne", x, y), ~O.binary("eq", x, y))
    assert torch.equal(O.binary("ge", x, y)[ordered], ~O.binary("lt", x, y)[ordered])
    assert torch.equal(O.binary("le", x, y), O.binary("ge", y, x))
    assert not O.binary("lt", x, y)[~ordered].any() and O.binary("ne", x, y)[~ordered].all()
    for op, ref in (("lt", torch.lt), ("le", torch.le), ("gt", torch.gt), ("ge", torch.ge), ("ne", torch.ne)):
        for da, db in itertools.product((F32, BF16, I32, I64, B), repeat=2):
            a = I.typed((6, 5), da, seed=514)
            b = I.typed((5,), db, seed=515)
            assert torch.equal(O.binary(op, a, b), ref(a, b)), (op, da, db)
    for da, db in itertools.product((F32, F16, I32, I64), repeat=2):
        a, b = I.typed((6, 5), da, seed=516), I.typed((6, 1), db, seed=517)
        assert torch.equal(O.binary("minimum", a, b), torch.minimum(a, b)), (da, db)
        assert torch.equal(O.binary("sub", a, b), torch.sub(a, b)), (da, db)


# --------------------------------------------------------------------------- log1p / expm1 / logsigmoid
MP = {"log1p": lambda v: mpmath.log1p(v), "expm1": lambda v: mpmath.expm1(v),
      "logsigmoid": lambda v: -mpmath.log1p(mpmath.exp(-v))}


@pytest.mark.parametrize("op", list(MP))
def test_new_transcendentals_against_60_digit_arithmetic(op):
    mpmath.mp.dps = 60
    x = I.normal((1500,), 3.0, seed=520)
    extra = [1e-30, -1e-30, 1e-10, -1e-10, 1e-4, -1e-4, 0.5, 20.0, 80.0]
    if op == "log1p":
        x = torch.cat([x.abs() * 3 - 0.999, torch.tensor(extra + [1e30, -0.9999999])])
    else:
        x = torch.cat([x, torch.tensor(extra + [-20.0, -80.0, -103.0])])
    out = O.unary(op, x)
    worst = 0
    for xi, oi in zip(x.tolist(), out.tolist()):
        wf = f32(float(MP[op](mpmath.mpf(xi))))
        worst = max(worst, ulp_distance(oi, wf))
    assert worst <= 1, worst


def test_new_transcendentals_special_values_and_identities():
    inf, nan = math.inf, math.nan
    t = lambda *v: torch.tensor(v, dtype=F32)
    r = O.unary("log1p", t(-1.0, -2.0, 0.0, -0.0, inf)).tolist()
    assert r[0] == -inf and math.isnan(r[1]) and r[2] == 0.0 and r[4] == inf
    assert O.unary("log1p", t(-0.0)).view(torch.int32).item() == -2 ** 31
    assert O.unary("expm1", t(-inf, inf, 0.0)).tolist() == [-1.0, inf, 0.0]
    assert O.unary("expm1", t(-0.0)).view(torch.int32).item() == -2 ** 31
    assert O.unary("logsigmoid", t(inf, -inf, 0.0)).tolist() == [0.0, -inf, f32(-math.log(2.0))]
    for op in MP:
        assert math.isnan(O.unary(op, t(nan)).item())
    # tiny arguments: log1p(x) ~ x, expm1(x) ~ x to the last bit; logsigmoid(x) ~ x for very negative x
    tiny = t(1e-20, -3e-25, 7e-12)
    assert torch.equal(O.unary("log1p", tiny), tiny) and torch.equal(O.unary("expm1", tiny), tiny)
    assert O.unary("logsigmoid", t(-50.0, -90.0)).tolist() == [-50.0, -90.0]
    big = 3.0e38                                                                  # exp(|x|) overflows even binary64
    assert O.unary("logsigmoid", t(-1000.0, 1000.0, -big, big)).tolist() == [-1000.0, 0.0, f32(-big), 0.0]
    x = I.normal((2000,), 2.0, seed=521)
    d = lambda v: v.double()
    back = d(O.unary("log1p", O.unary("expm1", x.abs())))                          # well conditioned for x >= 0
    assert ((back - d(x.abs())).abs() <= 3e-7 * d(x.abs()) + 1e-30).all()
    ls = d(O.unary("logsigmoid", x)) - d(O.unary("logsigmoid", -x))              # logsigmoid(x) - logsigmoid(-x) = x
    assert ((ls - d(x)).abs() <= 3e-7 * (d(x).abs() + 1)).all()
    sg = d(O.unary("sigmoid", x)).log()                                           # = log(sigmoid(x)) where that is accurate
    assert ((d(O.unary("logsigmoid", x)) - sg).abs() <= 2e-7 * sg.abs() + 1e-7).all()


def test_new_transcendentals_dtypes():
    for dt in (B, I32, I64):
        x = torch.tensor([0, 1, 1], dtype=dt)
        for op, want in (("log1p", math.log(2.0)), ("expm1", math.e - 1)):
            out = O.unary(op, x)
            assert out.dtype == F32 and out.tolist() == [0.0, f32(want), f32(want)]
        with pytest.raises(O.OracleError):
            O.unary("logsigmoid", x)
    # half types: evaluated on the exact half value, rounded once
    mpmath.mp.dps = 40
    for dt in (BF16, F16):
        x = I.normal((300,), 2.0, seed=522, dtype=dt)
        for op in ("expm1", "logsigmoid"):
            out = O.unary(op, x)
            assert out.dtype == dt
            for xi, oi in zip(x.tolist(), out.tolist()):
                want = torch.tensor(float(MP[op](mpmath.mpf(xi))), dtype=torch.float64).to(dt).item()
                assert oi == want or (math.isinf(want) and math.isinf(oi)), (op, xi, oi, want)


# --------------------------------------------------------------------------- amin / argmin
def test_amin_argmin_mirror_amax_argmax():
    x = I.normal((5, 7, 6), 1.0, seed=530, dtype=BF16)
    for d in (0, 1, 2, None):
        assert torch.equal(O.reduce("amin", x, d), O.unary("neg", O.reduce("amax", O.unary("neg", x), d)))
        assert torch.equal(O.reduce("argmin", x, d), O.reduce("argmax", O.unary("neg", x), d))
    xi = I.integers((4, 9), -50, 50, seed=531)
    assert torch.equal(O.reduce("amin", xi, 1), xi.min(1).values)
    idx = O.reduce("argmin", xi, 1, keepdim=True)
    assert torch.equal(torch.gather(xi, 1, idx), O.reduce("amin", xi, 1, keepdim=True))


def test_argmin_ties_nan_and_errors():
    inf, nan = math.inf, math.nan
    assert O.reduce("argmin", torch.tensor([3.0, 1.0, 1.0, 7.0])).item() == 1         # lowest index among ties
    assert O.reduce("argmin", torch.tensor([-inf, nan, 5.0])).item() == 1             # NaN outranks -inf
    assert O.reduce("argmin", torch.tensor([1.0, nan, 5.0, nan])).item() == 1         # first NaN wins
    assert math.isnan(O.reduce("amin", torch.tensor([1.0, nan, -5.0])).item())
    assert O.reduce("amin", torch.tensor([True, True, False])).item() is False
    assert O.reduce("argmin", torch.tensor([[4, -9, -9], [0, 0, -1]]), 1).tolist() == [1, 2]
    assert O.reduce("argmin", torch.tensor([[4, -9, -9], [0, 0, -10]])).item() == 5   # flat logical index
    with pytest.raises(O.OracleError):
        O.reduce("argmin", torch.tensor([True, False]))
    with pytest.raises(O.OracleError) as e:
        O.reduce("argmin", torch.ones(2, 3, 4), (0, 2))
    assert e.value.kind == "dim"
    with pytest.raises(O.OracleError) as e:
        O.reduce("amin", torch.zeros((3, 0)), 1)
    assert e.value.kind == "empty_reduction"


# --------------------------------------------------------------------------- std
@pytest.mark.parametrize("n", [2, 9, 1000])
def test_std_of_arange_closed_form(n):
    x = torch.arange(n, dtype=F32)
    assert O.reduce("std", x).item() == f32(math.sqrt(n * (n + 1) / 12.0))            # unbiased variance of 0..n-1
    assert O.reduce("std", x, correction=0.0).item() == f32(math.sqrt((n * n - 1) / 12.0))


def test_std_is_sqrt_of_var_and_edge_cases():
    x = I.normal((6, 50, 7), 2.0, seed=532).double().float()
    for dims in (0, 1, (0, 2), None):
        s = O.reduce("std", x, dims).double()
        v = O.reduce("var", x, dims).double()
        assert ((s * s - v).abs() <= 3e-7 * v).all()
    assert math.isnan(O.reduce("std", torch.tensor([3.0])).item())                    # n - 1 = 0 -> 0/0
    assert O.reduce("std", torch.tensor([3.0]), correction=0.0).item() == 0.0
    assert math.isinf(O.reduce("std", torch.tensor([1.0, 2.0]), correction=2.0).item())
    assert all(math.isnan(v) for v in O.reduce("std", torch.zeros((2, 0)), 1).tolist())
    assert O.reduce("std", torch.full((40,), 1e10)).item() == 0.0                     # two-pass: no cancellation
    with pytest.raises(O.OracleError):
        O.reduce("std", torch.tensor([1, 2]))
    h = I.normal((3, 200), 1.0, seed=533, dtype=F16)
    assert torch.equal(O.reduce("std", h, 1), h.double().std(1).to(F16))              # binary64 inside, one rounding


# --------------------------------------------------------------------------- any / all
def test_any_all_truth_and_dtypes():
    nan = math.nan
    assert O.reduce("any", torch.tensor([0.0, -0.0, 0.0])).item() is False
    assert O.reduce("any", torch.tensor([0.0, nan])).item() is True                   # NaN is not zero
    assert O.reduce("all", torch.tensor([1.0, nan, -3.0])).item() is True
    assert O.reduce("all", torch.tensor([1.0, -0.0])).item() is False
    assert O.reduce("any", torch.zeros((0,))).item() is False and O.reduce("all", torch.zeros((0,))).item() is True
    assert O.reduce("any", torch.zeros((3, 0)), 1).tolist() == [False] * 3
    assert O.reduce("all", torch.zeros((3, 0)), 1).tolist() == [True] * 3
    for dt in (F32, BF16, F16, I32, I64, B):
        x = I.typed((5, 6, 4), dt, seed=534)
        x[1] = 0
        x[:, 2] = 1
        for dims in (0, 1, 2, (0, 2), None):
            nz = x != 0
            want_any = nz.sum(dims).ne(0) if dims is not None else nz.sum().ne(0)
            cnt = 1
            for d in ((dims,) if isinstance(dims, int) else (dims or range(3))):
                cnt *= x.shape[d]
            want_all = (nz.sum(dims) if dims is not None else nz.sum()).eq(cnt)
            got_any, got_all = O.reduce("any", x, dims), O.reduce("all", x, dims)
            assert got_any.dtype == B and torch.equal(got_any, want_any), (dt, dims)
            assert torch.equal(got_all, want_all), (dt, dims)
    assert O.reduce("any", x, (0, 1), keepdim=True).shape == (1, 1, 4)
    # De Morgan: all(x) == not any(not x)
    b = I.booleans((7, 9), 0.8, seed=535)
    assert torch.equal(O.reduce("all", b, 1), ~O.reduce("any", ~b, 1))


# --------------------------------------------------------------------------- logsumexp
def test_logsumexp_against_60_digit_arithmetic_and_closed_forms():
    mpmath.mp.dps = 60
    x = I.normal((40, 33), 4.0, seed=540)
    out = O.reduce("logsumexp", x, 1)
    for row, o in zip(x.tolist(), out.tolist()):
        want = mpmath.log(mpmath.fsum(mpmath.exp(mpmath.mpf(v)) for v in row))
        assert ulp_distance(o, f32(float(want))) <= 1
    for n, v in ((1, 3.25), (8, -2.0), (1000, 100.0), (7, -1e4)):
        got = O.reduce("logsumexp", torch.full((n,), v)).item()
        assert got == f32(v + math.log(n))                                           # n equal terms
    big = torch.tensor([1000.0, 1000.0, -1000.0])
    assert O.reduce("logsumexp", big).item() == f32(1000.0 + math.log(2.0))           # no overflow


def test_logsumexp_invariants_and_special_values():
    inf, nan = math.inf, math.nan
    x = I.normal((9, 64), 3.0, seed=541)
    base = O.reduce("logsumexp", x, 1).double()
    shifted = O.reduce("logsumexp", x + 8.0, 1).double()                              # adding 8 is exact for these
    assert ((shifted - base - 8.0).abs() <= 4e-7 * (base.abs() + 8)).all()
    assert (base >= x.double().amax(1)).all() and (base <= x.double().amax(1) + math.log(64) + 1e-6).all()
    sm = O.softmax(x, 1).double()                                                     # softmax = exp(x - logsumexp)
    assert ((x.double() - base[:, None]).exp() - sm).abs().max() < 6e-7            # base itself is rounded to fp32
    assert O.reduce("logsumexp", torch.tensor([-inf, 2.0, -inf])).item() == 2.0
    assert O.reduce("logsumexp", torch.tensor([-inf, -inf])).item() == -inf
    assert O.reduce("logsumexp", torch.tensor([1.0, inf])).item() == inf
    assert math.isnan(O.reduce("logsumexp", torch.tensor([1.0, nan, inf])).item())
    assert math.isnan(O.reduce("logsumexp", torch.tensor([inf, -inf, nan])).item())
    assert O.reduce("logsumexp", torch.zeros((2, 0)), 1).tolist() == [-inf, -inf]     # empty sum: log 0
    # bool / integer input is converted to fp32 (as the ATen CPU operator does): log(e^1 + e^2), log(e^1 + e^0)
    r = O.reduce("logsumexp", torch.tensor([1, 2]))
    assert r.dtype == torch.float32 and r.item() == torch.tensor(math.log(math.e + math.e ** 2), dtype=torch.float64).float().item()
    r = O.reduce("logsumexp", torch.tensor([True, False]))
    assert r.dtype == torch.float32 and r.item() == torch.tensor(math.log(math.e + 1.0), dtype=torch.float64).float().item()
    y = I.normal((4, 6, 5), 2.0, seed=542)
    for dims in (0, (0, 2), None):
        ref = torch.logsumexp(y.double(), dims if dims is not None else (0, 1, 2)).float()
        assert torch.equal(O.reduce("logsumexp", y, dims), ref) or \
            ((O.reduce("logsumexp", y, dims).double() - ref.double()).abs() <= 2e-7 * ref.double().abs()).all()
    h = I.normal((5, 100), 2.0, seed=543, dtype=BF16)
    assert torch.equal(O.reduce("logsumexp", h, 1), torch.logsumexp(h.double(), 1).to(BF16))
