"""Pins for the oracle's layer_norm and binary_cross_entropy.

Both operators are worked examples of the paper (Appendix B.1 binary_cross_entropy,
Appendix B.3 layer_norm) and belong to its "Deep Learning" category (Table 1).
Their definition is the ATen CPU operator's (Section 3.2).  Expected values here
are closed forms, invariants of the two formulas, mpmath at 50 digits and the
ATen CPU operators themselves - nothing comes from the oracle or the HIP library.
"""
import math

import mpmath
import pytest
import torch
import torch.nn.functional as F

from oracle import oracle as O

F32, BF16, F16, F64 = torch.float32, torch.bfloat16, torch.float16, torch.float64
NAN = float("nan")


def mp_layer_norm_row(xs, ws, bs, eps):
    mpmath.mp.dps = 50
    xs = [mpmath.mpf(v) for v in xs]
    m = sum(xs) / len(xs)
    var = sum((v - m) ** 2 for v in xs) / len(xs)
    rstd = 1 / mpmath.sqrt(var + mpmath.mpf(eps))
    return [(v - m) * rstd * mpmath.mpf(w) + mpmath.mpf(b) for v, w, b in zip(xs, ws, bs)]


# --------------------------------------------------------------------------- layer_norm
def test_layer_norm_closed_form_row():
    # 1 2 3 4: mean 5/2, biased variance 5/4; with eps = 0 the outputs are (x - 5/2) / sqrt(5/4)
    x = torch.tensor([[1.0, 2.0, 3.0, 4.0]])
    got = O.layer_norm(x, 1, eps=0.0)[0].tolist()
    for xv, g in zip([1, 2, 3, 4], got):
        want = (xv - 2.5) / math.sqrt(1.25)
        assert g == torch.tensor(want, dtype=F64).to(F32).item()
    # eps enters under the root: eps = 5/4 doubles the variance term
    got = O.layer_norm(x, 1, eps=1.25)[0].tolist()
    assert got[3] == torch.tensor(1.5 / math.sqrt(2.5), dtype=F64).to(F32).item()


def test_layer_norm_matches_mpmath_to_the_last_bit_but_ties():
    g = torch.Generator().manual_seed(11)
    x = torch.randn(6, 37, generator=g) * 3 + 1.5
    w, b = torch.randn(37, generator=g), torch.randn(37, generator=g)
    got = O.layer_norm(x, 1, w, b, eps=1e-5)
    for r in range(6):
        exact = mp_layer_norm_row(x[r].tolist(), w.tolist(), b.tolist(), 1e-5)
        for j, e in enumerate(exact):
            gv = got[r, j].item()
            ulp = abs(float(e)) * 2.0 ** -23
            assert abs(mpmath.mpf(gv) - e) <= mpmath.mpf(ulp) * mpmath.mpf("0.5001") + mpmath.mpf(1e-45), (r, j)


def test_layer_norm_invariants():
    g = torch.Generator().manual_seed(12)
    x = torch.randn(5, 64, generator=g, dtype=F32)
    y = O.layer_norm(x, 1, eps=0.0).double()
    assert y.mean(1).abs().max() < 1e-7 and (y.var(1, unbiased=False) - 1).abs().max() < 1e-6
    # scale / shift invariance for eps = 0 (powers of two keep the inputs exact)
    y2 = O.layer_norm(x * 4 + 8, 1, eps=0.0).double()
    assert (y2 - y).abs().max() < 2e-6
    ym = O.layer_norm(-x, 1, eps=0.0).double()
    assert (ym + y).abs().max() < 1e-7
    # weight and bias act after the normalisation
    w, b = torch.randn(64, generator=g), torch.randn(64, generator=g)
    yw = O.layer_norm(x, 1, w, b, eps=0.0).double()
    assert (yw - (y * w.double() + b.double())).abs().max() < 1e-6
    # a constant row has variance 0: the output is the bias whatever eps is (and NaN without eps: 0 * inf)
    c = torch.full((2, 16), 3.25)
    assert torch.equal(O.layer_norm(c, 1, None, torch.arange(16.0), eps=1e-5), torch.arange(16.0).expand(2, 16))
    assert O.layer_norm(c, 1, eps=0.0).isnan().all()
    # eps matters: unit-variance row with eps = 3 is scaled by 1/2
    row = torch.tensor([[1.0, -1.0, 1.0, -1.0]])
    assert O.layer_norm(row, 1, eps=3.0).tolist() == [[0.5, -0.5, 0.5, -0.5]]


def test_layer_norm_several_dims_views_and_half_types():
    g = torch.Generator().manual_seed(13)
    x = torch.randn(3, 4, 5, 6, generator=g)
    w, b = torch.randn(5, 6, generator=g), torch.randn(5, 6, generator=g)
    want = F.layer_norm(x.double(), (5, 6), w.double(), b.double(), 1e-5)
    assert (O.layer_norm(x, 2, w, b).double() - want).abs().max() < 1e-6
    # a transposed leading view and a strided weight address the same values
    xt = x.permute(1, 0, 2, 3)
    assert torch.equal(O.layer_norm(xt, 2, w, b), O.layer_norm(xt.contiguous(), 2, w, b))
    wide = torch.randn(5, 12, generator=g)
    assert torch.equal(O.layer_norm(x, 2, wide[:, ::2], b), O.layer_norm(x, 2, wide[:, ::2].contiguous(), b))
    # normalising over every dim: one row
    assert (O.layer_norm(x, 4).double() - F.layer_norm(x.double(), x.shape)).abs().max() < 1e-6
    for dt in (BF16, F16):
        xh, wh, bh = x.to(dt), w.to(dt), b.to(dt)
        want = F.layer_norm(xh.double(), (5, 6), wh.double(), bh.double(), 1e-5).to(dt)   # one rounding from binary64
        got = O.layer_norm(xh, 2, wh, bh)
        assert got.dtype == dt
        assert (got.double() - want.double()).abs().max() <= 2.0 ** (-7 if dt == BF16 else -10) * want.double().abs().max()
        assert (got != want).float().mean() < 0.01                    # the roundings agree except at rare ties


def test_layer_norm_agrees_with_the_aten_cpu_operator():
    g = torch.Generator().manual_seed(14)
    for shape, k in (((64, 1000), 1), ((7, 3, 129), 2), ((2, 8192), 1)):
        x = torch.randn(shape, generator=g) * 2 + 0.5
        w, b = torch.randn(shape[-k:], generator=g), torch.randn(shape[-k:], generator=g)
        want = F.layer_norm(x, shape[-k:], w, b, 1e-5)
        got = O.layer_norm(x, k, w, b, 1e-5)
        assert (got - want).abs().max() <= 4e-6 * (1 + want.abs().max())


def test_layer_norm_errors_and_empty():
    x = torch.zeros(3, 4)
    for args, kind in (((x, 0), "dim"), ((x, 3), "dim"), ((x, 1, torch.zeros(3)), "shape"),
                       ((x, 1, None, torch.zeros(4, 1)), "shape"), ((x.long(), 1), "dtype"),
                       ((x, 1, torch.zeros(4, dtype=torch.int32)), "dtype")):
        with pytest.raises(O.OracleError) as e:
            O.layer_norm(*args)
        assert e.value.kind == kind, args
    assert O.layer_norm(torch.zeros(0, 4), 1).shape == (0, 4)
    assert O.layer_norm(torch.zeros(3, 0), 1).shape == (3, 0)


# --------------------------------------------------------------------------- binary_cross_entropy
def test_bce_closed_forms_and_clamp():
    ln2 = math.log(2.0)
    x = torch.tensor([0.5, 0.5, 0.5, 1.0, 0.0, 0.0, 1.0, 0.25])
    t = torch.tensor([0.0, 1.0, 0.3, 1.0, 0.0, 1.0, 0.0, 1.0])
    got = O.binary_cross_entropy(x, t, reduction="none").tolist()
    want = [ln2, ln2, ln2, 0.0, 0.0, 100.0, 100.0, 2 * ln2]
    for g, w in zip(got, want):
        assert g == torch.tensor(w, dtype=F64).to(F32).item()
    # sum and mean are the sum and mean of those terms
    total = sum(want)
    assert O.binary_cross_entropy(x, t, reduction="sum").item() == torch.tensor(total, dtype=F64).to(F32).item()
    assert O.binary_cross_entropy(x, t, reduction="mean").item() == torch.tensor(total / 8, dtype=F64).to(F32).item()
    # a soft target at a clamped end: t = 0.25, x = 0 -> 0.25 * 100 + 0.75 * 0
    assert O.binary_cross_entropy(torch.tensor([0.0]), torch.tensor([0.25]), reduction="none").item() == 25.0


def test_bce_matches_mpmath_within_half_ulp_and_keeps_small_losses():
    mpmath.mp.dps = 50
    g = torch.Generator().manual_seed(21)
    x = torch.rand(300, generator=g).clamp_(1e-6, 1 - 1e-6)
    t = torch.rand(300, generator=g)
    x[:4] = torch.tensor([1e-30, 1e-10, 1 - 2.0 ** -24, 2.0 ** -149])
    t[:4] = torch.tensor([0.0, 0.0, 1.0, 0.0])
    got = O.binary_cross_entropy(x, t, reduction="none").tolist()
    for xv, tv, gv in zip(x.tolist(), t.tolist(), got):
        xm, tm = mpmath.mpf(xv), mpmath.mpf(tv)
        exact = -(tm * max(mpmath.log(xm), -100) + (1 - tm) * max(mpmath.log(1 - xm), -100))
        assert abs(mpmath.mpf(gv) - exact) <= abs(exact) * mpmath.mpf(2) ** -23 * mpmath.mpf("0.5001") + mpmath.mpf(1e-45)
    assert got[0] == pytest.approx(1e-30, rel=1e-6) and got[3] > 0.0         # ln(1 - x) keeps tiny x


def test_bce_symmetry_weight_and_broadcast():
    g = torch.Generator().manual_seed(22)
    x = (torch.randint(1, 255, (40, 6), generator=g).float() / 256)          # 1 - x is exact
    t = (torch.randint(0, 257, (40, 6), generator=g).float() / 256)
    a = O.binary_cross_entropy(x, t, reduction="none").double()
    b = O.binary_cross_entropy(1 - x, 1 - t, reduction="none").double()
    assert (a - b).abs().max() <= 1.3e-7 * a.abs().max()
    w = torch.rand(6, generator=g)
    aw = O.binary_cross_entropy(x, t, w, reduction="none").double()
    assert (aw - a * w.double()).abs().max() <= 1.3e-7 * aw.abs().max()
    col = torch.rand(40, 1, generator=g)
    assert torch.equal(O.binary_cross_entropy(x, t, col, "none"), O.binary_cross_entropy(x, t, col.expand(40, 6).contiguous(), "none"))
    # views address the same values
    xt = x.t()
    assert torch.equal(O.binary_cross_entropy(xt, t.t(), reduction="none"), O.binary_cross_entropy(x, t, reduction="none").t())
    s = O.binary_cross_entropy(x, t, w, reduction="sum").item()
    assert s == pytest.approx(aw.sum().item(), rel=1e-6)
    assert O.binary_cross_entropy(x, t, w, reduction="mean").item() == pytest.approx(aw.mean().item(), rel=1e-6)


def test_bce_nan_empty_and_errors():
    r = O.binary_cross_entropy(torch.tensor([NAN, 0.5]), torch.tensor([1.0, NAN]), reduction="none")
    assert r.isnan().all()
    assert math.isnan(O.binary_cross_entropy(torch.tensor([-0.5]), torch.tensor([1.0]), reduction="none").item())
    e0 = torch.zeros(0, 3)
    assert O.binary_cross_entropy(e0, e0, reduction="none").shape == (0, 3)
    assert O.binary_cross_entropy(e0, e0, reduction="sum").item() == 0.0
    assert math.isnan(O.binary_cross_entropy(e0, e0, reduction="mean").item())
    x = torch.full((3, 4), 0.5)
    for args, kind in (((x, torch.zeros(4, 3)), "shape"), ((x, torch.zeros(4)), "shape"), ((x, x, torch.zeros(2, 3, 4)), "shape"),
                       ((x, x, torch.zeros(3)), "shape"), ((x.long(), x.long()), "dtype"), ((x, x.to(BF16)), "dtype"),
                       ((x, x, None, "median"), "scalar")):
        with pytest.raises(O.OracleError) as e:
            O.binary_cross_entropy(*args)
        assert e.value.kind == kind, args


def test_bce_agrees_with_the_aten_cpu_operator():
    g = torch.Generator().manual_seed(23)
    x, t, w = torch.rand(200, 33, generator=g), torch.rand(200, 33, generator=g), torch.rand(33, generator=g)
    x[0, :3] = torch.tensor([0.0, 1.0, 0.5])
    t[0, :3] = torch.tensor([1.0, 0.0, 0.5])
    for red in ("none", "mean", "sum"):
        for ww in (None, w):
            want = F.binary_cross_entropy(x, t, ww, reduction=red)
            got = O.binary_cross_entropy(x, t, ww, red)
            assert (got - want).abs().max() <= 2e-6 * want.abs().max(), (red, ww is None)
    for dt in (BF16, F16):
        want = F.binary_cross_entropy(x.to(dt).double(), t.to(dt).double(), reduction="none").to(dt)
        got = O.binary_cross_entropy(x.to(dt), t.to(dt), reduction="none")
        assert got.dtype == dt and (got != want).float().mean() < 0.01
