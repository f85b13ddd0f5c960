"""Pins for the oracle's scatter_reduce_ and index_put_.

The last two members of the paper's "Indexing & Selection" category (Table 1) that this library covers.  Expected
values: brute force over Python lists with exact integers / Fractions, hand-worked special cases (NaN, include_self,
floor division, negative indices, duplicates) and the ATen CPU operators (Section 3.2) - nothing comes from the oracle
or the HIP library.
"""
import math
from fractions import Fraction

import pytest
import torch

from oracle import oracle as O

F32, BF16, F16, I32, I64, B = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool
NAN, INF = float("nan"), float("inf")


def brute(self_rows, idx_rows, src_rows, reduce, include_self):
    """dim 0, 2-D, exact arithmetic on Python numbers."""
    out = [list(r) for r in self_rows]
    got = {}
    for i, row in enumerate(idx_rows):
        for c, k in enumerate(row):
            got.setdefault((k, c), []).append(src_rows[i][c])
    for (k, c), vals in got.items():
        vals = ([out[k][c]] if include_self else []) + vals
        if reduce == "sum":
            r = sum(vals)
        elif reduce == "prod":
            r = 1
            for v in vals:
                r *= v
        elif reduce == "mean":
            r = Fraction(sum(vals), len(vals)) if not isinstance(vals[0], int) else sum(vals) // len(vals)
        else:
            r = max(vals) if reduce == "amax" else min(vals)
        out[k][c] = r
    return out


@pytest.mark.parametrize("reduce", ["sum", "prod", "mean", "amax", "amin"])
@pytest.mark.parametrize("include_self", [True, False])
def test_scatter_reduce_integers_brute_force(reduce, include_self):
    g = torch.Generator().manual_seed(7)
    s = torch.randint(-9, 10, (6, 4), generator=g)
    src = torch.randint(-9, 10, (11, 4), generator=g)
    idx = torch.randint(0, 6, (11, 4), generator=g)
    want = brute(s.tolist(), idx.tolist(), src.tolist(), reduce, include_self)
    for dt in (I64, I32):
        assert O.scatter_reduce_(s.clone().to(dt), 0, idx, src.to(dt), reduce, include_self).tolist() == want, dt
    # int32 products wrap at 32 bits
    big = torch.tensor([[70000]], dtype=I32)
    assert O.scatter_reduce_(big.clone(), 0, torch.tensor([[0]]), big, "prod").item() == (70000 * 70000 + 2 ** 31) % 2 ** 32 - 2 ** 31


@pytest.mark.parametrize("reduce", ["sum", "prod", "mean", "amax", "amin"])
@pytest.mark.parametrize("include_self", [True, False])
def test_scatter_reduce_floats_round_once_from_exact_values(reduce, include_self):
    g = torch.Generator().manual_seed(8)
    s = (torch.randint(-40, 40, (5, 3), generator=g).float() / 8)
    src = (torch.randint(-40, 40, (9, 3), generator=g).float() / 8)
    idx = torch.randint(0, 5, (9, 3), generator=g)
    want = brute([[Fraction(v) for v in r] for r in s.tolist()], idx.tolist(), [[Fraction(v) for v in r] for r in src.tolist()],
                 reduce, include_self)
    got = O.scatter_reduce_(s.clone(), 0, idx, src, reduce, include_self)
    for r in range(5):
        for c in range(3):
            assert got[r, c].item() == torch.tensor(float(want[r][c]), dtype=torch.float64).float().item(), (r, c)


def test_scatter_reduce_special_cases_and_aten():
    # floor division for integer means: (-7 + 2) / 2 = -2.5 -> -3
    s = torch.tensor([0, 5])
    assert O.scatter_reduce_(s.clone(), 0, torch.tensor([0, 0]), torch.tensor([-7, 2]), "mean", False).tolist() == [-3, 5]
    assert O.scatter_reduce_(s.clone(), 0, torch.tensor([0, 0]), torch.tensor([-7, 2]), "mean", True).tolist() == [-2, 5]   # -5 // 3
    # NaN wins amax / amin; an untouched element keeps its bits; include_self = False drops the old value
    f = torch.tensor([1.0, -0.0, 9.0])
    r = O.scatter_reduce_(f.clone(), 0, torch.tensor([0, 0, 2]), torch.tensor([NAN, 5.0, 3.0]), "amax")
    assert math.isnan(r[0].item()) and math.copysign(1, r[1].item()) == -1 and r[2].item() == 9.0
    assert O.scatter_reduce_(f.clone(), 0, torch.tensor([2]), torch.tensor([3.0]), "amax", False).tolist()[2] == 3.0
    assert math.isnan(O.scatter_reduce_(torch.tensor([NAN]), 0, torch.tensor([0]), torch.tensor([1.0]), "amin", True).item())
    assert O.scatter_reduce_(torch.tensor([NAN]), 0, torch.tensor([0]), torch.tensor([1.0]), "amin", False).item() == 1.0
    # other dims, views, half types: the ATen CPU operator on exact inputs
    g = torch.Generator().manual_seed(9)
    s, src = torch.randn(4, 6, 5, generator=g), torch.randn(4, 9, 5, generator=g)
    idx = torch.randint(0, 6, (4, 9, 5), generator=g)
    for reduce in ("sum", "prod", "mean", "amax", "amin"):
        for inc in (True, False):
            want = s.double().scatter_reduce_(1, idx, src.double(), reduce, include_self=inc).float()
            got = O.scatter_reduce_(s.clone(), 1, idx, src, reduce, inc)
            assert (got.double() - want.double()).abs().max() <= 1.2e-7 * want.abs().max(), (reduce, inc)
            got_t = O.scatter_reduce_(s.permute(2, 0, 1).contiguous().permute(1, 2, 0), 1, idx, src, reduce, inc)
            assert torch.equal(got_t, got)
    for dt in (BF16, F16):
        want = s.to(dt).double().scatter_reduce_(1, idx, src.to(dt).double(), "amax", include_self=True).to(dt)
        assert torch.equal(O.scatter_reduce_(s.to(dt), 1, idx, src.to(dt), "amax"), want)
    sb, srcb = s > 0.3, src > 0.3                                             # bool: OR / AND
    for reduce in ("sum", "prod", "amax", "amin"):
        for inc in (True, False):
            assert torch.equal(O.scatter_reduce_(sb.clone(), 1, idx, srcb, reduce, inc),
                               sb.clone().scatter_reduce_(1, idx, srcb, reduce, include_self=inc)), (reduce, inc)
    assert O.scatter_reduce_(torch.tensor([False, True]), 0, torch.tensor([0, 0, 1]), torch.tensor([True, True, False]), "sum").tolist() == [True, True]
    assert O.scatter_reduce_(torch.tensor([True, True]), 0, torch.tensor([0, 0, 1]), torch.tensor([True, False, True]), "prod").tolist() == [False, True]
    for args, kind in (((s, 1, idx, src, "median"), "scalar"), ((s.bool(), 1, idx, src.bool(), "mean"), "dtype"),
                       ((s, 1, idx + 6, src, "sum"), "index"), ((s, 3, idx, src, "sum"), "dim"),
                       ((s, 1, idx, src[:, :8], "sum"), "shape"), ((s, 1, idx.float(), src, "sum"), "dtype")):
        with pytest.raises(O.OracleError) as e:
            O.scatter_reduce_(args[0].clone(), *args[1:])
        assert e.value.kind == kind, args[4]


# --------------------------------------------------------------------------- index_put_
def test_index_put_brute_force_accumulate_and_assign():
    g = torch.Generator().manual_seed(10)
    s = torch.randint(-50, 50, (4, 5, 3), generator=g)
    i0, i1 = torch.tensor([0, 3, 0, -1, 0]), torch.tensor([1, -1, 1, 4, -4])      # positions 0, 2 and 4 name (0, 1); 1 and 3 name (3, 4)
    v = torch.randint(-50, 50, (5, 3), generator=g)
    want = s.tolist()
    for p in range(5):
        a, b = i0[p].item() % 4, i1[p].item() % 5
        want[a][b] = [x + y for x, y in zip(want[a][b], v[p].tolist())]
    assert O.index_put_(s.clone(), [i0, i1], v, True).tolist() == want
    want = s.tolist()
    for p in range(5):                                                       # assignment: the last position wins here
        want[i0[p].item() % 4][i1[p].item() % 5] = v[p].tolist()
    assert O.index_put_(s.clone(), [i0, i1], v, False).tolist() == want
    # one index tensor (rows), all dims indexed (single elements), broadcast values, broadcast indices
    assert torch.equal(O.index_put_(s.clone(), [torch.tensor([2, 0])], v[:2].unsqueeze(1).expand(2, 5, 3), False),
                       s.clone().index_put_((torch.tensor([2, 0]),), v[:2].unsqueeze(1).expand(2, 5, 3)))
    i2 = torch.tensor([2, 0, 1, 1, 2])
    assert torch.equal(O.index_put_(s.clone(), [i0, i1, i2], v[:, 0], True), s.clone().index_put_((i0, i1, i2), v[:, 0], accumulate=True))
    assert torch.equal(O.index_put_(s.clone(), [i0, i1], torch.tensor(7), True), s.clone().index_put_((i0, i1), torch.tensor(7), accumulate=True))
    col, row = torch.tensor([[0], [3]]), torch.tensor([[1, 2, 4]])
    vv = torch.randint(-9, 9, (2, 3, 3), generator=g)
    assert torch.equal(O.index_put_(s.clone(), [col, row], vv, False), s.clone().index_put_((col, row), vv))


def test_index_put_floats_views_and_errors():
    # contributions that vanish one at a time in fp32 survive the binary64 accumulation
    s = torch.tensor([1.0, 0.0])
    got = O.index_put_(s.clone(), [torch.tensor([0, 0, 0, 1])], torch.tensor([1e8, 3.0, -1e8, 2.0 ** -30]), True)
    assert got.tolist() == [4.0, 2.0 ** -30]
    g = torch.Generator().manual_seed(11)
    s, v = torch.randn(6, 4, 5, generator=g), torch.randn(7, 5, generator=g)
    i0, i1 = torch.randint(-6, 6, (7,), generator=g), torch.randint(-4, 4, (7,), generator=g)
    want = s.double().index_put_((i0, i1), v.double(), accumulate=True).float()
    assert torch.equal(O.index_put_(s.clone(), [i0, i1], v, True), want)
    st = s.permute(2, 0, 1).contiguous().permute(1, 2, 0)
    assert torch.equal(O.index_put_(st, [i0.to(I32), i1], v, True), want)
    for dt in (BF16, F16, B):
        sd, vd = (s > 0, v > 0) if dt == B else (s.to(dt), v.to(dt))
        want = (sd.clone().index_put_((i0, i1), vd, accumulate=True) if dt == B
                else sd.double().index_put_((i0, i1), vd.double(), accumulate=True).to(dt))
        assert torch.equal(O.index_put_(sd.clone(), [i0, i1], vd, True), want), dt
    for args, kind in (((s, [i0 + 20, i1], v), "index"), ((s, [i0, i1], v[:, :4]), "shape"), ((s, [i0, i1[:5]], v), "shape"),
                       ((s, [i0.float(), i1], v), "dtype"), ((s, [i0, i1], v.double().to(BF16)), "dtype"), ((s, [], v), "dim"),
                       ((s, [i0, i1, i0, i1], v), "dim")):
        with pytest.raises(O.OracleError) as e:
            O.index_put_(args[0].clone(), args[1], args[2], True)
        assert e.value.kind == kind, kind
