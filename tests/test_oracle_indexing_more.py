"""Pins for the oracle's index_add_, take, masked_select and nonzero.

Further members of the paper's "Indexing & Selection" category (Table 1); the
definitions are the ATen CPU operators' (Section 3.2).  Expected values are
brute force in plain Python on small cases, exact integer / rational arithmetic,
counting identities and the ATen CPU operators themselves - nothing comes from
the oracle or the HIP library.
"""
import itertools
import math
from fractions import Fraction

import pytest
import torch

from oracle import oracle as O

F32, BF16, F16, I32, I64, B = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool


# --------------------------------------------------------------------------- index_add_
def py_index_add(self_rows, index, src_rows, alpha):
    out = [list(r) for r in self_rows]
    for i, k in enumerate(index):
        for c, v in enumerate(src_rows[i]):
            out[k][c] += alpha * v
    return out


def test_index_add_brute_force_integers_and_wrapping():
    g = torch.Generator().manual_seed(1)
    for dt, bits in ((I32, 32), (I64, 64)):
        lo, hi = -2 ** (bits - 2), 2 ** (bits - 2)          # sums and multiples still wrap
        s = torch.randint(lo, hi, (5, 3), generator=g, dtype=I64).to(dt)
        src = torch.randint(lo, hi, (7, 3), generator=g, dtype=I64).to(dt)
        idx = torch.tensor([4, 0, 4, 4, 2, 0, 1])
        for alpha in (1, -3, 2 ** 31 + 7):
            want = py_index_add(s.tolist(), idx.tolist(), src.tolist(), alpha)
            wrap = lambda v: (v + 2 ** (bits - 1)) % 2 ** bits - 2 ** (bits - 1)
            got = O.index_add_(s.clone(), 0, idx, src, alpha).tolist()
            assert got == [[wrap(v) for v in r] for r in want], (dt, alpha)


def test_index_add_floats_round_once_from_the_exact_sum():
    # contributions that cancel or vanish in fp32 one at a time survive in the exact sum
    s = torch.tensor([[1.0], [0.0]])
    src = torch.tensor([[1e8], [3.0], [-1e8], [2.0 ** -30]])
    idx = torch.tensor([0, 0, 0, 1])
    got = O.index_add_(s.clone(), 0, idx, src)
    assert got.tolist() == [[4.0], [2.0 ** -30]]
    # alpha multiplies every contribution: exact rationals on a small case
    g = torch.Generator().manual_seed(2)
    s, src = torch.randn(4, 5, generator=g), torch.randn(9, 5, generator=g)
    idx = torch.tensor([3, 3, 0, 1, 3, 0, 0, 2, 3])
    got = O.index_add_(s.clone(), 0, idx, src, alpha=0.375)
    for r in range(4):
        for c in range(5):
            exact = Fraction(s[r, c].item()) + sum(Fraction(3, 8) * Fraction(src[i, c].item()) for i in range(9) if idx[i] == r)
            assert got[r, c].item() == torch.tensor(float(exact), dtype=torch.float64).to(F32).item()


def test_index_add_other_dims_views_and_aten():
    g = torch.Generator().manual_seed(3)
    s, src = torch.randn(4, 6, 5, generator=g), torch.randn(4, 9, 5, generator=g)
    idx = torch.randint(0, 6, (9,), generator=g)
    want = torch.index_add(s.double(), 1, idx, src.double(), alpha=-1.5).float()
    assert torch.equal(O.index_add_(s.clone(), 1, idx, src, alpha=-1.5), want)
    assert torch.equal(O.index_add_(s.clone(), -2, idx.to(I32), src, alpha=-1.5), want)
    st = s.permute(2, 0, 1).contiguous().permute(1, 2, 0)                       # same values, other strides
    assert torch.equal(O.index_add_(st.clone(memory_format=torch.preserve_format), 1, idx, src, alpha=-1.5), want)
    # rows no index names keep their bits (a NaN payload, a negative zero)
    s2 = torch.tensor([[-0.0, float("nan")], [1.0, 2.0]])
    got = O.index_add_(s2.clone(), 0, torch.tensor([1]), torch.tensor([[0.5, 0.5]]))
    assert math.copysign(1, got[0, 0].item()) == -1 and math.isnan(got[0, 1].item()) and got[1].tolist() == [1.5, 2.5]
    for dt in (BF16, F16):
        want = torch.index_add(s.to(dt).double(), 1, idx, src.to(dt).double()).to(dt)
        assert torch.equal(O.index_add_(s.to(dt), 1, idx, src.to(dt)), want)
    z = torch.tensor(2.0)
    assert O.index_add_(z.clone(), 0, torch.tensor([0]), torch.tensor(3.0), alpha=2).item() == 8.0


def test_index_add_bool_is_or_with_alpha():
    s = torch.tensor([[True, False, False], [False, False, False]])
    src = torch.tensor([[False, True, False], [True, True, False], [False, False, False]])
    idx = torch.tensor([1, 1, 0])
    assert O.index_add_(s.clone(), 0, idx, src).tolist() == [[True, False, False], [True, True, False]]
    assert O.index_add_(s.clone(), 0, idx, src, alpha=False).tolist() == s.tolist()
    assert torch.equal(O.index_add_(s.clone(), 0, idx, src, alpha=True), torch.index_add(s, 0, idx, src, alpha=True))


def test_gather_zero_dim_counts_as_one_dim():
    x = torch.tensor(7.5)
    assert O.gather(x, 0, torch.tensor([0])).tolist() == [7.5]
    assert O.gather(torch.tensor([1.0, 2.0]), 0, torch.tensor(1)).item() == 2.0
    assert torch.equal(O.gather(x, 0, torch.tensor([0])), torch.gather(x, 0, torch.tensor([0])))
    with pytest.raises(O.OracleError):
        O.gather(x, 0, torch.tensor([[0]]))


def test_index_add_errors():
    s, src, idx = torch.zeros(4, 3), torch.zeros(2, 3), torch.tensor([0, 3])
    for args, kind in (((s, 0, torch.tensor([0, 4]), src), "index"), ((s, 0, torch.tensor([-1, 0]), src), "index"),
                       ((s, 0, idx, torch.zeros(3, 3)), "shape"), ((s, 0, idx, torch.zeros(2, 4)), "shape"),
                       ((s, 2, idx, src), "dim"), ((s, 0, idx.float(), src), "dtype"), ((s, 0, idx, src.double().float().long()), "dtype"),
                       ((s, 0, idx.view(1, 2), src), "shape"),
                       ((s.long(), 0, idx, src.long(), 0.5), "scalar")):
        with pytest.raises(O.OracleError) as e:
            O.index_add_(args[0].clone(), *args[1:])
        assert e.value.kind == kind, args
    before = torch.arange(12.0).view(4, 3)
    t = before.clone()
    with pytest.raises(O.OracleError):
        O.index_add_(t, 0, torch.tensor([0, 7]), torch.ones(2, 3))
    assert torch.equal(t, before)                                                # nothing written on error


# --------------------------------------------------------------------------- take
def test_take_is_flat_indexing_in_logical_order():
    x = torch.arange(24).view(2, 3, 4)
    flat = x.flatten().tolist()
    idx = torch.tensor([[0, 23, -1], [-24, 5, 12]])
    assert O.take(x, idx).tolist() == [[flat[i] for i in r] for r in idx.tolist()]
    # a permuted view is flattened in ITS logical order, not in memory order
    xp = x.permute(2, 0, 1)
    flat_p = [xp[i, j, k].item() for i in range(4) for j in range(2) for k in range(3)]
    assert O.take(xp, idx).tolist() == [[flat_p[i] for i in r] for r in idx.tolist()]
    assert O.take(x[:, ::2], torch.tensor([3, 4, 7])).tolist() == [3, 8, 11]
    for dt in (F32, BF16, F16, I32, I64, B):
        src = (torch.arange(24) % 5).to(dt).view(4, 6)
        i = torch.tensor([23, 0, 7, -3], dtype=I32)
        assert torch.equal(O.take(src, i), torch.take(src, i.long()))
    nanbits = torch.tensor([0x7fc12345], dtype=I32).view(F32)
    assert O.take(nanbits, torch.tensor([0])).view(I32).item() == 0x7fc12345    # a copy: payload intact
    assert O.take(x, torch.zeros((0, 2), dtype=I64)).shape == (0, 2)
    assert O.take(torch.tensor(7), torch.tensor([0, -1])).tolist() == [7, 7]


def test_take_errors():
    x = torch.arange(6).view(2, 3)
    for args, kind in (((x, torch.tensor([6])), "index"), ((x, torch.tensor([-7])), "index"), ((x, torch.tensor([0.0])), "dtype"),
                       ((torch.zeros(0), torch.tensor([0])), "index")):
        with pytest.raises(O.OracleError) as e:
            O.take(*args)
        assert e.value.kind == kind, args
    with pytest.raises(O.OracleError) as e:
        O.take(x, torch.tensor([0]), out=torch.zeros(1, dtype=F32))
    assert e.value.kind == "dtype"


# --------------------------------------------------------------------------- masked_select / nonzero
def test_masked_select_brute_force_and_broadcast():
    g = torch.Generator().manual_seed(5)
    x = torch.randn(3, 4, 5, generator=g)
    m = torch.rand(3, 4, 5, generator=g) < 0.4
    want = [x[i, j, k].item() for i in range(3) for j in range(4) for k in range(5) if m[i, j, k]]
    assert O.masked_select(x, m).tolist() == want
    # broadcasting both ways
    mrow = torch.tensor([True, False, True, True, False])
    assert O.masked_select(x, mrow).tolist() == [x[i, j, k].item() for i in range(3) for j in range(4) for k in range(5) if mrow[k]]
    col = torch.randn(4, 1, generator=g)
    m2 = torch.rand(3, 4, 5, generator=g) < 0.5
    assert O.masked_select(col, m2).tolist() == [col[j, 0].item() for i in range(3) for j in range(4) for k in range(5) if m2[i, j, k]]
    # views, dtypes, counting identity, empty results
    assert torch.equal(O.masked_select(x.transpose(0, 2), m.transpose(0, 2)), torch.masked_select(x.transpose(0, 2), m.transpose(0, 2)))
    for dt in (F32, BF16, F16, I32, I64, B):
        v = (torch.arange(60) % 7).to(dt).view(3, 4, 5)
        r = O.masked_select(v, m)
        assert r.dtype == dt and r.numel() == int(m.sum()) and torch.equal(r, torch.masked_select(v, m))
    assert O.masked_select(x, torch.zeros(3, 4, 5, dtype=B)).numel() == 0
    assert O.masked_select(x, torch.ones((), dtype=B)).tolist() == x.flatten().tolist()
    assert O.masked_select(torch.zeros(0, 3), torch.ones(3, dtype=B)).numel() == 0
    with pytest.raises(O.OracleError) as e:
        O.masked_select(x, m.float())
    assert e.value.kind == "dtype"
    with pytest.raises(O.OracleError) as e:
        O.masked_select(x, torch.ones(3, 4, 4, dtype=B))
    assert e.value.kind == "shape"


def test_nonzero_brute_force_order_and_zero_tests():
    x = torch.tensor([[0.0, -0.0, 1.0], [float("nan"), 0.0, float("-inf")]])
    assert O.nonzero(x).tolist() == [[0, 2], [1, 0], [1, 2]]                    # -0.0 is zero, NaN is not
    g = torch.Generator().manual_seed(6)
    v = torch.randint(-1, 2, (3, 2, 4), generator=g)
    want = [[i, j, k] for i, j, k in itertools.product(range(3), range(2), range(4)) if v[i, j, k] != 0]
    assert O.nonzero(v).tolist() == want
    assert O.nonzero(v.permute(2, 0, 1)).tolist() == sorted([k, i, j] for i, j, k in want)   # logical order of the view
    for dt in (F32, BF16, F16, I32, I64, B):
        t = v.to(dt)
        r = O.nonzero(t)
        assert r.dtype == I64 and torch.equal(r, torch.nonzero(t))
        # the selected elements are exactly masked_select with (x != 0)
        assert torch.equal(t[tuple(r.t())], O.masked_select(t, t != 0))
    assert O.nonzero(torch.zeros(4, 5)).shape == (0, 2)
    assert O.nonzero(torch.tensor(3.0)).shape == (1, 0) and O.nonzero(torch.tensor(0.0)).shape == (0, 0)
    assert O.nonzero(torch.zeros(0, 3)).shape == (0, 2)
