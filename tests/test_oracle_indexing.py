"""Pins for the oracle's gather, index_select, scatter_add_ (and their error rules).

Identity indices, brute force in pure Python on tiny shapes, cross-relations
between the operators and permutation invariance; the definitions are those of
the operators in Table 1's "Indexing & Selection" category, which the paper
validates against the ATen CPU result (Section 3.2).  No expected value comes
from the oracle or from the HIP library.
"""
import itertools
import math

import pytest
import torch

from oracle import oracle as O
from paper_2512_10977_amd import inputs as I

F32, BF16, F16, I32, I64, B = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool


def test_gather_brute_force_all_dims():
    src = I.normal((4, 3, 5), 1.0, seed=70)
    for dim in range(3):
        shape = [3, 2, 4]
        idx = I.uniform_indices(tuple(shape), src.shape[dim], seed=71 + dim)
        out = O.gather(src, dim, idx)
        assert out.shape == tuple(shape)
        for i, j, k in itertools.product(range(3), range(2), range(4)):
            c = [i, j, k]
            c[dim] = idx[i, j, k].item()
            assert out[i, j, k].item() == src[tuple(c)].item()
    # int32 indices are accepted too
    idx = I.uniform_indices((4, 3, 5), 4, seed=74)
    assert torch.equal(O.gather(src, 0, idx.to(I32)), O.gather(src, 0, idx))


def test_gather_identity_and_relation_to_index_select():
    src = I.normal((6, 4), 1.0, seed=75)
    ident = torch.arange(6).unsqueeze(1).expand(6, 4).contiguous()
    assert torch.equal(O.gather(src, 0, ident), src)
    rows = I.uniform_indices(9, 6, seed=76)
    g = O.gather(src, 0, rows.unsqueeze(1).expand(9, 4))          # stride-0 index view, all columns equal
    assert torch.equal(g, O.index_select(src, 0, rows))
    assert O.gather(torch.tensor(2.5), 0, torch.tensor(0)).item() == 2.5
    assert O.gather(src, 0, torch.zeros((0, 4), dtype=I64)).shape == (0, 4)


def test_index_select_brute_force_dims_dtypes_views():
    for dt in (F32, BF16, I64, B):
        src = I.make_view((5, 4, 6), dt, "transposed", seed=77)
        for dim in (0, 1, 2, -1):
            d = dim % 3
            idx = I.uniform_indices(7, src.shape[d], seed=78)
            out = O.index_select(src, dim, idx)
            want = torch.stack([src.select(d, k) for k in idx.tolist()], d)
            assert torch.equal(out, want)
    src = I.normal((5, 3), 1.0, seed=79)
    assert torch.equal(O.index_select(src, 0, torch.arange(5)), src)
    assert torch.equal(O.index_select(src, 0, torch.tensor(2)), src[2:3])     # 0-dim index = length 1
    assert O.index_select(torch.tensor(1.5), 0, torch.tensor([0])).item() == 1.5
    assert O.index_select(src, 0, torch.zeros((0,), dtype=I64)).shape == (0, 3)


def test_scatter_add_brute_force_and_closed_forms():
    src = I.integers((6, 4), -1000, 1000, seed=80, dtype=I32)
    dst0 = I.integers((5, 4), -1000, 1000, seed=81, dtype=I32)
    idx = I.uniform_indices((6, 4), 5, seed=82)
    out = O.scatter_add_(dst0.clone(), 0, idx, src)
    want = dst0.clone().tolist()
    for i, j in itertools.product(range(6), range(4)):
        want[idx[i, j].item()][j] += src[i, j].item()
    assert out.tolist() == want
    # all-zero index: row 0 receives the column sums
    z = O.scatter_add_(torch.zeros((5, 4), dtype=I32), 0, torch.zeros((6, 4), dtype=I64), src)
    assert torch.equal(z[0].to(I64), O.reduce("sum", src, 0)) and int(z[1:].abs().sum()) == 0
    # identity index: self + src
    ident = torch.arange(5).unsqueeze(1).expand(5, 4)
    s = O.scatter_add_(dst0.clone(), 0, ident, src[:5])
    assert torch.equal(s, dst0 + src[:5])
    # along dim 1
    idx1 = I.uniform_indices((6, 3), 4, seed=83)
    d1 = O.scatter_add_(torch.zeros((6, 4), dtype=I32), 1, idx1, src)
    w = [[0] * 4 for _ in range(6)]
    for i, j in itertools.product(range(6), range(3)):
        w[i][idx1[i, j].item()] += src[i, j].item()
    assert d1.tolist() == w


def test_scatter_add_counts_and_permutation_invariance():
    n, rows = 400, 16
    r = I.zipf_rows(n, rows, 1.1, seed=84)
    idx = r.unsqueeze(1).expand(n, 3)                                   # expanded (stride-0) index view
    ones = torch.ones((n, 3), dtype=I32)
    cnt = O.scatter_add_(torch.zeros((rows, 3), dtype=I32), 0, idx, ones)
    assert cnt[:, 0].tolist() == torch.bincount(r, minlength=rows).tolist()
    src = I.integers((n, 3), -1000, 1000, seed=85, dtype=I32)
    a = O.scatter_add_(torch.zeros((rows, 3), dtype=I32), 0, idx, src)
    perm = torch.randperm(n, generator=torch.Generator().manual_seed(86))
    b = O.scatter_add_(torch.zeros((rows, 3), dtype=I32), 0, idx[perm].contiguous(), src[perm].contiguous())
    assert torch.equal(a, b)
    # wrap-around in int32
    big = torch.full((4, 1), 2 ** 30, dtype=I32)
    assert O.scatter_add_(torch.zeros((1, 1), dtype=I32), 0, torch.zeros((4, 1), dtype=I64), big).item() == 0


def test_scatter_add_float_is_one_rounding_of_the_exact_sum():
    n, rows = 300, 8
    r = I.zipf_rows(n, rows, 1.1, seed=87)
    src = I.normal((n, 2), 1.0, seed=88)
    dst0 = I.normal((rows, 2), 1.0, seed=89)
    out = O.scatter_add_(dst0.clone(), 0, r.unsqueeze(1).expand(n, 2), src)
    for k in range(rows):
        for j in range(2):
            terms = [dst0[k, j].item()] + [src[i, j].item() for i in range(n) if r[i].item() == k]
            want = math.fsum(terms)
            assert abs(out[k, j].item() - want) <= 2.0 ** -23 * abs(want) + 1e-12
    # rows that receive nothing keep their exact bits
    lone = O.scatter_add_(dst0.clone(), 0, torch.zeros((1, 2), dtype=I64), src[:1])
    assert torch.equal(lone[1:], dst0[1:])


def test_scatter_add_bool_is_or():
    out = O.scatter_add_(torch.tensor([False, False, True]), 0, torch.tensor([0, 0, 1]), torch.tensor([False, True, False]))
    assert out.tolist() == [True, False, True]


def test_indexing_error_rules():
    src = torch.zeros((4, 3))
    for bad in (-1, 4):
        with pytest.raises(O.OracleError) as e:
            O.gather(src, 0, torch.tensor([[bad, 0, 0]]))
        assert e.value.kind == "index"                                   # no negative wrap-around
        with pytest.raises(O.OracleError):
            O.index_select(src, 0, torch.tensor([bad]))
        with pytest.raises(O.OracleError):
            O.scatter_add_(torch.zeros((4, 3)), 0, torch.tensor([[bad, 0, 0]]), torch.ones((1, 3)))
    with pytest.raises(O.OracleError) as e:
        O.gather(src, 0, torch.zeros((2,), dtype=I64))                   # index.ndim != src.ndim
    assert e.value.kind == "shape"
    with pytest.raises(O.OracleError):
        O.gather(src, 0, torch.zeros((2, 4), dtype=I64))                 # index wider than src off-dim
    with pytest.raises(O.OracleError):
        O.index_select(src, 0, torch.zeros((2, 2), dtype=I64))           # index must be 1-D
    with pytest.raises(O.OracleError):
        O.index_select(src, 2, torch.zeros((2,), dtype=I64))
    with pytest.raises(O.OracleError) as e:
        O.scatter_add_(torch.zeros((4, 3)), 0, torch.zeros((1, 3), dtype=I64), torch.ones((1, 3), dtype=I32))
    assert e.value.kind == "dtype"
    with pytest.raises(O.OracleError):
        O.scatter_add_(torch.zeros((4, 3)), 0, torch.zeros((2, 3), dtype=I64), torch.ones((1, 3)))   # index > src
    with pytest.raises(O.OracleError):
        O.gather(src, 0, torch.zeros((1, 3), dtype=F32))                 # index dtype


def test_library_cross_check_tiny_shapes():
    # non-authoritative: torch CPU on tiny inputs (integer data, so order does not matter)
    src = I.integers((9, 5), -1000, 1000, seed=90)
    idx = I.uniform_indices((7, 5), 9, seed=91)
    assert torch.equal(O.gather(src, 0, idx), torch.gather(src, 0, idx))
    assert torch.equal(O.index_select(src, 1, idx[:, 0] % 5), torch.index_select(src, 1, idx[:, 0] % 5))
    dst = I.integers((9, 5), -1000, 1000, seed=92)
    assert torch.equal(O.scatter_add_(dst.clone(), 0, idx, src[:7]), dst.clone().scatter_add_(0, idx, src[:7]))
