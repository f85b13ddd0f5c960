"""Pins for the oracle's searchsorted / bucketize (Table 1: one of the indexing operators).

Expected values: the counting definition on sorted sequences (how many elements lie below / at most the value), brute
force in Python, numpy.searchsorted, and the ATen CPU operator - nothing comes from the oracle or the HIP library.
"""
import numpy as np
import pytest
import torch

from oracle import oracle as O

F32, BF16, F16, I32, I64, B = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool


@pytest.mark.parametrize("dt", [F32, BF16, F16, I32, I64])
@pytest.mark.parametrize("right", [False, True])
def test_counting_definition_on_sorted_rows(dt, right):
    g = torch.Generator().manual_seed(3)
    for n in (0, 1, 2, 7, 64, 257):
        seq = torch.randint(-20, 20, (n,), generator=g).to(dt).sort().values          # many ties
        vals = torch.randint(-25, 25, (3, 41), generator=g).to(dt)
        got = O.searchsorted(seq, vals, right=right)
        assert got.dtype == I64 and got.shape == vals.shape
        for i in range(3):
            for j in range(41):
                v = vals[i, j].item()
                want = sum(1 for e in seq.tolist() if (e <= v if right else e < v))
                assert got[i, j].item() == want, (n, v)


def test_against_numpy_and_int32_output():
    rng = np.random.default_rng(4)
    seq = np.sort(rng.standard_normal(1000).astype(np.float32))
    vals = rng.standard_normal((17, 33)).astype(np.float32)
    vals[0, :5] = seq[[0, 10, 500, 998, 999]]                                   # exact hits
    for right in (False, True):
        want = np.searchsorted(seq, vals, side="right" if right else "left")
        got = O.searchsorted(torch.from_numpy(seq), torch.from_numpy(vals), right=right, out_int32=True)
        assert got.dtype == I32 and np.array_equal(got.numpy(), want)


def test_rows_are_searched_separately_and_views_are_honoured():
    g = torch.Generator().manual_seed(5)
    seq = torch.randn((4, 5, 30), generator=g).sort(dim=-1).values
    vals = torch.randn((4, 5, 9), generator=g)
    got = O.searchsorted(seq, vals)
    for a in range(4):
        for b in range(5):
            assert np.array_equal(got[a, b].numpy(), np.searchsorted(seq[a, b].numpy(), vals[a, b].numpy()))
    # strided sequence and values
    wide = torch.randn((60,), generator=g).sort().values
    v2 = torch.randn((8, 12), generator=g)
    assert torch.equal(O.searchsorted(wide[::2], v2.t()), torch.searchsorted(wide[::2].contiguous(), v2.t().contiguous()))


def test_special_values_and_errors():
    inf, nan = float("inf"), float("nan")
    seq = torch.tensor([-inf, -1.0, 0.0, 0.0, 2.0, inf], dtype=F32)
    vals = torch.tensor([-inf, -0.0, 0.0, inf, nan, 1e30, -1e30], dtype=F32)
    assert O.searchsorted(seq, vals).tolist() == [0, 2, 2, 5, 6, 5, 1]          # a NaN goes to the end
    assert O.searchsorted(seq, vals, right=True).tolist() == [1, 4, 4, 6, 6, 5, 1]
    assert O.searchsorted(torch.zeros((0,)), torch.tensor([1.0, 2.0])).tolist() == [0, 0]
    assert O.searchsorted(seq, torch.zeros((0, 3))).shape == (0, 3)
    with pytest.raises(O.OracleError):
        O.searchsorted(seq, torch.tensor([1, 2]))                               # dtypes differ
    with pytest.raises(O.OracleError):
        O.searchsorted(torch.tensor([False, True]), torch.tensor([True]))       # bool
    with pytest.raises(O.OracleError):
        O.searchsorted(torch.zeros((2, 3)), torch.zeros((3, 3)))                # leading dims differ
    with pytest.raises(O.OracleError):
        O.searchsorted(torch.zeros((2, 3)), torch.zeros((3,)))                  # ranks differ


@pytest.mark.parametrize("dt", [F32, BF16, F16, I32, I64])
def test_against_aten_cpu(dt):
    g = torch.Generator().manual_seed(6)
    seq = (torch.randn((6, 200), generator=g) * 50).to(dt).sort(dim=-1).values
    vals = (torch.randn((6, 77), generator=g) * 60).to(dt)
    for right in (False, True):
        assert torch.equal(O.searchsorted(seq, vals, right=right), torch.searchsorted(seq, vals, right=right))
        assert torch.equal(O.searchsorted(seq[0], vals, right=right), torch.bucketize(vals, seq[0], right=right))
        assert torch.equal(O.searchsorted(seq, vals, right=right, out_int32=True),
                           torch.searchsorted(seq, vals, right=right, out_int32=True))
