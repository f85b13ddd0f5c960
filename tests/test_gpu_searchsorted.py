"""searchsorted / bucketize on the GPU against the oracle: exact integer outputs."""
import pytest
import torch

from oracle import oracle as O
from paper_2512_10977_amd import binding as B
from tests.parity import to_device_view

pytestmark = pytest.mark.gpu
F32, BF16, F16, I32, I64 = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64


def check(seq, vals, right=False, out_int32=False, out_view=None, what="", forced=None):
    want = O.searchsorted(seq, vals, right=right, out_int32=out_int32)
    out = torch.empty(vals.shape, dtype=I32 if out_int32 else I64, device="cuda") if out_view is None else out_view
    B.tx_force_path(forced)
    try:
        B.tx_searchsorted(out, to_device_view(seq), to_device_view(vals), right)
    finally:
        B.tx_force_path(None)
    torch.cuda.synchronize()
    tree = seq.dim() == 1 and seq.numel() >= 2048 and vals.numel() >= 65536 and forced is None
    assert B.tx_last_path() == (("searchsorted-tree" if tree else "searchsorted") if vals.numel() else "")
    assert torch.equal(out.cpu(), want), (what, seq.dtype, tuple(seq.shape), tuple(vals.shape), right)


@pytest.mark.parametrize("dt", [F32, BF16, F16, I32, I64])
def test_sweep(dt):
    g = torch.Generator().manual_seed(11)
    for n in (0, 1, 2, 5, 63, 64, 65, 1000, 4097):
        seq = (torch.randn((n,), generator=g) * 30).to(dt).sort().values
        for shape in ((), (1,), (7,), (3, 300), (2, 3, 129), (0, 4)):
            vals = (torch.randn(shape, generator=g) * 40).to(dt)
            for right in (False, True):
                check(seq, vals, right)
    # rows searched separately, int32 output, ragged tail of the 1024-value workgroup tile
    seq = (torch.randn((5, 7, 333), generator=g) * 30).to(dt).sort(dim=-1).values
    vals = (torch.randn((5, 7, 59), generator=g) * 40).to(dt)
    check(seq, vals, False, out_int32=True)
    check(seq, vals, True)
    # exact hits and runs of equal elements
    ties = torch.randint(-5, 5, (2000,), generator=g).to(dt).sort().values
    check(ties, torch.randint(-7, 7, (1025,), generator=g).to(dt), False)
    check(ties, torch.randint(-7, 7, (1025,), generator=g).to(dt), True)


def test_views_special_values_and_unsorted_input():
    g = torch.Generator().manual_seed(12)
    wide = torch.randn((4, 600), generator=g).sort(dim=-1).values
    vals = torch.randn((300, 4), generator=g)
    check(wide[:, ::3], vals.t(), what="strided sequence rows, transposed values")
    check(wide[1, 5:500:2], vals, what="1-D strided boundaries")
    out = torch.zeros((4, 600), dtype=I64, device="cuda")[:, ::2]
    check(wide, torch.randn((4, 300), generator=g), out_view=out, what="strided out")
    inf, nan = float("inf"), float("nan")
    seq = torch.tensor([-inf, -1.0, 0.0, 0.0, 2.0, inf, nan, nan])
    v = torch.tensor([-inf, -0.0, 0.0, inf, nan, 1e30, -1e30, 2.0])
    check(seq, v, False)
    check(seq, v, True)
    # unsorted input: both sides take the same bisection steps
    check(torch.randn((4, 600), generator=g), torch.randn((4, 77), generator=g), what="unsorted")


def test_errors():
    z = lambda shape, dt=F32: torch.zeros(shape, dtype=dt, device="cuda")
    with pytest.raises(B.TxError) as e:
        B.tx_searchsorted(z((3,), I64), z((5,)), z((3,), I32))
    assert e.value.kind == "DTYPE"
    with pytest.raises(B.TxError) as e:
        B.tx_searchsorted(z((3,), I64), z((5,), torch.bool), z((3,), torch.bool))
    assert e.value.kind == "DTYPE"
    with pytest.raises(B.TxError) as e:
        B.tx_searchsorted(z((3,), F32), z((5,)), z((3,)))
    assert e.value.kind == "DTYPE"
    with pytest.raises(B.TxError) as e:
        B.tx_searchsorted(z((3, 4), I64), z((2, 5)), z((3, 4)))
    assert e.value.kind == "SHAPE"
    with pytest.raises(B.TxError) as e:
        B.tx_searchsorted(z((4,), I64), z((5,)), z((3,)))
    assert e.value.kind == "SHAPE"
    with pytest.raises(B.TxError) as e:
        B.tx_searchsorted(z((3,), I64), z(()), z((3,)))
    assert e.value.kind == "NDIM"


def test_full_size_bucketize():
    g = torch.Generator().manual_seed(13)
    bounds = torch.randn((65536,), generator=g).sort().values
    vals = torch.randn((4096, 4096), generator=g)
    check(bounds, vals, False)
    check(bounds, vals, True, out_int32=True)
    check(bounds, vals[:512], False, forced="searchsorted")


@pytest.mark.parametrize("dt", [F32, BF16, F16, I32, I64])
def test_lds_tree_takes_the_same_steps(dt):
    """Lengths around the threshold and far from powers of two, ties, strided views, a ragged last tile, and unsorted
    input, where only identical bisection steps give identical answers."""
    g = torch.Generator().manual_seed(14)
    for n in (2047, 2048, 2049, 3000, 4095, 65537):
        seq = (torch.randn((n,), generator=g) * 30).to(dt).sort().values
        vals = (torch.randn((65536 + 777,), generator=g) * 35).to(dt)
        check(seq, vals, False)
        check(seq, vals, True)
    wide = (torch.randn((20000,), generator=g) * 30).to(dt)
    check(wide, (torch.randn((300, 250), generator=g) * 35).to(dt).t(), False, what="unsorted, transposed values")
    check(wide.sort().values[::2], (torch.randn((70000,), generator=g) * 35).to(dt), True, what="strided boundaries")
