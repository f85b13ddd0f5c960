"""GPU test of tx_reduce_static, the entry point that allocates nothing: its output must equal tx_reduce's (same kernels,
partials in the library's built-in scratch instead of a caller workspace) on two calls in a row, the second on a smaller
input, and match the CPU oracle; a reduction whose partials do not fit the built-in scratch is refused before any launch.
"""
import pytest
import torch

from oracle import oracle as O
from paper_2512_10977_amd import binding as B
from paper_2512_10977_amd import inputs as I
from tests.parity import assert_exact, assert_rel

pytestmark = pytest.mark.gpu

F32, BF16, I64 = torch.float32, torch.bfloat16, torch.int64
LIMIT = 4 << 20


def both(op, x_cpu, dims, keepdim=False):
    """(tx_reduce_static result, tx_reduce result, oracle result, path) on the same input."""
    want = O.reduce(op, x_cpu, dims, keepdim)
    x = x_cpu.cuda()
    ref = torch.empty(want.shape, dtype=want.dtype, device="cuda")
    nbytes = B.tx_reduce_workspace_bytes(op, ref, x, dims, keepdim)
    B.tx_reduce(op, ref, x, dims, keepdim, 1.0, B.workspace(nbytes) if nbytes else None)
    path = B.tx_last_path()
    torch.cuda.synchronize()
    got = torch.full(want.shape, 7, dtype=want.dtype, device="cuda")
    # the allocator's running count of allocation requests: it only grows, whatever the garbage collector frees meanwhile
    # (bytes in use can drop inside the call when a collection releases tensors of earlier tests)
    requests = torch.cuda.memory_stats()["allocation.all.allocated"]
    B.tx_reduce_static(op, got, x, dims, keepdim, 1.0)
    assert B.tx_last_path() == path
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == requests        # nothing was allocated through torch by the call
    torch.cuda.synchronize()
    return got, ref, want, path, nbytes


def compare(op, x_cpu, got, ref, want, what):
    if want.dtype.is_floating_point:
        # same kernels in the same order: the two entry points agree bit for bit; the oracle to the reduction tolerance
        assert torch.equal(got.view(torch.int32 if got.dtype == F32 else torch.int16),
                           ref.view(torch.int32 if ref.dtype == F32 else torch.int16)), what
        scale = (x_cpu.double() ** 2).sum().sqrt() if want.dim() == 0 else 0.0
        assert_rel(got, want, 1e-5 if want.dtype == F32 else 1e-2, scale, what)
    else:
        assert_exact(got, ref.cpu(), what)
        assert_exact(got, want, what)


@pytest.mark.parametrize("op,dtype", [("sum", F32), ("sum", I64), ("argmax", F32), ("var", F32), ("sum", BF16)])
def test_two_calls_in_a_row_second_smaller(op, dtype):
    big = I.reduction_input((48, 1000, 173), dtype, seed=11)         # 8.3 M elements, ragged: split across workgroups
    small = I.reduction_input((5, 333, 41), dtype, seed=12)          # 68 k elements: fewer partials than the first call left
    got, ref, want, path, nbytes = both(op, big, None)
    assert path == "rows-split" and 0 < nbytes <= LIMIT, (path, nbytes)
    compare(op, big, got, ref, want, "%s %s big" % (op, dtype))
    got, ref, want, path, nbytes = both(op, small, None)
    compare(op, small, got, ref, want, "%s %s small after big" % (op, dtype))


def test_column_split_then_unsplit():
    x = I.reduction_input((40000, 96), F32, seed=13)                  # few columns, long reduced dim: cols-split
    got, ref, want, path, nbytes = both("sum", x, 0)
    assert path == "cols-split" and 0 < nbytes <= LIMIT, (path, nbytes)
    assert torch.equal(got.view(torch.int32), ref.view(torch.int32))
    assert_rel(got, want, 1e-5, (x.double() ** 2).sum(0).sqrt(), "cols-split")
    y = I.reduction_input((64, 3000), F32, seed=14)                   # no split: the scratch is not touched at all
    got, ref, want, path, nbytes = both("amax", y, -1, keepdim=True)
    assert nbytes == 0
    assert_exact(got, want, "amax rows")


def test_refuses_what_does_not_fit():
    x = torch.zeros((4096, 4096), device="cuda")
    out = torch.empty((4096,), device="cuda")
    need = B.tx_reduce_workspace_bytes("prod", out, x, 0)
    assert need > LIMIT, need                                        # 4096 columns x 256 slices x 8-byte partials
    out.fill_(3.0)
    with pytest.raises(B.TxError) as e:
        B.tx_reduce_static("prod", out, x, 0)
    assert e.value.kind == "WORKSPACE" and "tx_reduce_static" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == 3.0).all())                                   # nothing was launched
    B.tx_reduce("prod", out, x, 0, False, 1.0, B.workspace(need))     # the workspace form still serves it
    torch.cuda.synchronize()
    assert bool((out == 0.0).all())
