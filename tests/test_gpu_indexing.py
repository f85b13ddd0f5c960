"""GPU parity: gather, index_select, scatter_add_ (HIP library through the C ABI) vs. the CPU oracle."""
import itertools

import pytest
import torch

from oracle import oracle as O
from paper_2512_10977_amd import binding as B
from paper_2512_10977_amd import inputs as I
from tests.parity import assert_exact, assert_rel, to_device_view

pytestmark = pytest.mark.gpu

F32, BF16, F16, I32, I64, BOOL = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool
ALL = [F32, BF16, F16, I32, I64, BOOL]


def check_gather(src_cpu, dim, idx_cpu, what=""):
    want = O.gather(src_cpu, dim, idx_cpu)
    out = torch.empty(want.shape, dtype=want.dtype, device="cuda")
    B.tx_gather(out, to_device_view(src_cpu), dim, to_device_view(idx_cpu))
    torch.cuda.synchronize()
    assert_exact(out, want, "gather %s %s dim=%d %s" % (src_cpu.dtype, tuple(idx_cpu.shape), dim, what))


def check_index_select(src_cpu, dim, idx_cpu, what=""):
    want = O.index_select(src_cpu, dim, idx_cpu)
    out = torch.empty(want.shape, dtype=want.dtype, device="cuda")
    B.tx_index_select(out, to_device_view(src_cpu), dim, to_device_view(idx_cpu))
    used = B.tx_last_path()
    torch.cuda.synchronize()
    assert_exact(out, want, "index_select %s %s dim=%d %s [%s]" % (src_cpu.dtype, tuple(src_cpu.shape), dim, what, used))
    return used


def scatter_scale(self_cpu, dim, idx_cpu, src_cpu):
    """sqrt of the sum of squares of everything that lands on each destination element (binary64)."""
    s2 = self_cpu.double() ** 2
    window = tuple(slice(0, n) for n in idx_cpu.shape)
    s2.scatter_add_(dim, idx_cpu.to(torch.int64).contiguous(), (src_cpu.double() ** 2)[window].contiguous())
    return s2.sqrt()


def check_scatter_add(self_cpu, dim, idx_cpu, src_cpu, deterministic=True, what=""):
    want = O.scatter_add_(self_cpu.clone(), dim, idx_cpu, src_cpu)
    dst = to_device_view(self_cpu).clone() if self_cpu.is_contiguous() else to_device_view(self_cpu)
    idx, src = to_device_view(idx_cpu), to_device_view(src_cpu)
    nbytes = B.tx_scatter_add_workspace_bytes(dst, dim, idx, src, deterministic)
    ws = B.workspace(nbytes) if nbytes else None
    B.tx_scatter_add_(dst, dim, idx, src, deterministic, ws)
    used = B.tx_last_path()
    torch.cuda.synchronize()
    what = "scatter_add %s self%s idx%s dim=%d %s [%s]" % (self_cpu.dtype, tuple(self_cpu.shape), tuple(idx_cpu.shape), dim, what, used)
    if not self_cpu.dtype.is_floating_point:
        assert_exact(dst, want, what)
    else:
        rel = 1e-5 if self_cpu.dtype == F32 else 1e-2
        assert_rel(dst, want, rel, scatter_scale(self_cpu, dim, idx_cpu, src_cpu), what)
        if deterministic:                                   # run again: bitwise identical
            dst2 = to_device_view(self_cpu).clone() if self_cpu.is_contiguous() else to_device_view(self_cpu)
            B.tx_scatter_add_(dst2, dim, idx, src, True, ws)
            torch.cuda.synchronize()
            assert_exact(dst2, dst.cpu(), what + " (run-to-run)")
    return used


# --------------------------------------------------------------------------- gather / index_select
def test_gather_sweep():
    for dt in ALL:
        src = I.make_view((9, 6, 11), dt, "contig", seed=401)
        for dim in (0, 1, 2, -1):
            idx = I.uniform_indices((5, 4, 7), src.shape[dim], seed=402)
            check_gather(src, dim, idx)
            check_gather(src, dim, idx.to(I32), "int32 index")
        check_gather(I.make_view((9, 6, 11), dt, "transposed", seed=403), 1, I.uniform_indices((9, 20, 11), 6, seed=404), "view")
    src = I.typed((1000, 64), F32, seed=405)
    check_gather(src, 0, I.uniform_indices((4096, 64), 1000, seed=406), "tall")
    rows = I.uniform_indices(300, 1000, seed=407)
    check_gather(src, 0, rows.unsqueeze(1).expand(300, 64), "expanded index")
    check_gather(torch.tensor(2.5), 0, torch.tensor(0))
    check_gather(src, 0, torch.zeros((0, 64), dtype=I64))


def test_index_select_sweep():
    paths = set()
    for dt in ALL:
        src = I.make_view((50, 6, 64), dt, "contig", seed=410)
        for dim in (0, 1, 2, -1):
            idx = I.uniform_indices(37, src.shape[dim], seed=411)
            paths.add(check_index_select(src, dim, idx))
            paths.add(check_index_select(src, dim, idx.to(I32), "int32 index"))
        paths.add(check_index_select(I.make_view((50, 6, 64), dt, "transposed", seed=412), 0, I.uniform_indices(9, 50, seed=413), "view"))
        paths.add(check_index_select(I.make_view((50, 64), dt, "step2_outer", seed=414), 0, I.uniform_indices(77, 50, seed=415), "step2_outer"))
    src = I.typed((5, 3), F32, seed=416)
    check_index_select(src, 0, torch.tensor(2))
    check_index_select(torch.tensor(1.5), 0, torch.tensor([0]))
    check_index_select(src, 0, torch.zeros((0,), dtype=I64))
    check_index_select(I.typed((3000, 256), F32, seed=417), 0, I.uniform_indices(10001, 3000, seed=418), "rows ragged")
    check_index_select(I.typed((3000, 1000), BF16, seed=419), 0, I.uniform_indices(501, 3000, seed=420), "wide rows")
    assert {"index-select-rows", "index-select-generic"} <= paths, paths


# --------------------------------------------------------------------------- scatter_add
def test_scatter_add_integer_atomics():
    for dt in (I32, I64, BOOL):
        n, rows, w = 5000, 64, 40
        r = I.zipf_rows(n, rows, 1.1, seed=430)
        src = I.typed((n, w), dt, seed=431)
        dst = I.typed((rows, w), dt, seed=432)
        check_scatter_add(dst, 0, r.unsqueeze(1).expand(n, w), src, what="expanded")
        full = I.zipf_rows(n * w, rows, 1.1, seed=433).reshape(n, w)
        check_scatter_add(dst, 0, full, src, what="materialised")
        check_scatter_add(dst, 0, full.to(I32), src, what="int32 index")
        idx1 = I.uniform_indices((rows, 17), w, seed=434)
        check_scatter_add(dst, 1, idx1, I.typed((rows, 17), dt, seed=435), what="dim 1")
    big = torch.full((4, 1), 2 ** 30, dtype=I32)
    check_scatter_add(torch.zeros((1, 1), dtype=I32), 0, torch.zeros((4, 1), dtype=I64), big, what="wrap")


@pytest.mark.parametrize("dt", [I32, I64])
def test_scatter_add_integer_rows_sorted(dt):
    # broadcast row index with at least 4096 rows: grouped by destination, whole-row sums, no atomics
    for n, rows, w in [(5000, 64, 256), (20000, 700, 64), (4100, 70000, 32), (9000, 4, 20), (4096, 3, 16)]:
        r = I.zipf_rows(n, rows, 1.1, seed=460)
        src = I.integers((n, w), -1000, 1000, seed=461, dtype=dt)
        dst = I.integers((rows, w), -1000, 1000, seed=462, dtype=dt)
        assert check_scatter_add(dst, 0, r.unsqueeze(1).expand(n, w), src, what="row mode").startswith("scatter-sort-rows")
    n, w = 9000, 64                                      # one destination for everything: a single run over all chunks
    src = I.integers((n, w), -1000, 1000, seed=463, dtype=dt)
    dst = I.integers((4, w), -1000, 1000, seed=464, dtype=dt)
    assert check_scatter_add(dst, 0, torch.full((n, 1), 2).expand(n, w), src, what="one run") == "scatter-sort-rows"
    big = torch.full((5000, 16), 2 ** 30 if dt == I32 else 2 ** 62, dtype=dt)      # wraps like two's complement
    assert check_scatter_add(torch.zeros((2, 16), dtype=dt), 0, torch.ones((5000, 1), dtype=I64).expand(5000, 16), big,
                             what="wrap") == "scatter-sort-rows"
    # without a workspace the same call falls back to one atomic per element
    r = I.zipf_rows(5000, 64, 1.1, seed=465)
    src = I.integers((5000, 32), -1000, 1000, seed=466, dtype=dt)
    want = O.scatter_add_(torch.zeros((64, 32), dtype=dt), 0, r.unsqueeze(1).expand(5000, 32), src)
    dst = torch.zeros((64, 32), dtype=dt, device="cuda")
    B.tx_scatter_add_(dst, 0, r.cuda().unsqueeze(1).expand(5000, 32), src.cuda(), True, None)
    assert B.tx_last_path() == "scatter-atomic"
    torch.cuda.synchronize()
    assert_exact(dst, want, "no workspace")


@pytest.mark.parametrize("dt", [F32, BF16, F16])
def test_scatter_add_float_deterministic(dt):
    paths = set()
    for n, rows, w in [(5000, 64, 256), (20000, 700, 64), (3000, 70000, 32), (129, 5, 20), (1, 3, 16)]:
        r = I.zipf_rows(n, rows, 1.1, seed=440)
        src = I.normal((n, w), 1.0, seed=441, dtype=dt)
        dst = I.normal((rows, w), 1.0, seed=442, dtype=dt)
        paths.add(check_scatter_add(dst, 0, r.unsqueeze(1).expand(n, w), src, what="row mode"))
    # one row id for everything: a single run cut across many chunks
    n, w = 9000, 64
    src = I.normal((n, w), 1.0, seed=443, dtype=dt)
    paths.add(check_scatter_add(I.normal((4, w), 1.0, seed=444, dtype=dt), 0, torch.full((n, 1), 2).expand(n, w), src, what="one run"))
    # element mode: materialised index, other dims, windows smaller than src
    full = I.zipf_rows(400 * 24, 16, 1.1, seed=445).reshape(400, 24)
    paths.add(check_scatter_add(I.normal((16, 24), 1.0, seed=446, dtype=dt), 0, full, I.normal((400, 24), 1.0, seed=447, dtype=dt), what="element mode"))
    idx1 = I.uniform_indices((30, 11), 8, seed=448)
    paths.add(check_scatter_add(I.normal((30, 8), 1.0, seed=449, dtype=dt), 1, idx1, I.normal((32, 12), 1.0, seed=450, dtype=dt), what="dim 1 window"))
    assert {"scatter-sort-rows", "scatter-sort-elem"} <= paths, paths
    # deterministic=0: fp32 uses float atomics (tolerance only); the half types keep the sorted fp32-accumulating path
    r = I.zipf_rows(2000, 16, 1.1, seed=451)
    used = check_scatter_add(I.normal((16, 8), 1.0, seed=452, dtype=dt), 0, r.unsqueeze(1).expand(2000, 8),
                             I.normal((2000, 8), 1.0, seed=453, dtype=dt), deterministic=False, what="deterministic=0")
    assert used == ("scatter-atomic" if dt == F32 else "scatter-sort-elem")


@pytest.mark.parametrize("dt", [F32, I32])
def test_scatter_add_rows_chunk_sizes(dt):
    # the sorted row path cuts its input into chunks of 64, 128 or 256 rows by input size: sizes on both sides of the
    # two thresholds, with hot destinations (runs over many chunks), cold ones (runs inside a chunk) and a ragged tail
    for n, rows, w in [(524288 - 3, 3000, 16), (524288 + 77, 3000, 16), (1048576 + 129, 40000, 16)]:
        r = I.zipf_rows(n, rows, 1.1, seed=470)
        if dt == F32:
            src, dst = I.normal((n, w), 1.0, seed=471), I.normal((rows, w), 1.0, seed=472)
        else:
            src, dst = I.integers((n, w), -1000, 1000, seed=471, dtype=dt), I.integers((rows, w), -1000, 1000, seed=472, dtype=dt)
        assert check_scatter_add(dst, 0, r.unsqueeze(1).expand(n, w), src, what="n=%d" % n) == "scatter-sort-rows"


def test_indexing_error_codes():
    d = lambda *s, dt=F32: torch.zeros(s, dtype=dt, device="cuda")
    with pytest.raises(B.TxError) as e:
        B.tx_gather(d(2), d(4, 3), 0, d(2, dt=I64))
    assert e.value.kind == "SHAPE"
    with pytest.raises(B.TxError) as e:
        B.tx_gather(d(2, 4), d(4, 3), 0, d(2, 4, dt=I64))
    assert e.value.kind == "SHAPE"
    with pytest.raises(B.TxError) as e:
        B.tx_gather(d(1, 3), d(4, 3), 0, d(1, 3))
    assert e.value.kind == "DTYPE"
    with pytest.raises(B.TxError) as e:
        B.tx_index_select(d(2, 2, 3), d(4, 3), 0, d(2, 2, dt=I64))
    assert e.value.kind == "SHAPE"
    with pytest.raises(B.TxError) as e:
        B.tx_index_select(d(4, 2), d(4, 3), 2, d(2, dt=I64))
    assert e.value.kind == "DIM"
    with pytest.raises(B.TxError) as e:
        B.tx_scatter_add_(d(4, 3), 0, d(1, 3, dt=I64), d(1, 3, dt=I32))
    assert e.value.kind == "DTYPE"
    with pytest.raises(B.TxError) as e:
        B.tx_scatter_add_(d(4, 3), 0, d(2, 3, dt=I64), d(1, 3))
    assert e.value.kind == "SHAPE"
    with pytest.raises(B.TxError) as e:
        B.tx_scatter_add_(d(64, 64), 0, d(100, 1, dt=I64).expand(100, 64), d(100, 64), True, None)
    assert e.value.kind == "WORKSPACE"


# --------------------------------------------------------------------------- full workload
@pytest.fixture(scope="module")
def big_src():
    return I.normal((1048576, 256), 1.0, seed=4)


def test_index_select_full_size(big_src):
    idx = I.uniform_indices(4194304, 1048576, seed=4)
    want = O.index_select(big_src, 0, idx)
    out = torch.empty(want.shape, dtype=F32, device="cuda")
    B.tx_index_select(out, big_src.cuda(), 0, idx.cuda())
    assert B.tx_last_path() == "index-select-rows"
    torch.cuda.synchronize()
    assert_exact(out, want, "index_select full")


def test_gather_full_size(big_src):
    idx = I.uniform_indices((16384, 256), 1048576, seed=5)
    check_gather(big_src, 0, idx, "full")


def test_scatter_add_full_size(big_src):
    r = I.zipf_rows(1048576, 65536, 1.1, seed=4)
    idx = r.unsqueeze(1).expand(1048576, 256)
    dst = I.normal((65536, 256), 1.0, seed=6)
    assert check_scatter_add(dst, 0, idx, big_src, what="fp32 full") == "scatter-sort-rows"
    src_i = I.integers((1048576, 256), -1000, 1000, seed=7, dtype=I32)
    dst_i = I.integers((65536, 256), -1000, 1000, seed=8, dtype=I32)
    assert check_scatter_add(dst_i, 0, idx, src_i, what="int32 full") == "scatter-sort-rows"
    B.tx_force_path("scatter-atomic")          # the same workload with one atomic per element
    try:
        assert check_scatter_add(dst_i, 0, idx, src_i, what="int32 full, plain atomics") == "scatter-atomic"
    finally:
        B.tx_force_path(None)
    # materialised index, one Zipf draw per element (general path)
    full = I.zipf_rows(131072 * 256, 65536, 1.1, seed=9).reshape(131072, 256)
    check_scatter_add(dst_i, 0, full, src_i[:131072], what="int32 materialised")
    # the same index with fp32 values: element keys, sorted, every run summed in position order; held to the
    # tolerance and to bitwise run-to-run equality (check_scatter_add runs it twice)
    assert check_scatter_add(dst, 0, full, big_src[:131072], what="fp32 materialised") == "scatter-sort-elem"


def test_masked_fill_full_size(big_src):
    m = I.bernoulli_mask((1048576, 256), 0.3, seed=4)
    want = O.masked_fill(big_src, m, -1.0)
    out = torch.empty(want.shape, dtype=F32, device="cuda")
    B.tx_masked_fill(out, big_src.cuda(), m.cuda(), -1.0)
    torch.cuda.synchronize()
    assert_exact(out, want, "masked_fill full")
