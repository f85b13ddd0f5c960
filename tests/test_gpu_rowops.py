"""GPU parity: softmax / log_softmax and cumsum (HIP library through the C ABI) vs. the CPU oracle."""
import itertools

import pytest
import torch

from oracle import oracle as O
from paper_2512_10977_amd import binding as B
from paper_2512_10977_amd import inputs as I
from tests.parity import assert_exact, assert_rel, to_device_view

pytestmark = pytest.mark.gpu

F32, BF16, F16, I32, I64, BOOL = torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.int64, torch.bool
FLT_MIN = 1.1754943508222875e-38


def check_softmax(x_cpu, dim=-1, log=False, out_dtype=None, what=""):
    want = O.softmax(x_cpu, dim, log, out_dtype=out_dtype)
    x = to_device_view(x_cpu)
    out = torch.empty(want.shape, dtype=want.dtype, device="cuda")
    B.tx_softmax(out, x, dim, log)
    used = B.tx_last_path()
    torch.cuda.synchronize()
    what = "%s %s %s dim=%d %s [%s]" % ("log_softmax" if log else "softmax", x_cpu.dtype, tuple(x_cpu.shape), dim, what, used)
    rel = 1e-5 if want.dtype == F32 else 1e-2
    # softmax outputs are non-negative (no cancellation): the floor is the smallest normal of the output format
    floor = 6.2e-5 if want.dtype == F16 else FLT_MIN
    assert_rel(out, want, rel, 1.0 if log else floor, what)
    return used


def check_cumsum(x_cpu, dim=-1, out_dtype=None, what=""):
    want = O.cumsum(x_cpu, dim, out_dtype=out_dtype)
    x = to_device_view(x_cpu)
    out = torch.empty(want.shape, dtype=want.dtype, device="cuda")
    nbytes = B.tx_cumsum_workspace_bytes(out, x, dim)
    ws = B.workspace(nbytes) if nbytes else None
    B.tx_cumsum(out, x, dim, ws)
    used = B.tx_last_path()
    torch.cuda.synchronize()
    what = "cumsum %s %s dim=%d %s [%s]" % (x_cpu.dtype, tuple(x_cpu.shape), dim, what, used)
    if not want.dtype.is_floating_point:
        assert_exact(out, want, what)
    else:
        xd = x_cpu.double()
        xd = torch.where(xd.isfinite(), xd, torch.zeros_like(xd))
        scale = (xd * xd).cumsum(dim if x_cpu.dim() else 0).sqrt() if x_cpu.dim() else xd.abs()
        assert_rel(out, want, 1e-5 if want.dtype == F32 else 1e-2, scale, what)
    if ws is not None and (used.startswith("scan-lookback") or used.startswith("scan-cols-lookback")):
        B.tx_lookback_status(ws)                       # raises if a bounded look-back wait gave up
    return used


# --------------------------------------------------------------------------- softmax
@pytest.mark.parametrize("log", [False, True])
def test_softmax_shapes_and_paths(log):
    paths = set()
    for dt in (F32, BF16, F16):
        for shape in [(7, 13, 5), (33, 64), (33, 300), (9, 1000), (5, 4096), (3, 5000), (2, 70001), (1, 17), (40, 1)]:
            x = I.softmax_logits(shape, dt, seed=3)
            paths.add(check_softmax(x, -1, log))
        x = I.softmax_logits((6, 50, 7), dt, seed=301)
        for dim in (0, 1, 2, -3):
            paths.add(check_softmax(x, dim, log))
        paths.add(check_softmax(I.make_view((30, 257), dt, "transposed", seed=302), -1, log, what="transposed"))
        paths.add(check_softmax(I.make_view((30, 256), dt, "step2_outer", seed=303), -1, log, what="step2_outer"))
        paths.add(check_softmax(I.make_view((30, 256), dt, "step2_inner", seed=304), -1, log, what="step2_inner"))
    assert {"softmax-wave", "softmax-row", "softmax-wave-scalar", "softmax-block", "softmax-strided"} <= paths, paths
    check_softmax(I.softmax_logits((64, 512), BF16, seed=305), -1, log, out_dtype=F32, what="fp32 out")
    # both register-resident forms on every row length they share, ragged multiples of the vector width included,
    # and the workgroup form up to its longest rows (16 vectors per lane)
    for dt, shape in [(F32, (37, 260)), (F32, (9, 1028)), (F32, (5, 2048)), (F32, (3, 4096)), (BF16, (7, 520)), (BF16, (5, 8192)),
                      (F16, (6, 4104))]:
        x = I.softmax_logits(shape, dt, seed=306)
        for path in ("softmax-wave", "softmax-row"):
            B.tx_force_path(path)
            try:
                assert check_softmax(x, -1, log, what="forced " + path) == path
            finally:
                B.tx_force_path(None)
    for dt, shape in [(F32, (3, 4100)), (F32, (2, 16384)), (F32, (2, 12292)), (BF16, (2, 32768)), (BF16, (3, 9000))]:
        assert check_softmax(I.softmax_logits(shape, dt, seed=307), -1, log, what="long rows") == "softmax-row"
    assert check_softmax(I.softmax_logits((2, 16388), F32, seed=308), -1, log, what="beyond registers") == "softmax-block"


def test_softmax_special_rows_and_edges():
    inf, nan = float("inf"), float("nan")
    rows = torch.tensor([[0.0, -inf, 1.0, 2.0], [-inf, -inf, -inf, -inf], [0.0, inf, 1.0, 0.5], [0.0, nan, 1.0, 0.5],
                         [5.0, 5.0, 5.0, 5.0]])
    for log in (False, True):
        check_softmax(rows, -1, log, what="specials")
        check_softmax(rows.repeat(1, 300), -1, log, what="specials wide")
        check_softmax(rows.t().contiguous(), 0, log, what="specials dim0")
        check_softmax(torch.tensor(2.5), 0, log)
        check_softmax(torch.zeros((3, 0)), -1, log)
        check_softmax(torch.zeros((0, 3)), -1, log)
    d = lambda *s, dt=F32: torch.zeros(s, dtype=dt, device="cuda")
    with pytest.raises(B.TxError) as e:
        B.tx_softmax(d(2, 2, dt=I32), d(2, 2, dt=I32))
    assert e.value.kind == "DTYPE"
    with pytest.raises(B.TxError) as e:
        B.tx_softmax(d(2, 2), d(2, 2), 2)
    assert e.value.kind == "DIM"


@pytest.mark.parametrize("dt", [F32, BF16])
@pytest.mark.parametrize("log", [False, True])
def test_softmax_full_size(dt, log):
    x = I.softmax_logits((32768, 4096), dt, seed=3)
    assert check_softmax(x, -1, log) == "softmax-row"


# --------------------------------------------------------------------------- cumsum
def test_cumsum_shapes_and_paths():
    paths = set()
    for dt in (F32, BF16, F16, I32, I64, BOOL):
        for shape in [(7, 13, 5), (33, 64), (9, 1000), (5, 4096), (3, 5000), (2, 70001), (1, 17), (40, 1), (4100,),
                      (1, 300000)]:
            x = I.cumsum_input(shape, dt, seed=3) if dt != BOOL else I.booleans(shape, 0.5, seed=3)
            paths.add(check_cumsum(x, -1))
        x = I.cumsum_input((6, 50, 7), dt, seed=310) if dt != BOOL else I.booleans((6, 50, 7), 0.5, seed=310)
        for dim in (0, 1, 2, -3):
            paths.add(check_cumsum(x, dim))
        paths.add(check_cumsum(I.make_view((30, 257), dt, "transposed", seed=311, std=1.0), -1, what="transposed"))
        paths.add(check_cumsum(I.make_view((30, 2048), dt, "step2_outer", seed=312, std=1.0), -1, what="step2_outer"))
        paths.add(check_cumsum(I.make_view((30, 256), dt, "step2_inner", seed=313, std=1.0), -1, what="step2_inner"))
    assert {"scan-lookback", "scan-lookback-scalar", "scan-carry", "scan-carry-scalar", "scan-strided"} <= paths, paths
    check_cumsum(I.cumsum_input((16, 9000), BF16, seed=314), -1, out_dtype=F32, what="fp32 out")


def test_cumsum_both_row_kernels_agree_with_oracle():
    for dt in (F32, I64, BF16):
        x = I.cumsum_input((1500, 6000), dt, seed=317)      # many short rows: the dispatcher's row-carry case
        assert check_cumsum(x, -1).startswith("scan-carry")
        B.tx_force_path("scan-lookback")
        try:
            assert check_cumsum(x, -1).startswith("scan-lookback")
        finally:
            B.tx_force_path(None)
        y = I.cumsum_input((3, 50000), dt, seed=318)
        B.tx_force_path("scan-carry")
        try:
            assert check_cumsum(y, -1).startswith("scan-carry")
        finally:
            B.tx_force_path(None)


def test_cumsum_many_tiles_per_row_repeated():
    # long rows: many look-back hops; run several times with the same workspace to cover re-use
    for n, path in ((1 << 20, "scan-lookback"), ((1 << 22) + 12344, "scan-lookback-wide")):   # 16 KiB and 64 KiB tiles
        x_cpu = I.cumsum_input((3, n), I64, seed=315)
        want = O.cumsum(x_cpu, -1)
        x = x_cpu.cuda()
        out = torch.empty_like(x)
        ws = B.workspace(B.tx_cumsum_workspace_bytes(out, x, -1))
        for _ in range(5):
            out.zero_()
            B.tx_cumsum(out, x, -1, ws)
            torch.cuda.synchronize()
            assert B.tx_last_path() == path
            assert_exact(out, want, "cumsum int64 repeated")
            assert ws[4:8].view(torch.int32).item() == 0
    xf = I.cumsum_input((2, 1 << 21), F32, seed=316)
    assert check_cumsum(xf, -1) == "scan-lookback"
    xf = I.cumsum_input((5, (1 << 22) + 776), F32, seed=319)
    assert check_cumsum(xf, -1) == "scan-lookback-wide"
    B.tx_force_path("scan-lookback-narrow")
    try:
        assert check_cumsum(xf, -1) == "scan-lookback"
    finally:
        B.tx_force_path(None)
    xh = I.cumsum_input((2, (1 << 23) + 64), BF16, seed=320)     # half input, 8-element vectors
    assert check_cumsum(xh, -1) == "scan-lookback-wide"
    xs = I.cumsum_input((3, 3000001), F32, seed=321)             # rows not 16-byte aligned: scalar accesses
    assert check_cumsum(xs, -1) == "scan-lookback-wide-scalar"


def test_cumsum_edges_and_errors():
    inf = float("inf")
    check_cumsum(torch.tensor([1.0, inf, 2.0, -inf, 5.0]), 0)
    check_cumsum(torch.tensor(4.0), 0)
    check_cumsum(torch.zeros((0, 4)), 1)
    check_cumsum(torch.zeros((4, 0)), 1)
    check_cumsum(torch.tensor([2 ** 62, 2 ** 62, 2 ** 62]), 0)
    d = lambda *s, dt=F32: torch.zeros(s, dtype=dt, device="cuda")
    with pytest.raises(B.TxError) as e:
        B.tx_cumsum(d(4, dt=I32), d(4, dt=I32), 0)
    assert e.value.kind == "DTYPE"                     # integer input needs an int64 out
    with pytest.raises(B.TxError) as e:
        B.tx_cumsum(d(4, 4), d(4, 4), 2)
    assert e.value.kind == "DIM"
    with pytest.raises(B.TxError) as e:
        B.tx_cumsum(d(4, 4), d(4, 4), 1, ws=None)
    assert e.value.kind == "WORKSPACE"


@pytest.mark.parametrize("dt", [F32, I64])
def test_cumsum_full_size(dt):
    x = I.cumsum_input((4096, 65536), dt, seed=3)
    assert check_cumsum(x, -1) == "scan-lookback-wide"   # long rows: the single-pass look-back scan, 64 KiB tiles
    B.tx_force_path("scan-carry")                        # the same workload with one workgroup walking each row
    try:
        assert check_cumsum(x, -1) == "scan-carry"
    finally:
        B.tx_force_path(None)


# --------------------------------------------------------------------------- column forms (dim is not the innermost)
COL_SHAPES = [((1, 2, 16), 1), ((3, 65, 64), 1), ((2, 257, 100), 1), ((1000, 300), 0), ((64, 1028), 0), ((63, 17), 0),
              ((2, 3, 130, 8, 4), 2), ((5, 1, 40), 1), ((129, 2, 256), 0), ((4, 2100, 36), 1)]


@pytest.mark.parametrize("log", [False, True])
def test_softmax_column_form(log):
    for dt in (F32, BF16, F16):
        for shape, dim in COL_SHAPES:
            x = I.softmax_logits(shape, dt, seed=330 + len(shape))
            used = check_softmax(x, dim, log)
            L = shape[dim]
            # an operated dim of at most 128 stays in registers (one read); longer ones take the two-read kernel
            assert used.startswith("softmax-cols-reg" if 2 <= L <= 128 else "softmax-cols" if L >= 2 else "softmax-strided"), (shape, dim, used)
            if 2 <= L <= 128:
                B.tx_force_path("softmax-cols")
                try:
                    assert check_softmax(x, dim, log, what="two reads by name") == "softmax-cols"
                finally:
                    B.tx_force_path(None)
        for L in (2, 16, 17, 32, 33, 64, 65, 128, 129):                 # every workgroup size of the register form, and just past it
            x = I.softmax_logits((3, L, 132), dt, seed=334 + L)
            assert check_softmax(x, 1, log) == ("softmax-cols-reg" if L <= 128 else "softmax-cols"), L
        x = I.softmax_logits((6, 70, 48), dt, seed=331)
        assert check_softmax(x.transpose(0, 1), 1, log, what="outer stride") == "softmax-cols-reg"
        assert check_softmax(x[:, ::2], 1, log, what="strided L") == "softmax-cols-reg"
        assert check_softmax(x[..., 1:33], 1, log, what="offset columns") == "softmax-cols-reg-scalar"
        assert check_softmax(x[..., ::2], 1, log, what="strided inner") == "softmax-strided"
    check_softmax(I.softmax_logits((300, 512), BF16, seed=332), 0, log, out_dtype=F32, what="fp32 out")
    inf, nan = float("inf"), float("nan")
    cols = torch.tensor([[0.0, -inf, 1.0, 2.0], [-inf, -inf, -inf, -inf], [0.0, inf, 1.0, 0.5], [0.0, nan, 1.0, 0.5],
                         [5.0, 5.0, 5.0, 5.0], [-inf, 1.0, inf, nan]]).t().contiguous()        # one case per column
    assert check_softmax(cols.repeat(40, 8), 0, log, what="special columns") == "softmax-cols"
    assert check_softmax(cols.repeat(10, 8), 0, log, what="special columns, short") == "softmax-cols-reg"
    B.tx_force_path("softmax-strided")
    try:
        assert check_softmax(I.softmax_logits((40, 64), F32, seed=333), 0, log) == "softmax-strided"
    finally:
        B.tx_force_path(None)


def test_cumsum_column_form():
    for dt in (F32, BF16, F16, I32, I64, BOOL):
        for shape, dim in COL_SHAPES:
            x = I.cumsum_input(shape, dt, seed=340) if dt != BOOL else I.booleans(shape, 0.5, seed=340)
            used = check_cumsum(x, dim)
            assert used.startswith("scan-cols" if shape[dim] >= 2 else "scan-strided"), (shape, dim, used)
        x = I.cumsum_input((6, 70, 48), dt, seed=341) if dt != BOOL else I.booleans((6, 70, 48), 0.5, seed=341)
        assert check_cumsum(x.transpose(0, 1), 1, what="outer stride").startswith("scan-cols")
        assert check_cumsum(x[:, ::2], 1, what="strided L").startswith("scan-cols")
        assert check_cumsum(x[..., 1:33], 1, what="offset columns") == "scan-cols-lookback-scalar"
        assert check_cumsum(x[..., ::2], 1, what="strided inner") == "scan-strided"
    check_cumsum(I.cumsum_input((3000, 64), BF16, seed=342), 0, out_dtype=F32, what="fp32 out")
    # long columns on few strips: several tiles per column (the single pass with look-back between the tiles, and the
    # three-pass form by name, on every accumulator type and vector width) and the workspace check
    paths = set()
    for dt, shape in [(F32, (70000, 128)), (I64, (70000, 48)), (I32, (9000, 260)), (BOOL, (5000, 64)), (BF16, (4, 3000, 520)),
                      (F16, (2500, 33)), (F32, (2, 129, 4100))]:
        x = I.cumsum_input(shape, dt, seed=343) if dt != BOOL else I.booleans(shape, 0.5, seed=343)
        dim = len(shape) - 2
        paths.add(check_cumsum(x, dim, what="look-back"))
        B.tx_force_path("scan-cols-3pass")
        try:
            paths.add(check_cumsum(x, dim, what="three passes"))
        finally:
            B.tx_force_path(None)
    assert paths == {"scan-cols-lookback", "scan-cols-lookback-scalar", "scan-cols-3pass", "scan-cols-3pass-scalar"}, paths
    x = I.cumsum_input((70000, 128), F32, seed=343)
    dx, out = x.cuda(), torch.empty(x.shape, device="cuda")
    assert B.tx_cumsum_workspace_bytes(out, dx, 0) > 0
    with pytest.raises(B.TxError) as e:
        B.tx_cumsum(out, dx, 0, None)
    assert e.value.kind == "WORKSPACE"
    # a poll limit of zero (set by the host): every tile below the first gives up at once, ends normally and leaves the flag
    ws = B.workspace(B.tx_cumsum_workspace_bytes(out, dx, 0))
    B.tx_cumsum(out, dx, 0, ws)
    B.tx_lookback_status(ws)
    B.tx_force_path("scan-cols-lookback-giveup")
    try:
        B.tx_cumsum(out, dx, 0, ws)
        assert B.tx_last_path() == "scan-cols-lookback"
    finally:
        B.tx_force_path(None)
    with pytest.raises(B.TxError) as e:
        B.tx_lookback_status(ws)
    assert e.value.kind == "LAUNCH" and "gave up" in str(e.value)
    B.tx_cumsum(out, dx, 0, ws)                                      # the next run clears the flag
    B.tx_lookback_status(ws)


def test_cumsum_column_look_back_seeded_shapes():
    """Seeded random shapes on the look-back form (ragged last tiles in rows and columns, one to five outer slices, every
    accumulator type), each scanned three times: the association of the column sums depends on which tiles have
    published by the time a tile looks back, and must stay inside the tolerance every time (integers exactly)."""
    import random
    rnd = random.Random(360)
    seen = set()
    for case in range(24):
        outer = rnd.choice([1, 1, 2, 3, 5])
        L = rnd.choice([129, 200, 257, 1000, 4097, 9000])
        inner = rnd.choice([16, 33, 64, 100, 256, 260, 512, 1000])
        dt = rnd.choice([F32, I64, I32, BF16, BOOL])
        shape = (outer, L, inner) if outer > 1 else (L, inner)
        x = I.cumsum_input(shape, dt, seed=361 + case) if dt != BOOL else I.booleans(shape, 0.5, seed=361 + case)
        for rep in range(3):
            seen.add(check_cumsum(x, len(shape) - 2, what="case %d call %d" % (case, rep)))
    assert {"scan-cols-lookback", "scan-cols-lookback-scalar"} <= seen, seen


def test_softmax_short_column_full_size():
    x = I.softmax_logits((512, 128, 2048), F32, seed=351)             # softmax over 128 channels: rows stay in registers
    for log in (False, True):
        assert check_softmax(x, 1, log) == "softmax-cols-reg"
    assert check_softmax(I.softmax_logits((512, 128, 2048), BF16, seed=352), 1, False) == "softmax-cols-reg"


@pytest.mark.parametrize("shape,dim", [((4096, 32768), 0), ((64, 4096, 512), 1), ((65536, 2048), 0)])
def test_column_forms_full_size(shape, dim):
    x = I.softmax_logits(shape, F32, seed=350)
    assert check_softmax(x, dim, False) == "softmax-cols"
    assert check_cumsum(x, dim) == "scan-cols-lookback"
    B.tx_force_path("scan-cols-3pass")
    try:
        assert check_cumsum(x, dim) == "scan-cols-3pass"
    finally:
        B.tx_force_path(None)


# --------------------------------------------------------------------------- cumprod, logcumsumexp
def scan_input(op, shape, dt, seed):
    if op == "cumprod":
        return I.cumprod_input(shape, dt, seed=seed) if dt != BOOL else I.booleans(shape, 0.97, seed=seed)
    return I.typed(shape, dt, seed=seed, std=3.0)


def check_scan(op, x_cpu, dim=-1, out_dtype=None, what=""):
    want = O.scan(op, x_cpu, dim, out_dtype=out_dtype)
    x = to_device_view(x_cpu)
    out = torch.empty(want.shape, dtype=want.dtype, device="cuda")
    nbytes = B.tx_scan_workspace_bytes(op, out, x, dim)
    ws = B.workspace(nbytes) if nbytes else None
    B.tx_scan(op, out, x, dim, ws)
    used = B.tx_last_path()
    torch.cuda.synchronize()
    if ws is not None and used.startswith("scan-lookback"):
        B.tx_lookback_status(ws)                       # raises if a bounded look-back wait gave up
    what = "%s %s %s dim=%d %s [%s]" % (op, x_cpu.dtype, tuple(x_cpu.shape), dim, what, used)
    if not want.dtype.is_floating_point:
        assert_exact(out, want, what)
    elif op == "cumprod":                       # binary64 products, one rounding: no cancellation to allow for
        assert_rel(out, want, 1e-6 if want.dtype == F32 else 1e-2, FLT_MIN, what)
    else:                                       # a logarithm: absolute error of a few fp32 roundings of values of order |max|
        assert_rel(out, want, 1e-5 if want.dtype == F32 else 1e-2, 1.0, what)
    if ws is not None and used.startswith("scan-lookback"):
        B.tx_lookback_status(ws)                       # raises if a bounded look-back wait gave up
    return used


@pytest.mark.parametrize("op", ["cumprod", "logcumsumexp"])
def test_scan_shapes_and_paths(op):
    paths = set()
    dtypes = (F32, BF16, F16, I32, I64, BOOL) if op == "cumprod" else (F32, BF16, F16)
    for dt in dtypes:
        for shape in [(7, 13, 5), (33, 64), (9, 1000), (5, 4096), (3, 5000), (2, 70001), (1, 17), (40, 1), (2, 300000)]:
            paths.add(check_scan(op, scan_input(op, shape, dt, 330), -1))
        x = scan_input(op, (6, 50, 7), dt, 331)
        for dim in (0, 1, 2, -2):
            paths.add(check_scan(op, x, dim))
        paths.add(check_scan(op, scan_input(op, (257, 30), dt, 332).t(), -1, what="transposed"))
        paths.add(check_scan(op, scan_input(op, (30, 4096), dt, 333)[:, ::2], -1, what="step2_inner"))
        paths.add(check_scan(op, scan_input(op, (60, 2048), dt, 334)[::2], -1, what="step2_outer"))
    assert {"scan-carry", "scan-lookback", "scan-strided"} <= paths and any(p.endswith("-scalar") for p in paths), paths
    check_scan(op, scan_input(op, (16, 9000), BF16, 335), -1, out_dtype=F32, what="fp32 out")
    for dt in (F32, I64) if op == "cumprod" else (F32,):
        x = scan_input(op, (1500, 6000), dt, 336)            # many short rows: row-carry
        assert check_scan(op, x, -1).startswith("scan-carry")
        B.tx_force_path("scan-lookback")
        try:
            assert check_scan(op, x, -1).startswith("scan-lookback")
        finally:
            B.tx_force_path(None)
        assert check_scan(op, scan_input(op, (5, (1 << 22) + 776), dt, 337), -1) == "scan-lookback-wide"
        assert check_scan(op, scan_input(op, (3, 3000001), dt, 338), -1) == "scan-lookback-wide-scalar"


def test_scan_special_values_edges_and_errors():
    inf, nan = float("inf"), float("nan")
    check_scan("cumprod", torch.tensor([2.0, inf, 0.5, 0.0, 3.0]), 0)
    check_scan("cumprod", torch.tensor([2.0, nan, 0.5]), 0)
    check_scan("cumprod", torch.tensor([2 ** 31, 2 ** 31, 2, 3]), 0)                      # wraps to 0, stays 0
    check_scan("logcumsumexp", torch.tensor([-inf, -inf, 1.0, -inf, 2.0]), 0)
    check_scan("logcumsumexp", torch.tensor([0.0, inf, 1.0, -inf, inf]), 0)
    check_scan("logcumsumexp", torch.tensor([1.0, nan, 2.0, inf]), 0)
    check_scan("logcumsumexp", torch.tensor([1000.0, 999.0, -1000.0, 1001.0]), 0)
    x = I.typed((9, 5000), F32, seed=339, specials=0.001)                                  # a few NaN / inf inside long rows
    check_scan("logcumsumexp", x, -1, what="specials")
    for op in ("cumprod", "logcumsumexp"):
        check_scan(op, torch.tensor(4.0), 0)
        check_scan(op, torch.zeros((0, 4)), 1)
        check_scan(op, torch.zeros((4, 0)), 1)
    d = lambda *s, dt=F32: torch.zeros(s, dtype=dt, device="cuda")
    for args, kind in [(("logcumsumexp", d(4, dt=I64), d(4, dt=I64), 0), "DTYPE"), (("cumprod", d(4, dt=I32), d(4, dt=I32), 0), "DTYPE"),
                       (("cumprod", d(4, 4), d(4, 4), 2), "DIM"), (("cummax", d(4), d(4), 0), "SCALAR"),
                       (("cumprod", d(4, 5), d(4, 4), 1), "SHAPE")]:
        with pytest.raises(B.TxError) as e:
            B.tx_scan(*args)
        assert e.value.kind == kind, args
    with pytest.raises(B.TxError) as e:
        B.tx_scan("cumprod", d(4, 4), d(4, 4), 1, ws=None)
    assert e.value.kind == "WORKSPACE"
    # the sum through the same entry point is cumsum
    xs = I.cumsum_input((5, 3000), F32, seed=340)
    dx, o1, o2 = xs.cuda(), d(5, 3000), d(5, 3000)
    ws = B.workspace(B.tx_scan_workspace_bytes("cumsum", o1, dx, -1))
    B.tx_scan("cumsum", o1, dx, -1, ws)
    B.tx_cumsum(o2, dx, -1, ws)
    assert torch.equal(o1, o2)


@pytest.mark.parametrize("op,dt", [("cumprod", F32), ("logcumsumexp", F32), ("cumprod", I64), ("logcumsumexp", BF16)])
def test_scan_full_size(op, dt):
    x = scan_input(op, (4096, 65536), dt, 341)
    assert check_scan(op, x, -1) == "scan-lookback-wide"
