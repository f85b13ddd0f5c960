"""CPU-side checks of the HIP library: it loads, exports every declared entry point, and its
host-only inference helpers agree with the oracle's (no kernel is launched here)."""
import itertools
import os
import re

import pytest
import torch

from oracle import oracle as O
from paper_2512_10977_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DT = [torch.bool, torch.int32, torch.int64, torch.float16, torch.bfloat16, torch.float32]


def declared_functions():
    text = open(os.path.join(ROOT, "include", "txops.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tx_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 20
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names           # the binding covers exactly the header


def test_strerror_and_status_names():
    lib = B.lib()
    assert lib.tx_strerror(0) == b"ok"
    for code in range(-12, 0):
        assert lib.tx_strerror(code) not in (b"ok", b"unknown status")
    assert lib.tx_strerror(-99) == b"unknown status"


@pytest.mark.parametrize("op", ["add", "mul", "div", "maximum", "eq"])
def test_infer_binary_matches_oracle(op):
    for da, db in itertools.product(DT, DT):
        for sa, sb in [((3,), (3,)), ((3,), ()), ((), (3,)), ((), ()), ((4, 1), (1, 5)), ((0, 3), (3,))]:
            a, b = torch.zeros(sa, dtype=da), torch.zeros(sb, dtype=db)
            assert B.tx_infer_binary(op, a, b) == O.infer_binary(op, a, b), (da, db, sa, sb)
    with pytest.raises(B.TxError) as e:
        B.tx_infer_binary(op, torch.zeros(3, 2), torch.zeros(3))
    assert e.value.kind == "SHAPE"


def test_infer_unary_where_reduce_match_oracle():
    for op, dt in itertools.product(B.UNARY, DT):
        try:
            want = O.unary_result_dtype(op, dt)
        except O.OracleError:
            with pytest.raises(B.TxError) as e:
                B.tx_infer_unary_dtype(op, dt)
            assert e.value.kind == "DTYPE"
            continue
        assert B.tx_infer_unary_dtype(op, dt) == want
    for da, db in itertools.product(DT, DT):
        for sa, sb in [((3,), (3,)), ((3,), ()), ((), (3,))]:
            x, y = torch.zeros(sa, dtype=da), torch.zeros(sb, dtype=db)
            assert B.tx_infer_where(x, y) == O.where_result_dtype(x, y)
    x = torch.zeros((2, 3, 4))
    for op, dims, keep in itertools.product(B.REDUCE, [None, 0, -1, (0, 2), (2, 0)], [False, True]):
        for dt in DT:
            xx = x.to(dt)
            try:
                want = O.infer_reduce(op, xx, dims, keep)
            except O.OracleError as err:
                with pytest.raises(B.TxError) as e:
                    B.tx_infer_reduce(op, xx, dims, keep)
                assert e.value.kind.lower() == err.kind
                continue
            assert B.tx_infer_reduce(op, xx, dims, keep) == want, (op, dims, keep, dt)
    for bad in ((0, 0), 3, -4):
        with pytest.raises(B.TxError) as e:
            B.tx_infer_reduce("sum", x, bad)
        assert e.value.kind == "DIM"


def test_host_validation_needs_no_gpu():
    # every semantic check happens before any launch, so these fail the same way without a device
    z = lambda *s, dt=torch.float32: torch.zeros(s, dtype=dt)
    null_stream = B.ctypes.c_void_p(0)
    with pytest.raises(B.TxError) as e:
        B.tx_add(z(3, 3), z(3, 2), z(3), stream=null_stream)
    assert e.value.kind == "SHAPE"
    with pytest.raises(B.TxError) as e:
        B.tx_add(z(3, dt=torch.int32), z(3, dt=torch.int32), z(3, dt=torch.int32), 0.5, stream=null_stream)
    assert e.value.kind == "SCALAR"
    with pytest.raises(B.TxError) as e:
        B.tx_add(z(1).expand(3), z(3), z(3), stream=null_stream)
    assert e.value.kind == "OVERLAP"
    buf = z(10)
    with pytest.raises(B.TxError) as e:
        B.tx_add(buf[1:9], buf[0:8], buf[0:8], stream=null_stream)
    assert e.value.kind == "OVERLAP"
    with pytest.raises(B.TxError) as e:
        B.tx_unary("abs", z(3, dt=torch.bool), z(3, dt=torch.bool), stream=null_stream)
    assert e.value.kind == "DTYPE"
    with pytest.raises(B.TxError) as e:
        B.tx_reduce("amax", z(3), z(3, 0), 1, stream=null_stream)
    assert e.value.kind == "EMPTY_REDUCTION"
    with pytest.raises(B.TxError) as e:
        B.tx_softmax(z(2, 2), z(2, 2), 5, stream=null_stream)
    assert e.value.kind == "DIM"
    with pytest.raises(B.TxError) as e:
        B.tx_cumsum(z(4, dt=torch.int32), z(4, dt=torch.int32), 0, stream=null_stream)
    assert e.value.kind == "DTYPE"
    with pytest.raises(B.TxError) as e:
        B.tx_gather(z(2), z(4, 3), 0, z(2, dt=torch.int64), stream=null_stream)
    assert e.value.kind == "SHAPE"
    with pytest.raises(B.TxError) as e:
        B.tx_scatter_add_(z(4, 3), 0, z(1, 3, dt=torch.int64), z(1, 3, dt=torch.int32), stream=null_stream)
    assert e.value.kind == "DTYPE"
    # empty outputs return OK without touching a device
    B.tx_add(z(0, 3), z(0, 3), z(3), stream=null_stream)
    B.tx_unary("exp", z(0), z(0), stream=null_stream)
    assert B.tx_last_path() == ""


def test_workspace_queries_are_host_only():
    x = torch.zeros((4, 65536))
    out = torch.zeros((4, 65536))
    assert B.tx_cumsum_workspace_bytes(out, x, -1) == 256 + 4 * 16 * 8          # 16 tiles of 4096 per row
    xi = torch.zeros((4, 65536), dtype=torch.int64)
    oi = torch.zeros((4, 65536), dtype=torch.int64)
    assert B.tx_cumsum_workspace_bytes(oi, xi, -1) == 256 + 4 * 32 * 32         # 32 tiles of 2048, 4 words each
    assert B.tx_cumsum_workspace_bytes(out.t(), x.t(), 0) > 0                   # still rows after merging? (strided rows)
    # columns cut into tiles: the query covers both forms, so a path forced by name never finds the workspace short.
    # [4096, 512] over dim 0: 2 strips of 256 columns, 32 look-back tiles of 128 rows each (one 8-byte status word per
    # column and tile, after the 256-byte header), against 64 tile sums per column for the three-pass form
    xc, oc = torch.zeros((4096, 512)), torch.zeros((4096, 512))
    look = 256 + 2 * 32 * 256 * 8
    three = 64 * 512 * 4
    assert B.tx_cumsum_workspace_bytes(oc, xc, 0) == max(look, three)
    # int64 accumulators: 128-column strips, four status words per column and tile
    xl, ol = torch.zeros((4096, 512), dtype=torch.int32), torch.zeros((4096, 512), dtype=torch.int64)
    assert B.tx_cumsum_workspace_bytes(ol, xl, 0) == max(256 + 4 * 32 * 128 * 32, 64 * 512 * 8)
    # enough strips to fill the chip: every workgroup walks its whole column, no workspace
    assert B.tx_cumsum_workspace_bytes(torch.zeros((64, 1 << 20)), torch.zeros((64, 1 << 20)), 0) == 0
    big = torch.zeros((1 << 22,))
    assert B.tx_reduce_workspace_bytes("sum", torch.zeros(()), big, None) > 0
    assert B.tx_reduce_workspace_bytes("sum", torch.zeros((4096,)), torch.zeros((4096, 1024)), 1) == 0
    idx = torch.zeros((100, 1), dtype=torch.int64).expand(100, 64)
    assert B.tx_scatter_add_workspace_bytes(torch.zeros((8, 64)), 0, idx, torch.zeros((100, 64)), True) > 0
    assert B.tx_scatter_add_workspace_bytes(torch.zeros((8, 64)), 0, idx, torch.zeros((100, 64)), False) == 0


def test_later_entry_points_infer_and_validate_on_the_host():
    z = lambda *s, dt=torch.float32: torch.zeros(s, dtype=dt)
    null_stream = B.ctypes.c_void_p(0)
    for op, dt in itertools.product(B.UNARY_PARAM, DT):
        try:
            want = O.unary_param(op, torch.zeros(2, dtype=dt), 1.0, 1.0, 1.0).dtype
        except O.OracleError as err:
            with pytest.raises(B.TxError) as e:
                B.tx_infer_unary_param_dtype(op, dt)
            assert e.value.kind.lower() == err.kind, (op, dt)
            continue
        assert B.tx_infer_unary_param_dtype(op, dt) == want, (op, dt)
    for op in B.TERNARY:
        for da, db, dc in itertools.product(DT, DT, DT):
            a, b, c = z(3, dt=da), z(3, dt=db), z(3, dt=dc) + 1
            try:
                want = O.ternary(op, a, b, c).dtype
            except O.OracleError as err:
                with pytest.raises(B.TxError) as e:
                    B.tx_infer_ternary_dtype(op, a, b, c)
                assert e.value.kind.lower() == err.kind, (op, da, db, dc)
                continue
            assert B.tx_infer_ternary_dtype(op, a, b, c) == want, (op, da, db, dc)
    for call, kind in [(lambda: B.tx_unary_param("celu", z(3), z(3), 0.0, stream=null_stream), "SCALAR"),
                       (lambda: B.tx_unary_param("round_decimals", z(3), z(3), 0.5, stream=null_stream), "SCALAR"),
                       (lambda: B.tx_ternary("lerp", z(3), z(3), z(3, dt=torch.bfloat16), None, 0.5, stream=null_stream), "DTYPE"),
                       (lambda: B.tx_ternary("addcmul", z(3), z(3), z(4), z(3), stream=null_stream), "SHAPE"),
                       (lambda: B.tx_scan("logcumsumexp", z(4, dt=torch.int64), z(4, dt=torch.int64), 0, stream=null_stream), "DTYPE"),
                       (lambda: B.tx_scan("cummax", z(4), z(4), 0, stream=null_stream), "SCALAR"),
                       (lambda: B.tx_copy(z(3), z(4, 3), stream=null_stream), "SHAPE"),
                       (lambda: B.tx_flip(z(2, 3), z(2, 3), [0, 0], stream=null_stream), "DIM"),
                       (lambda: B.tx_roll(z(2, 3), z(2, 3), [1], [2], stream=null_stream), "DIM"),
                       (lambda: B.tx_tri(z(5), z(5), 0, False, stream=null_stream), "NDIM"),
                       (lambda: B.tx_loss("huber", z(), z(3), z(3), "mean", 0.0, None, stream=null_stream), "SCALAR"),
                       (lambda: B.tx_loss("mse", z(), z(3), z(3), "mean", 1.0, None, stream=null_stream), "WORKSPACE"),
                       (lambda: B.tx_reduce("norm", z(), z(0), None, False, float("inf"), stream=null_stream), "EMPTY_REDUCTION"),
                       (lambda: B.tx_reduce("nanmean", z(dt=torch.int64), z(3, dt=torch.int64), None, stream=null_stream), "DTYPE")]:
        with pytest.raises(B.TxError) as e:
            call()
        assert e.value.kind == kind, kind
    buf = z(12)
    with pytest.raises(B.TxError) as e:
        B.tx_copy(buf[1:9], buf[0:8], stream=null_stream)                     # a shifted alias
    assert e.value.kind == "OVERLAP"
    B.tx_copy(z(0, 3), z(3), stream=null_stream)                              # nothing to do: no device needed
    B.tx_flip(z(0, 3), z(0, 3), [0], stream=null_stream)
    assert B.tx_scan_workspace_bytes("cumprod", z(4, 65536), z(4, 65536), -1) == 256 + 4 * 16 * 32     # binary64 accumulators: 4 words per tile
    assert B.tx_scan_workspace_bytes("cumsum", z(4, 65536), z(4, 65536), -1) == B.tx_cumsum_workspace_bytes(z(4, 65536), z(4, 65536), -1)
    assert B.tx_loss_workspace_bytes("mse", z(), z(64, 64), z(64, 64), "none", 1.0) == 0
    assert B.tx_loss_workspace_bytes("mse", z(), z(64, 64), z(64), "sum", 1.0) > B.tx_loss_workspace_bytes("mse", z(), z(64, 64), z(64, 64), "sum", 1.0)


def test_index_validation_switch_follows_the_environment():
    """The switch's initial state comes from TX_VALIDATE_INDICES (host logic only: no device call is made)."""
    import subprocess
    import sys
    code = ("import sys; sys.path.insert(0, %r); from paper_2512_10977_amd import binding as B; "
            "a = B.tx_get_index_validation(); B.tx_set_index_validation(not a); print(int(a), int(B.tx_get_index_validation()))" % ROOT)
    for value, want in ((None, "0 1"), ("1", "1 0"), ("0", "0 1"), ("yes", "1 0"), ("", "0 1")):
        env = dict(os.environ)
        env.pop("TX_VALIDATE_INDICES", None)
        if value is not None:
            env["TX_VALIDATE_INDICES"] = value
        out = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, check=True).stdout
        assert out.strip() == want, (value, out)


def test_sorted_scatter_refuses_two_to_the_31_entries():
    """The sort-based paths decode positions with 32-bit magic-number divisions (dividends below 2^31): a larger index is
    refused on the host, by the workspace query (0 bytes) and by the call (before any launch; the descriptors here
    point at no real memory of that size)."""
    big = 1 << 31
    keep = []

    def fake(shape, strides, dtype):
        keep.append(torch.zeros(16, dtype=dtype))
        d = B.desc(keep[-1])
        d.data = len(keep) << 40                            # addresses 1 TiB apart, so that no operand overlaps another whatever
        d.ndim = len(shape)                                 # extent its descriptor claims (never dereferenced: every call is refused)
        for i, (n, s) in enumerate(zip(shape, strides)):
            d.sizes[i], d.strides[i] = n, s
        return d

    lib = B.lib()
    self_d = fake((4, 2), (2, 1), torch.float32)
    idx_d = fake((big, 2), (0, 0), torch.int64)              # 2^32 element keys
    src_d = fake((big, 2), (0, 0), torch.float32)
    assert lib.tx_scatter_add_workspace_bytes(self_d, 0, idx_d, src_d, 1) == 0
    ws = torch.zeros(1024, dtype=torch.uint8)
    rc = lib.tx_scatter_add_(self_d, 0, idx_d, src_d, 1, ws.data_ptr(), 1024, None)
    assert B.STATUS[rc] == "UNSUPPORTED", (rc, lib.tx_last_error())
    assert b"2^31" in lib.tx_last_error()
    rc = lib.tx_scatter_reduce_(self_d, 0, idx_d, src_d, B.SCATTER_REDUCE["amax"], 1, ws.data_ptr(), 1024, None)
    assert B.STATUS[rc] == "UNSUPPORTED", (rc, lib.tx_last_error())
    rows_d = fake((big, 2), (1, 0), torch.int64)             # row mode: 2^31 source rows
    assert lib.tx_scatter_add_workspace_bytes(self_d, 0, rows_d, src_d, 1) == 0
    rc = lib.tx_scatter_add_(self_d, 0, rows_d, src_d, 1, ws.data_ptr(), 1024, None)
    assert B.STATUS[rc] == "UNSUPPORTED", (rc, lib.tx_last_error())
    # rows of 4 GiB or more do not take the row path (a lane's byte offset inside a row is kept in 32 bits): the call
    # falls to element keys, whose own limit (2^32 destination elements) then refuses it
    wide = 1 << 30
    self_w = fake((4, wide), (wide, 1), torch.float32)
    idx_w = fake((8, wide), (1, 0), torch.int64)
    src_w = fake((8, wide), (wide, 1), torch.float32)
    assert lib.tx_scatter_add_workspace_bytes(self_w, 0, idx_w, src_w, 1) == 0
    rc = lib.tx_scatter_add_(self_w, 0, idx_w, src_w, 1, ws.data_ptr(), 1024, None)
    assert B.STATUS[rc] == "UNSUPPORTED", (rc, lib.tx_last_error())
