"""GPU tests of the two failure reports the boundary makes on request: index validation (TX_ERR_INDEX before any data
kernel is launched) and the look-back status query.  No test here launches a data kernel with an out-of-range index:
with validation on the library returns before it would, and nothing is ever run on bad indices with validation off.
The give-up of a look-back wait is forced from the host (a poll limit of zero), so every kernel still ends normally."""
import pytest
import torch

from oracle import oracle as O
from paper_2512_10977_amd import binding as B
from paper_2512_10977_amd import inputs as I
from tests.parity import assert_exact

pytestmark = pytest.mark.gpu

F32, I32, I64 = torch.float32, torch.int32, torch.int64


@pytest.fixture
def validation():
    B.tx_set_index_validation(True)
    yield
    B.tx_set_index_validation(False)


def expect_index_error(call, out, oracle_call):
    """The oracle refuses the indices with an index error; the library must too, and must leave `out` alone."""
    with pytest.raises(O.OracleError) as oe:
        oracle_call()
    assert oe.value.kind == "index", oe.value.kind
    before = out.clone()
    with pytest.raises(B.TxError) as e:
        call()
    assert e.value.kind == "INDEX", str(e.value)
    torch.cuda.synchronize()
    assert torch.equal(out, before), "output written although the call returned TX_ERR_INDEX"
    return str(e.value)


def test_switch_is_off_by_default_and_per_thread():
    import threading
    assert B.tx_get_index_validation() is False
    B.tx_set_index_validation(True)
    seen = []
    t = threading.Thread(target=lambda: seen.append(B.tx_get_index_validation()))
    t.start()
    t.join()
    assert B.tx_get_index_validation() is True and seen == [False]
    B.tx_set_index_validation(False)


@pytest.mark.parametrize("idt", [I64, I32])
def test_gather_index_select_take(validation, idt):
    src = I.typed((50, 6, 64), F32, seed=901)
    dsrc = src.cuda()
    for bad in (50, -1, 2 ** 31 - 1 if idt == I32 else 2 ** 40):
        idx = I.uniform_indices(37, 50, seed=902).to(idt)
        idx[11] = bad
        out = torch.zeros((37, 6, 64), device="cuda")
        msg = expect_index_error(lambda: B.tx_index_select(out, dsrc, 0, idx.cuda()), out, lambda: O.index_select(src, 0, idx))
        assert str(bad) in msg and "[0, 50)" in msg, msg
        g = I.uniform_indices((5, 6, 64), 50, seed=903).to(idt)
        g[4, 5, 63] = bad
        out = torch.zeros((5, 6, 64), device="cuda")
        expect_index_error(lambda: B.tx_gather(out, dsrc, 0, g.cuda()), out, lambda: O.gather(src, 0, g))
    # a strided index view and the last position of each dim
    base = I.uniform_indices((37, 2), 50, seed=904).to(idt)
    base[36, 0] = 50
    view = base[:, 0]
    out = torch.zeros((37, 6, 64), device="cuda")
    expect_index_error(lambda: B.tx_index_select(out, dsrc, 0, base.cuda()[:, 0]), out, lambda: O.index_select(src, 0, view))
    # valid indices: results as without validation, equal to the oracle's
    idx = I.uniform_indices(37, 6, seed=905).to(idt)
    out = torch.empty((50, 37, 64), device="cuda")
    B.tx_index_select(out, dsrc, 1, idx.cuda())
    assert_exact(out, O.index_select(src, 1, idx), "index_select with validation on")
    # take wraps negative indices once: [-n, n) is valid, n and -n - 1 are not
    n = src.numel()
    t = torch.tensor([0, -1, n - 1, -n], dtype=idt)
    out = torch.empty((4,), device="cuda")
    B.tx_take(out, dsrc, t.cuda())
    assert_exact(out, O.take(src, t), "take with validation on")
    for bad in (n, -n - 1):
        t2 = t.clone()
        t2[2] = bad
        out = torch.zeros((4,), device="cuda")
        expect_index_error(lambda: B.tx_take(out, dsrc, t2.cuda()), out, lambda: O.take(src, t2))


def test_scatter_family(validation):
    rows = I.zipf_rows(4096, 128, 1.1, seed=910)
    src = I.normal((4096, 256), 1.0, seed=911)
    dst0 = I.normal((128, 256), 1.0, seed=912)
    dsrc = src.cuda()
    for bad in (128, -1):
        r = rows.clone()
        r[4095] = bad
        e_cpu = r.unsqueeze(1).expand(4096, 256)
        e = r.cuda().unsqueeze(1).expand(4096, 256)                 # broadcast row index: the sorted whole-row path
        d = dst0.cuda()
        ws = B.workspace(B.tx_scatter_add_workspace_bytes(d, 0, e, dsrc, True))
        expect_index_error(lambda: B.tx_scatter_add_(d, 0, e, dsrc, True, ws), d, lambda: O.scatter_add_(dst0.clone(), 0, e_cpu, src))
        m_cpu = e_cpu[:64].contiguous()                             # materialised index: element keys / atomics
        m_cpu[63, 255] = bad
        m = m_cpu.cuda()
        ws = B.workspace(B.tx_scatter_add_workspace_bytes(d, 0, m, dsrc[:64], True))
        expect_index_error(lambda: B.tx_scatter_add_(d, 0, m, dsrc[:64], True, ws), d,
                           lambda: O.scatter_add_(dst0.clone(), 0, m_cpu, src[:64]))
        di = torch.zeros((128, 256), dtype=I32, device="cuda")      # integer atomics, no workspace
        si = torch.ones((64, 256), dtype=I32)
        expect_index_error(lambda: B.tx_scatter_add_(di, 0, m, si.cuda(), True, None), di,
                           lambda: O.scatter_add_(torch.zeros((128, 256), dtype=I32), 0, m_cpu, si))
        ws = B.workspace(B.tx_scatter_reduce_workspace_bytes(d, 0, m, dsrc[:64], "amax", True))
        expect_index_error(lambda: B.tx_scatter_reduce_(d, 0, m, dsrc[:64], "amax", True, ws), d,
                           lambda: O.scatter_reduce_(dst0.clone(), 0, m_cpu, src[:64], "amax", True))
        ws = B.workspace(B.tx_index_add_workspace_bytes(d, 0, r.cuda(), dsrc, True))
        expect_index_error(lambda: B.tx_index_add_(d, 0, r.cuda(), dsrc, 1, True, ws), d,
                           lambda: O.index_add_(dst0.clone(), 0, r, src, 1))
    # valid indices with validation on: the usual result
    d = dst0.cuda()
    e = rows.cuda().unsqueeze(1).expand(4096, 256)
    ws = B.workspace(B.tx_scatter_add_workspace_bytes(d, 0, e, dsrc, True))
    B.tx_scatter_add_(d, 0, e, dsrc, True, ws)
    want = O.scatter_add_(dst0.clone(), 0, rows.unsqueeze(1).expand(4096, 256), src)
    torch.cuda.synchronize()
    assert (d.cpu() - want).abs().max() <= 1e-4 * want.abs().max()


def test_index_put_wraps_negative_and_refuses_beyond(validation):
    self0 = I.normal((20, 7, 5), 1.0, seed=920)
    vals = I.normal((6, 5), 1.0, seed=921)
    i0 = torch.tensor([0, -20, 19, 3, -1, 7])
    i1 = torch.tensor([6, -7, 0, 1, 2, 3])
    d = self0.cuda()
    B.tx_index_put_(d, [i0.cuda(), i1.cuda()], vals.cuda(), False, None)
    assert_exact(d, O.index_put_(self0.clone(), [i0, i1], vals, False), "index_put_ with validation on")
    for j, bad in ((0, 20), (0, -21), (1, 7), (1, -8)):
        idx = [i0.clone(), i1.clone()]
        idx[j][4] = bad
        d = self0.cuda()
        expect_index_error(lambda: B.tx_index_put_(d, [t.cuda() for t in idx], vals.cuda(), False, None), d,
                           lambda: O.index_put_(self0.clone(), idx, vals, False))


def test_lookback_status_reports_a_forced_give_up():
    x = I.cumsum_input((6, 200000), F32, seed=930)                   # long rows: the look-back kernel
    dx = x.cuda()
    out = torch.empty_like(dx)
    ws = B.workspace(B.tx_cumsum_workspace_bytes(out, dx, -1))
    B.tx_cumsum(out, dx, -1, ws)
    assert B.tx_last_path().startswith("scan-lookback")
    B.tx_lookback_status(ws)                                         # a normal run: nothing to report
    good = out.clone()
    # the host sets the poll limit to zero: every tile but the first of a row gives up at once, ends normally, and
    # leaves the flag set; the call itself has returned TX_OK
    B.tx_force_path("scan-lookback-giveup")
    try:
        B.tx_cumsum(out, dx, -1, ws)
        assert B.tx_last_path().startswith("scan-lookback")
    finally:
        B.tx_force_path(None)
    with pytest.raises(B.TxError) as e:
        B.tx_lookback_status(ws)
    assert e.value.kind == "LAUNCH" and "gave up" in str(e.value)
    assert not torch.equal(out, good)                                # which is why the caller has to be told
    B.tx_cumsum(out, dx, -1, ws)                                     # the next run clears the flag
    B.tx_lookback_status(ws)
    assert torch.equal(out[:, :1000], good[:, :1000])
    # a workspace whose last user was not a look-back path has no header tag: nothing to report
    y = I.cumsum_input((2048, 300), F32, seed=931).cuda()
    oy = torch.empty_like(y)
    ws2 = B.workspace(max(256, B.tx_cumsum_workspace_bytes(oy, y, -1)))
    ws2.fill_(0xff)
    B.tx_cumsum(oy, y, -1, ws2)
    assert not B.tx_last_path().startswith("scan-lookback")
    B.tx_lookback_status(ws2)
