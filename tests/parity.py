"""Comparison helpers for the GPU parity tests (HIP library vs. CPU oracle).

Tolerance classes:
  exact     integer / bool / index outputs and pure copies: identical bits.
  exact_fp  fp add / mul / where / neg / abs / maximum / eq: identical bits,
            except that any NaN equals any NaN (hosts and GPUs produce
            different default NaN payloads).
  ulp       fp32 transcendentals: at most 2 units in the last place from the
            oracle's correctly rounded value, infinities equal, NaN to NaN;
            where the oracle's value is subnormal an absolute error of FLT_MIN
            is accepted (hardware may flush, and fp32-composed forms stop
            there).
  rel       |g - o| <= rel * max(|o|, scale): rel 1e-5 for fp32 reductions /
            softmax / cumsum / scatter_add, 1e-2 for fp16 / bf16 outputs.
            `scale` is the natural magnitude of the terms (e.g. sqrt(sum x^2))
            so that sums which cancel are judged against what they were made of.
"""
import torch

FLT_MIN = 1.1754943508222875e-38


def to_device_view(t, device="cuda"):
    """Copy t's whole storage to the device and rebuild the same strided view there."""
    if t.numel() == 0:
        return torch.empty(t.shape, dtype=t.dtype, device=device)
    flat = torch.empty(0, dtype=t.dtype).set_(t.untyped_storage())
    dflat = flat.to(device)
    return torch.as_strided(dflat, t.size(), t.stride(), t.storage_offset())


def empty_like_layout(t, dtype, device="cuda", layout="contig"):
    """An uninitialised device output of t's shape: row-major, or with t's own stride order."""
    if layout == "contig" or t.dim() < 2:
        return torch.empty(t.shape, dtype=dtype, device=device)
    # dims ordered like t's strides (what ATen allocates for a dense permuted input)
    order = sorted(range(t.dim()), key=lambda d: (-t.stride(d), d))
    shape = [t.size(d) for d in order]
    base = torch.empty(shape, dtype=dtype, device=device)
    inv = [0] * t.dim()
    for i, d in enumerate(order):
        inv[d] = i
    return base.permute(inv)


def _bits(t):
    t = t.contiguous()
    if t.dtype in (torch.float16, torch.bfloat16):
        return t.view(torch.int16)
    if t.dtype == torch.float32:
        return t.view(torch.int32)
    return t


def assert_exact(got, want, what=""):
    got = got.cpu()
    assert got.dtype == want.dtype and got.shape == want.shape, (what, got.dtype, want.dtype, got.shape, want.shape)
    bad = _bits(got) != _bits(want)
    if bad.any():
        idx = bad.nonzero()[0].tolist()
        raise AssertionError("%s: %d of %d differ, first at %s: got %r want %r" % (
            what, int(bad.sum()), bad.numel(), idx, got[tuple(idx)].item(), want[tuple(idx)].item()))


def assert_exact_fp(got, want, what=""):
    got = got.cpu()
    assert got.dtype == want.dtype and got.shape == want.shape, (what, got.dtype, want.dtype, got.shape, want.shape)
    if not got.dtype.is_floating_point:
        return assert_exact(got, want, what)
    both_nan = got.isnan() & want.isnan()
    bad = (_bits(got) != _bits(want)) & ~both_nan
    if bad.any():
        idx = bad.nonzero()[0].tolist()
        raise AssertionError("%s: %d of %d differ, first at %s: got %r want %r" % (
            what, int(bad.sum()), bad.numel(), idx, got[tuple(idx)].item(), want[tuple(idx)].item()))


def _ordered(t):
    """Monotone integer image of fp32 values (+0 and -0 coincide)."""
    i = t.contiguous().view(torch.int32).to(torch.int64)
    return torch.where(i >= 0, i, -(i & 0x7FFFFFFF))


def assert_ulp(got, want, max_ulp=2, what=""):
    got = got.cpu()
    assert got.dtype == torch.float32 and want.dtype == torch.float32 and got.shape == want.shape, what
    nan_ok = got.isnan() == want.isnan()
    fin = ~want.isnan() & ~got.isnan()
    inf_ok = torch.where(want.isinf() | got.isinf(), got == want, torch.ones_like(nan_ok))
    d = (_ordered(got) - _ordered(want)).abs()
    small = want.abs() < FLT_MIN
    ok_val = (d <= max_ulp) | (small & ((got.double() - want.double()).abs() <= FLT_MIN))
    ok = nan_ok & (~fin | (inf_ok & ok_val))
    if not ok.all():
        idx = (~ok).nonzero()[0].tolist()
        worst = int(d[fin & ~want.isinf() & ~got.isinf()].max()) if fin.any() else -1
        raise AssertionError("%s: %d of %d outside %d ulp (worst %d), first at %s: got %r want %r" % (
            what, int((~ok).sum()), ok.numel(), max_ulp, worst, idx, got[tuple(idx)].item(), want[tuple(idx)].item()))
    sel = d[fin & ~want.isinf() & ~got.isinf() & ~small]
    return int(sel.max()) if sel.numel() else 0


def assert_rel(got, want, rel, scale=0.0, what="", overflow_max=None):
    """|g-o| <= rel*max(|o|, scale); NaN to NaN; infinities equal (or, for half types, a value within 1 % of the
    format's maximum may be either inf or finite)."""
    got = got.cpu()
    assert got.dtype == want.dtype and got.shape == want.shape, (what, got.dtype, want.dtype, got.shape, want.shape)
    g, o = got.double(), want.double()
    if not torch.is_tensor(scale):
        scale = torch.full_like(o, float(scale))
    scale = scale.double().expand_as(o)
    nan_ok = g.isnan() == o.isnan()
    both_fin = g.isfinite() & o.isfinite()
    ok = torch.where(both_fin, (g - o).abs() <= rel * torch.maximum(o.abs(), scale), g == o)
    if overflow_max is not None:
        edge = (g.abs() >= 0.99 * overflow_max) & (o.abs() >= 0.99 * overflow_max) & (g.sign() == o.sign())
        ok = ok | edge
    ok = (ok | (g.isnan() & o.isnan())) & nan_ok
    if not ok.all():
        idx = (~ok).nonzero()[0].tolist()
        raise AssertionError("%s: %d of %d outside rel %g, first at %s: got %r want %r (scale %r)" % (
            what, int((~ok).sum()), ok.numel(), rel, idx, got[tuple(idx)].item(), want[tuple(idx)].item(),
            scale[tuple(idx)].item()))


HALF_MAX = {torch.float16: 65504.0, torch.bfloat16: 3.3895313892515355e38}
