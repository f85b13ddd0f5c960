"""Seeded synthetic inputs shared by the test suite, the smoke check and the benchmark.

Only data generation lives here: no operator arithmetic.  Everything is drawn on
the host from a torch.Generator with a stated seed, so the CPU oracle and the
HIP library see identical bits.  The shapes and distributions are those of the
five workloads this library is measured on; they stand in for the OpInfo samples
and production-captured inputs the paper tests with (Section 3.3), which are not
reproduced here.

Conventions: "N(0, s)" means standard deviation s.  Special-value injection
uses its own generator stream (seed + 1000) so the clean data are the same with
and without injection.
"""
import math

import torch

FLOAT_DTYPES = (torch.float32, torch.bfloat16, torch.float16)
INT_DTYPES = (torch.int32, torch.int64)
ALL_DTYPES = FLOAT_DTYPES + INT_DTYPES + (torch.bool,)


def _gen(seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def normal(shape, std=1.0, seed=0, dtype=torch.float32):
    """i.i.d. N(0, std) drawn in fp32, then rounded to `dtype`."""
    x = torch.randn(shape, generator=_gen(seed), dtype=torch.float32)
    if std != 1.0:
        x.mul_(std)
    return x.to(dtype)


def inject_specials(x, p=0.01, seed=0):
    """Independently with probability p replace an element by NaN, +inf or -inf (uniform choice)."""
    g = _gen(seed + 1000)
    hit = torch.rand(x.shape, generator=g) < p
    kind = torch.randint(0, 3, x.shape, generator=g)
    out = x.clone()
    out[hit & (kind == 0)] = float("nan")
    out[hit & (kind == 1)] = float("inf")
    out[hit & (kind == 2)] = float("-inf")
    return out


def inject_neg_inf(x, p=0.001, seed=0):
    """Independently with probability p set an element to -inf."""
    g = _gen(seed + 1000)
    hit = torch.rand(x.shape, generator=g) < p
    out = x.clone()
    out[hit] = float("-inf")
    return out


def integers(shape, lo=-1000, hi=1000, seed=0, dtype=torch.int64):
    """Uniform integers in [lo, hi] inclusive."""
    return torch.randint(lo, hi + 1, shape, generator=_gen(seed), dtype=torch.int64).to(dtype)


def booleans(shape, p=0.5, seed=0):
    return torch.rand(shape, generator=_gen(seed)) < p


def typed(shape, dtype, seed=0, std=3.0, specials=0.0):
    """The elementwise sweep's value recipe for one dtype."""
    if dtype == torch.bool:
        return booleans(shape, 0.5, seed)
    if dtype in INT_DTYPES:
        return integers(shape, -1000, 1000, seed, dtype)
    x = normal(shape, std, seed, torch.float32)
    if specials > 0:
        x = inject_specials(x, specials, seed)
    return x.to(dtype)


VIEW_KINDS = ("contig", "transposed", "step2_inner", "step2_outer", "expand_row", "expand_col")


def make_view(shape, dtype, kind, seed=0, std=3.0, specials=0.0):
    """A tensor of logical `shape` whose memory layout is of the given kind.

    contig       plain row-major
    transposed   the dims are stored in rotated order (2-D: base[n,m].t(); 3-D: permute(2,0,1) of a
                 base stored as [s2,s0,s1]... i.e. the last logical dim is the slowest in memory)
    step2_inner  every second element of a base twice as long in the last dim
    step2_outer  every second slice of a base twice as long in the first dim
    expand_row   a [s0,1,...] column broadcast along the remaining dims (stride 0 there)
    expand_col   a [1,...,s_last] row broadcast along the leading dims
    """
    shape = tuple(shape)
    nd = len(shape)
    if kind == "contig" or nd == 0:
        return typed(shape, dtype, seed, std, specials)
    if kind == "transposed":
        if nd == 1:
            return typed(shape, dtype, seed, std, specials)
        # store with the last logical dim first, view back
        perm = (nd - 1,) + tuple(range(nd - 1))
        base = typed(tuple(shape[p] for p in perm), dtype, seed, std, specials)
        inv = [0] * nd
        for i, p in enumerate(perm):
            inv[p] = i
        return base.permute(inv)
    if kind == "step2_inner":
        base = typed(shape[:-1] + (2 * shape[-1],), dtype, seed, std, specials)
        return base[..., ::2]
    if kind == "step2_outer":
        base = typed((2 * shape[0],) + shape[1:], dtype, seed, std, specials)
        return base[::2]
    if kind == "expand_row":
        base = typed((shape[0],) + (1,) * (nd - 1), dtype, seed, std, specials)
        return base.expand(shape)
    if kind == "expand_col":
        base = typed((1,) * (nd - 1) + (shape[-1],), dtype, seed, std, specials)
        return base.expand(shape)
    raise ValueError(kind)


def zipf_rows(n, support=65536, s=1.1, seed=0, permute=True):
    """n draws from the bounded Zipf law P(k) ~ k^-s on k = 1..support, by inverse CDF,
    mapped to row ids 0..support-1 (through a fixed random permutation when `permute`)."""
    g = _gen(seed)
    w = torch.arange(1, support + 1, dtype=torch.float64).pow(-s)
    cdf = torch.cumsum(w, 0)
    cdf /= cdf[-1].clone()
    u = torch.rand(n, generator=g, dtype=torch.float64)
    k = torch.searchsorted(cdf, u).clamp_(max=support - 1)
    if permute:
        perm = torch.randperm(support, generator=g)
        k = perm[k]
    return k.to(torch.int64)


# --------------------------------------------------------------------------- the five workloads
def broadcast_add_inputs(n=4096, m=4096, seed=0):
    """a[n,1], b[1,m] fp32 N(0,1), both from one generator stream."""
    g = _gen(seed)
    a = torch.randn((n, 1), generator=g, dtype=torch.float32)
    b = torch.randn((1, m), generator=g, dtype=torch.float32)
    return a, b


def reduction_input(shape=(64, 4096, 1024), dtype=torch.float32, seed=2):
    if dtype in INT_DTYPES:
        return integers(shape, -(2 ** 20), 2 ** 20, seed, dtype)
    return normal(shape, 1.0, seed, dtype)


def softmax_logits(shape=(32768, 4096), dtype=torch.float32, seed=3):
    return inject_neg_inf(normal(shape, 4.0, seed, torch.float32), 0.001, seed).to(dtype)


def cumsum_input(shape=(4096, 65536), dtype=torch.float32, seed=3):
    if dtype in INT_DTYPES:
        return integers(shape, -100, 100, seed, dtype)
    return normal(shape, 1.0, seed, dtype)


def cumprod_input(shape, dtype=torch.float32, seed=3):
    """Factors whose running product stays finite over long rows: 1 + 0.001 N(0,1) with one sign in ten flipped for the
    floating dtypes, odd integers in [-9, 9] (products wrap but never collapse to zero) for the integer ones."""
    if dtype in INT_DTYPES:
        return (integers(shape, -4, 4, seed, torch.int64) * 2 + 1).to(dtype)
    x = 1.0 + 0.001 * normal(shape, 1.0, seed, torch.float32)
    flip = torch.rand(shape, generator=_gen(seed + 1)) < 0.1
    return torch.where(flip, -x, x).to(dtype)


def uniform_indices(n, hi, seed=4, dtype=torch.int64):
    return torch.randint(0, hi, n if isinstance(n, tuple) else (n,), generator=_gen(seed), dtype=torch.int64).to(dtype)


def bernoulli_mask(shape, p=0.3, seed=4):
    return booleans(shape, p, seed + 7)
