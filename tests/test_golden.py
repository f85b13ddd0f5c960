"""The stored fixtures of tests/golden: the oracle still reproduces them, mpmath agrees with them, and (GPU) the HIP
library reproduces them through the C ABI.  The operators are the three whose kernels the paper prints (Appendix B,
B.1 and D); the values were written by tests/golden/make_golden.py, which calls only the oracle."""
import math
import os

import mpmath
import pytest
import torch

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
F32, BF16, F16 = torch.float32, torch.bfloat16, torch.float16


def rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [[float.fromhex(c) for c in line.split()] for line in f if line.strip() and not line.startswith("#")]


SUBNORMAL = {23: -149, 7: -133, 10: -24}                # spacing of the format's smallest numbers, by mantissa width


def ulp_of(v, bits):
    floor = mpmath.mpf(2) ** SUBNORMAL[bits]
    return max(mpmath.mpf(2) ** (math.floor(math.log2(abs(v))) - bits), floor) if v else floor


def test_stored_values_agree_with_mpmath():
    mpmath.mp.dps = 50
    for r in rows("logsigmoid_appendix_d.txt"):
        for (x, y), bits in zip(((r[0], r[1]), (r[2], r[3]), (r[4], r[5])), (23, 7, 10)):
            exact = -mpmath.log(1 + mpmath.exp(-mpmath.mpf(x)))
            assert abs(mpmath.mpf(y) - exact) <= ulp_of(float(exact), bits) * mpmath.mpf("0.5001"), (x, y)
    for x, t, loss in rows("bce_appendix_b1.txt"):
        lx = max(mpmath.log(mpmath.mpf(x)), -100) if x > 0 else mpmath.mpf(-100)
        l1x = max(mpmath.log(1 - mpmath.mpf(x)), -100) if x < 1 else mpmath.mpf(-100)
        exact = -(mpmath.mpf(t) * lx + (1 - mpmath.mpf(t)) * l1x)
        assert abs(mpmath.mpf(loss) - exact) <= ulp_of(float(exact), 23) * mpmath.mpf("0.5001"), (x, t, loss)
    r = rows("layer_norm_appendix_b.txt")
    xs = [mpmath.mpf(v[0]) for v in r]
    mean = sum(xs) / 8
    var = sum((v - mean) ** 2 for v in xs) / 8
    for x, w, b, y in r:
        exact = (mpmath.mpf(x) - mean) / mpmath.sqrt(var + mpmath.mpf(float.fromhex((1e-5).hex()))) * mpmath.mpf(w) + mpmath.mpf(b)
        assert abs(mpmath.mpf(y) - exact) <= ulp_of(float(exact), 23) * mpmath.mpf("0.5001") + mpmath.mpf(2) ** -26, (x, y)


def test_oracle_reproduces_the_stored_values():
    from oracle import oracle as O
    for r in rows("logsigmoid_appendix_d.txt"):
        for (x, y), dt in zip(((r[0], r[1]), (r[2], r[3]), (r[4], r[5])), (F32, BF16, F16)):
            assert O.unary("logsigmoid", torch.tensor([x], dtype=dt)).double().item() == y
    for x, t, loss in rows("bce_appendix_b1.txt"):
        assert O.binary_cross_entropy(torch.tensor([x]), torch.tensor([t]), None, "none").item() == loss
    r = torch.tensor(rows("layer_norm_appendix_b.txt"), dtype=torch.float64)
    y = O.layer_norm(r[:, 0].float().view(1, 8), 1, r[:, 1].float(), r[:, 2].float(), 1e-5)
    assert torch.equal(y.view(-1).double(), r[:, 3])


@pytest.mark.gpu
def test_library_reproduces_the_stored_values():
    from paper_2512_10977_amd import binding as B
    from tests.parity import assert_rel, assert_ulp
    r = torch.tensor(rows("logsigmoid_appendix_d.txt"), dtype=torch.float64)
    for k, dt in enumerate((F32, BF16, F16)):
        x, want = r[:, 2 * k].to(dt), r[:, 2 * k + 1].to(dt)
        out = torch.empty(x.shape, dtype=dt, device="cuda")
        B.tx_unary("logsigmoid", out, x.cuda())
        if dt == F32:
            assert_ulp(out, want, 2, "logsigmoid fixture fp32")
        else:
            assert_rel(out, want, 1e-2, scale=1e-30, what="logsigmoid fixture %s" % dt)
    r = torch.tensor(rows("bce_appendix_b1.txt"), dtype=torch.float64)
    x, t, want = r[:, 0].float(), r[:, 1].float(), r[:, 2].float()
    out = torch.empty(x.shape, dtype=F32, device="cuda")
    B.tx_binary_cross_entropy(out, x.cuda(), t.cuda(), None, "none")
    assert_rel(out, want, 1e-5, scale=1e-30, what="binary_cross_entropy fixture")
    r = torch.tensor(rows("layer_norm_appendix_b.txt"), dtype=torch.float64)
    out = torch.empty((1, 8), dtype=F32, device="cuda")
    B.tx_layer_norm(out, r[:, 0].float().view(1, 8).cuda(), 1, r[:, 1].float().cuda(), r[:, 2].float().cuda(), 1e-5)
    assert_rel(out.view(-1), r[:, 3].float(), 1e-5, scale=1.0, what="layer_norm fixture")
