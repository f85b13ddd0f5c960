"""Writes the text fixtures of this directory.  Run from the repository root: python tests/golden/make_golden.py

The paper prints no numeric worked example (its appendices hold prompts and kernels, not values), so there is no
paper value to store.  What is stored are the CPU oracle's results at fixed, hand-picked points for the three
operators whose kernels the paper does print - logsigmoid (Appendix D), binary_cross_entropy (Appendix B.1) and
layer_norm (Appendix B) - so that a change of the oracle's arithmetic shows up as a diff of a small text file, and
so that the GPU tests have expected values that do not depend on the oracle being built.  This script calls only
oracle/ (and torch to hold the numbers); tests/test_golden.py checks the stored values against mpmath as well.
"""
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import oracle as O  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
POINTS = [-100.0, -20.0, -5.0, -1.0, -0.125, -1e-6, 0.0, 1e-6, 0.125, 1.0, 5.0, 20.0, 100.0]
PROBS = [0.0, 1e-30, 0.001, 0.25, 0.5, 0.75, 0.999, 1.0]
TARGETS = [0.0, 0.25, 1.0]
ROW = [0.5, -1.25, 3.0, 0.0, 2.75, -0.875, 1.5, 4.0]


def hx(v):
    return float(v).hex()


def main():
    with open(os.path.join(HERE, "logsigmoid_appendix_d.txt"), "w") as f:
        f.write("# logsigmoid(x) = log(1 / (1 + exp(-x))) (the operator of Appendix D), CPU oracle, hexadecimal floats\n")
        f.write("# columns: x  fp32 result  bf16 result  fp16 result (inputs are exact in all three dtypes)\n")
        for x in POINTS:
            cols = [O.unary("logsigmoid", torch.tensor([x], dtype=dt)).double().item() for dt in (torch.float32, torch.bfloat16, torch.float16)]
            xs = [torch.tensor([x], dtype=dt).double().item() for dt in (torch.float32, torch.bfloat16, torch.float16)]
            f.write("%s %s %s %s %s %s\n" % (hx(xs[0]), hx(cols[0]), hx(xs[1]), hx(cols[1]), hx(xs[2]), hx(cols[2])))
    with open(os.path.join(HERE, "bce_appendix_b1.txt"), "w") as f:
        f.write("# binary_cross_entropy(x, t), reduction none, fp32 (the operator of Appendix B.1; logs clamped at -100), CPU oracle\n")
        f.write("# columns: x  t  loss\n")
        for x in PROBS:
            for t in TARGETS:
                loss = O.binary_cross_entropy(torch.tensor([x]), torch.tensor([t]), None, "none").item()
                f.write("%s %s %s\n" % (hx(torch.tensor(x).item()), hx(t), hx(loss)))
    with open(os.path.join(HERE, "layer_norm_appendix_b.txt"), "w") as f:
        f.write("# layer_norm of one row of 8 values, eps = 1e-5, weight w[j] = 1 + j / 8, bias b[j] = j / 4 - 1, fp32 (Appendix B), CPU oracle\n")
        f.write("# columns: x  w  b  y\n")
        x = torch.tensor([ROW])
        w = torch.tensor([1 + j / 8 for j in range(8)])
        b = torch.tensor([j / 4 - 1 for j in range(8)])
        y = O.layer_norm(x, 1, w, b, 1e-5)
        for j in range(8):
            f.write("%s %s %s %s\n" % (hx(x[0, j].item()), hx(w[j].item()), hx(b[j].item()), hx(y[0, j].item())))


if __name__ == "__main__":
    main()
