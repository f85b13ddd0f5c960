# Generates the polynomials used by gelu_erf_f32 (degree 16, binary64) and gelu_erf_half (degree 5, fp32)
# in math_fp.h:
#   erfcx(z) = exp(z^2) erfc(z) ~= P(t) / (z + 1.5),   t = (z - 1.5) / (z + 1.5),   z >= 0,
# fitted at Chebyshev nodes against 40-digit mpmath values.  Maximum relative error on [0, 60]:
# 2.1e-11 (degree 16, evaluated in binary64) and 5.5e-5 (degree 5, evaluated in fp32).
import mpmath
import numpy as np
from numpy.polynomial import chebyshev as C

mpmath.mp.dps = 40
K = 1.5


def erfcx(z):
    z = mpmath.mpf(z)
    return mpmath.exp(z * z) * mpmath.erfc(z)


def fit(degree, dtype):
    m = 400
    tn = np.cos(np.pi * (np.arange(m) + 0.5) / m)
    zn = K * (1 + tn) / (1 - tn)
    fn = np.array([float(K * (1 + z / K) * erfcx(z)) for z in zn])   # (z + 1.5) * erfcx(z)
    mono = C.cheb2poly(C.chebfit(tn, fn, degree)).astype(dtype)
    zt = np.concatenate([np.linspace(0, 10, 5001), np.linspace(10, 60, 300)]).astype(dtype)
    exact = np.array([float(erfcx(z)) for z in zt])
    r = (dtype(1) / (zt + dtype(K))).astype(dtype)
    t = ((zt - dtype(K)) * r).astype(dtype)
    acc = np.zeros_like(t)
    for co in mono[::-1]:
        acc = (acc * t + co).astype(dtype)
    err = np.max(np.abs(acc.astype(np.float64) * r / exact - 1))
    return mono, err


if __name__ == "__main__":
    for degree, dtype, fmt in ((16, np.float64, "%.17e"), (5, np.float32, "%.9ef")):
        mono, err = fit(degree, dtype)
        print("degree %d, max relative error %.3g" % (degree, err))
        for i, co in enumerate(mono):
            print(("  " + fmt + ",  // t^%d") % (co, i))
