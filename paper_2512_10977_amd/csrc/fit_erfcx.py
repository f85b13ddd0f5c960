# Generates the degree-16 polynomial used by gelu_erf_f32 in math_fp.h:
# erfcx(z) = exp(z^2) erfc(z) ~= P(t) / (z + 1.5), t = (z - 1.5) / (z + 1.5), z >= 0,
# fitted at Chebyshev nodes against 40-digit mpmath values (max relative error 2.1e-11).
import numpy as np, mpmath
from numpy.polynomial import chebyshev as C, polynomial as P
mpmath.mp.dps = 40
def erfcx(z):
    z = mpmath.mpf(z); return mpmath.exp(z*z)*mpmath.erfc(z)
k=1.5; N=16; M=400
tn = np.cos(np.pi*(np.arange(M)+0.5)/M)
zn = k*(1+tn)/(1-tn)
fn = np.array([float(k*(1+z/k)*erfcx(z)) for z in zn])   # fold the 1.5 factor in: erfcx = P(t) * r, r = 1/(z+1.5)
c = C.chebfit(tn, fn, N)
mono = C.cheb2poly(c)
zt = np.concatenate([np.linspace(0, 10, 5001), np.linspace(10,60,300)])
exact = np.array([float(erfcx(z)) for z in zt])
r = 1/(zt+k); tt=(zt-k)*r
acc = np.zeros_like(tt)
for co in mono[::-1]: acc = acc*tt + co
print(np.max(np.abs(acc*r/exact-1)))
for i,co in enumerate(mono): print("  %.17e,  // t^%d" % (co,i))
