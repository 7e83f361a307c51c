"""Fit behind the GELU kernel's complementary error function (xp_memops.hip: erfc_pos).

    erfc(z) = t * exp(-z*z + p(t)),   t = 1 / (1 + z/2),   z >= 0

p is a degree-8 polynomial: a Chebyshev least-squares fit of ln(erfcx(z) / t) over t in [1/6, 1]
(z in [0, 10]; scipy's scaled complementary error function erfcx is the target), converted to
power-series coefficients.  The script prints the coefficients and the relative error of the fp32
evaluation, which is dominated by the rounding of -z*z + p(t) ahead of the exponential
(about 1e-6 for z <= 3, 4e-6 for z <= 6), not by the fit.

    python paper_2505_02146_amd/csrc/fit_erfc.py
"""
import numpy as np
from numpy.polynomial import chebyshev as C, polynomial as P
from scipy.special import erfc, erfcx

DEGREE, ZMAX = 8, 10.0


def fit():
    t = np.linspace(1.0 / (1.0 + ZMAX / 2), 1.0, 20001)
    z = 2.0 * (1.0 / t - 1.0)
    cheb = C.Chebyshev.fit(t, np.log(erfcx(z) / t), DEGREE, domain=[t[0], 1.0])
    return cheb.convert(kind=P.Polynomial, domain=[-1, 1], window=[-1, 1]).coef.astype(np.float32)


def fp32_error(co):
    z = np.linspace(0, 9.0, 400001).astype(np.float32)
    t = (np.float32(1) / (np.float32(1) + np.float32(0.5) * z)).astype(np.float32)
    acc = np.full_like(t, co[-1])
    for c in co[-2::-1]:
        acc = (acc * t + c).astype(np.float32)
    val = t * np.exp((-(z * z) + acc).astype(np.float32)).astype(np.float32)
    ref = erfc(z.astype(np.float64))
    rel = np.abs(val.astype(np.float64) - ref) / ref
    return rel[z <= 3].max(), rel[z <= 6].max(), rel.max()


if __name__ == "__main__":
    co = fit()
    print("coefficients of t^0 .. t^%d:" % DEGREE)
    print(", ".join(f"{float(c):.9g}f" for c in co))
    print("max relative error in fp32: z <= 3: %.2e   z <= 6: %.2e   z <= 9: %.2e" % fp32_error(co))
