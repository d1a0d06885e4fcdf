"""Fits the constants of the GELU epilogue in device_common.h.

gelu(v) = v/2 (1 + erf(v / sqrt 2)) is evaluated as v * sigmoid(a v + b v^3 + c v^5) with v^2 clamped
at 81 (beyond |v| = 9 the sigmoid is 0 or 1 to within 1e-11).  a, b, c minimise the largest absolute
deviation from the erf form on [-10, 10]; the script prints them, the deviation, and the constants
folded with -log2(e) as the kernel uses them.  Needs numpy and scipy.

Run:  python fit_gelu_sigmoid.py
"""
import math

import numpy as np
from scipy.optimize import minimize


def main() -> None:
    v = np.linspace(-10.0, 10.0, 80001)
    ref = 0.5 * v * (1.0 + np.vectorize(math.erf)(v / math.sqrt(2.0)))

    def model(p):
        t = np.minimum(v * v, 81.0)
        return v / (1.0 + np.exp(-v * (p[0] + p[1] * t + p[2] * t * t)))

    res = minimize(lambda p: np.max(np.abs(model(p) - ref)), [1.6, 0.07, 0.0], method="Nelder-Mead",
                   options=dict(xatol=1e-12, fatol=1e-13, maxiter=40000, maxfev=80000))
    a, b, c = res.x
    print("a, b, c =", a, b, c, " max |error| =", res.fun)
    log2e = 1.4426950408889634
    print("kernel constants (times -log2 e):", -log2e * a, -log2e * b, -log2e * c)


if __name__ == "__main__":
    main()
