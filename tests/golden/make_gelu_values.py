"""Writes gelu_values.json: GELU(u) = u * Phi(u) with the normal cdf Phi obtained by
Gauss-Legendre quadrature of the normal density, i.e. without calling erf."""
import json
import math
import os

import numpy as np
from numpy.polynomial.legendre import leggauss

xs, ws = leggauss(200)


def Phi(u):
    t = 0.5 * u * (xs + 1)
    return 0.5 + 0.5 * u * float(np.sum(ws * np.exp(-0.5 * t * t))) / math.sqrt(2 * math.pi)


u = [-3.0, -1.5, -0.5, 0.25, 1.0, 2.0, 4.0]
out = {"_source": "GELU(u) = u * Phi(u), Phi by 200-point Gauss-Legendre quadrature of the normal pdf "
                  "(written by tests/golden/make_gelu_values.py)",
       "u": u, "gelu": [x * Phi(x) for x in u]}
with open(os.path.join(os.path.dirname(__file__), "gelu_values.json"), "w") as f:
    json.dump(out, f, indent=1)
