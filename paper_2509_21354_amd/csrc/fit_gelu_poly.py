"""Derives the constants of ``gelu_poly`` in ``pool_token_mfma.hip``.

GELU(z) = z * Phi(z) = max(z, 0) - |z| * E(|z|) with E(u) = erfc(u / sqrt 2) / 2 (the upper tail of
the normal distribution).  On [0, U_MAX] the function log2 E(u) + 1 is smooth and vanishes at 0,
so it is fitted as u * P(u) with P a polynomial; E comes back through one hardware exp2.  The fit
is a least-squares fit on Chebyshev nodes, re-weighted a few times towards the minimax error of E
itself (what matters is the absolute error of Phi).  Beyond U_MAX the argument is clamped
(E(U_MAX) = 7.7e-9).  Run ``python fit_gelu_poly.py`` to print the coefficients and the error of a
float32 evaluation; ``coefficients()`` is what the test of the constants imports.
"""
import numpy as np
from scipy import special

U_MAX = 4.0 * np.sqrt(2.0)
DEGREE = 7          # number of coefficients of P


def tail(u):
    return special.erfc(np.asarray(u, dtype=np.float64) / np.sqrt(2.0)) * 0.5


def coefficients(degree: int = DEGREE) -> np.ndarray:
    n = 4000
    x = np.cos(np.pi * (np.arange(n) + 0.5) / n)
    u = (x + 1.0) * U_MAX / 2.0
    E = tail(u)
    target = np.log2(E) + 1.0
    w = E.copy()                               # d E = ln 2 * E * d(log2 E)
    A = np.stack([u ** (k + 1) for k in range(degree)], 1)
    coef = None
    for _ in range(30):
        coef, *_ = np.linalg.lstsq(A * w[:, None], target * w, rcond=None)
        err = np.abs((A @ coef - target) * E * np.log(2.0))
        w = w * (1.0 + 3.0 * err / err.max())
    return coef


def tail_f32(u: np.ndarray, coef: np.ndarray) -> np.ndarray:
    """The kernel's evaluation order in float32 (Horner; exp2 taken exactly)."""
    u = np.minimum(np.asarray(u).astype(np.float32), np.float32(U_MAX))
    c = np.asarray(coef).astype(np.float32)
    q = np.full_like(u, c[-1])
    for k in range(len(c) - 2, -1, -1):
        q = (q * u + c[k]).astype(np.float32)
    q = (q * u - np.float32(1.0)).astype(np.float32)
    return np.exp2(q.astype(np.float64)).astype(np.float32)


if __name__ == "__main__":
    c = coefficients()
    for k, v in enumerate(c):
        print(f"c{k} = {np.float32(v)!r:>16}  ({v:.17e})")
    print("U_MAX =", repr(np.float32(U_MAX)))
    uu = np.linspace(0.0, 12.0, 400001)
    print("max |E_poly - E| in float32:", np.abs(tail_f32(uu, c) - tail(uu)).max())
