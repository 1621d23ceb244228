"""Clebsch-Gordan blocks P^(l1,l2,l3) in the real spherical-harmonic basis (oracle side).

The paper (Sec. 2.2-2.3) takes the coefficient tensor as given (it obtains it from a
third-party package, Sec. 4).  Here it is built from first principles:

  1. complex SU(2) Clebsch-Gordan coefficients from Racah's closed form, in exact
     rational arithmetic up to the final square root;
  2. Wigner 3j symbols from them (a fully symmetric invariant 3-tensor);
  3. change of basis complex -> real spherical harmonics with the unitary U^l below;
     for odd l1+l2+l3 the result is purely imaginary and is multiplied by i;
  4. overall sign fixed so that the first nonzero entry in lexicographic (m1,m2,m3)
     order is positive (an overall sign per block is pure convention);
  5. "component" normalisation: C = sqrt(2*l3+1) * w with ||w||_F = 1, so that
     sum_{m1 m2} C[m1,m2,k] C[m1,m2,k'] = delta_{kk'}.

Steps 3-5 are conventions the paper leaves to the packages it builds on; no claim of
element-wise equality with any other package is made (parity unpinned against e3nn; the
block is pinned by orthogonality, equivariance, closed forms and Gaunt's formula instead).

Test infrastructure only; the HIP library has its own, separately written generator.
"""
from __future__ import annotations

from fractions import Fraction
from functools import lru_cache
from math import factorial, sqrt

import numpy as np

ZERO_TOL = 1e-12


def su2_cg(j1: int, m1: int, j2: int, m2: int, j3: int, m3: int) -> float:
    """<j1 m1 j2 m2 | j3 m3> for integer angular momenta, Racah's closed form."""
    if m1 + m2 != m3 or not (abs(j1 - j2) <= j3 <= j1 + j2):
        return 0.0
    if abs(m1) > j1 or abs(m2) > j2 or abs(m3) > j3:
        return 0.0
    f = factorial
    pref = Fraction((2 * j3 + 1) * f(j3 + j1 - j2) * f(j3 - j1 + j2) * f(j1 + j2 - j3), f(j1 + j2 + j3 + 1))
    pref *= f(j3 + m3) * f(j3 - m3) * f(j1 - m1) * f(j1 + m1) * f(j2 - m2) * f(j2 + m2)
    s = Fraction(0)
    for k in range(0, j1 + j2 - j3 + 1):
        args = (k, j1 + j2 - j3 - k, j1 - m1 - k, j2 + m2 - k, j3 - j2 + m1 + k, j3 - j1 - m2 + k)
        if min(args) < 0:
            continue
        den = 1
        for a in args:
            den *= f(a)
        s += Fraction((-1) ** k, den)
    # sqrt(pref) * s, with pref a positive rational
    return float(s) * sqrt(pref.numerator) / sqrt(pref.denominator)


def wigner_3j(j1, j2, j3, m1, m2, m3) -> float:
    """(j1 j2 j3; m1 m2 m3) = (-1)^(j1-j2-m3) / sqrt(2 j3+1) <j1 m1 j2 m2 | j3 -m3>."""
    if m1 + m2 + m3 != 0:
        return 0.0
    return (-1) ** ((j1 - j2 - m3) % 2) / sqrt(2 * j3 + 1) * su2_cg(j1, m1, j2, m2, j3, -m3)


def real_basis_matrix(l: int) -> np.ndarray:
    """U^l with Y^real_{l m} = sum_mu U[m, mu] Y^complex_{l mu}; rows/cols ordered -l..l.

    m > 0:  (Y^{-m} + (-1)^m Y^{m}) / sqrt2  = sqrt2 (-1)^m Re Y^m
    m < 0:  i (Y^{m} - (-1)^m Y^{-m}) / sqrt2 = sqrt2 (-1)^m Im Y^{|m|}
    (Condon-Shortley phase in the complex harmonics.)  Degree 1 comes out as (y, z, x).
    """
    U = np.zeros((2 * l + 1, 2 * l + 1), dtype=complex)
    r = 1.0 / sqrt(2.0)
    for m in range(-l, l + 1):
        if m < 0:
            U[m + l, m + l] = 1j * r
            U[m + l, -m + l] = -1j * r * (-1) ** (m % 2)
        elif m == 0:
            U[l, l] = 1.0
        else:
            U[m + l, -m + l] = r
            U[m + l, m + l] = r * (-1) ** (m % 2)
    return U


@lru_cache(maxsize=None)
def _real_invariant(l1: int, l2: int, l3: int):
    """Unit-norm, sign-canonical real invariant tensor w[m1, m2, m3] (steps 1-4)."""
    t = np.zeros((2 * l1 + 1, 2 * l2 + 1, 2 * l3 + 1))
    for a in range(-l1, l1 + 1):
        for b in range(-l2, l2 + 1):
            c = -a - b
            if abs(c) <= l3:
                t[a + l1, b + l2, c + l3] = wigner_3j(l1, l2, l3, a, b, c)
    U1c, U2c, U3c = (np.conj(real_basis_matrix(l)) for l in (l1, l2, l3))
    w = np.einsum("abc,ia,jb,kc->ijk", t.astype(complex), U1c, U2c, U3c)
    if (l1 + l2 + l3) % 2 == 1:
        w = 1j * w
    if np.abs(w.imag).max() > 1e-13:
        raise AssertionError("real-basis CG block is not real")
    w = w.real.copy()
    w[np.abs(w) < ZERO_TOL] = 0.0
    nz = np.flatnonzero(w)  # C order == lexicographic (m1, m2, m3)
    if nz.size and w.flat[nz[0]] < 0:
        w = -w
    w.setflags(write=False)
    return w


def cg_block(l1: int, l2: int, l3: int) -> np.ndarray:
    """C[i, j, k] = sqrt(2 l3 + 1) * w[i, j, k]; zero array shape if triangle rule fails."""
    if not (abs(l1 - l2) <= l3 <= l1 + l2):
        return np.zeros((2 * l1 + 1, 2 * l2 + 1, 2 * l3 + 1))
    return sqrt(2 * l3 + 1) * _real_invariant(l1, l2, l3)


def cg_nonzeros(l1: int, l2: int, l3: int):
    """List of (i, j, k, v) with v != 0, lexicographic in (i, j, k): nz(P) of Alg. 2."""
    C = cg_block(l1, l2, l3)
    return [(int(i), int(j), int(k), float(C[i, j, k])) for i, j, k in zip(*np.nonzero(C))]
