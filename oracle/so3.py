"""Real spherical harmonics and Wigner D matrices (oracle side).

Paper Sec. 2.1: a function is equivariant when f(D_in(g) v) = D_out(g) f(v), and the
representations are block diagonal with Wigner blocks D^(l)(g) of size 2l+1.  The paper's
workloads take y = spherical harmonics of an edge direction.  Both objects are written
here from their textbook definitions, in the real basis fixed by cg.real_basis_matrix
and with "component" normalisation ||Y_l(v)||^2 = 2l+1 on the unit sphere.

Test infrastructure only.
"""
from __future__ import annotations

from math import factorial, sqrt, pi

import numpy as np
from scipy.special import lpmv

from .cg import real_basis_matrix


def complex_sh(l: int, v: np.ndarray) -> np.ndarray:
    """Y_l^m(v/|v|), m = -l..l along the last axis (orthonormal on the sphere,
    Condon-Shortley phase): sqrt((2l+1)/(4pi) (l-m)!/(l+m)!) P_l^m(cos th) e^{i m ph}."""
    v = np.asarray(v, dtype=float)
    r = np.linalg.norm(v, axis=-1)
    ct = v[..., 2] / r
    ph = np.arctan2(v[..., 1], v[..., 0])
    out = np.zeros(v.shape[:-1] + (2 * l + 1,), dtype=complex)
    for m in range(0, l + 1):
        n = sqrt((2 * l + 1) / (4 * pi) * factorial(l - m) / factorial(l + m))
        ylm = n * lpmv(m, l, ct) * np.exp(1j * m * ph)
        out[..., l + m] = ylm
        if m > 0:
            out[..., l - m] = (-1) ** m * np.conj(ylm)
    return out


def real_sh(l: int, v: np.ndarray) -> np.ndarray:
    """Component-normalised real harmonics sqrt(4 pi) U^l Y^complex_l(v/|v|), m = -l..l."""
    yc = complex_sh(l, v)
    yr = sqrt(4 * pi) * np.einsum("mu,...u->...m", real_basis_matrix(l), yc)
    assert np.abs(yr.imag).max(initial=0.0) < 1e-12
    return yr.real


def real_sh_all(lmax: int, v: np.ndarray) -> np.ndarray:
    """Concatenation of real_sh(0..lmax): the y operand "1x0e+1x1o+...": dim (lmax+1)^2."""
    return np.concatenate([real_sh(l, v) for l in range(lmax + 1)], axis=-1)


def rot_z(a: float) -> np.ndarray:
    c, s = np.cos(a), np.sin(a)
    return np.array([[c, -s, 0.0], [s, c, 0.0], [0.0, 0.0, 1.0]])


def rot_y(b: float) -> np.ndarray:
    c, s = np.cos(b), np.sin(b)
    return np.array([[c, 0.0, s], [0.0, 1.0, 0.0], [-s, 0.0, c]])


def euler_matrix(alpha: float, beta: float, gamma: float) -> np.ndarray:
    """Active rotation R = Rz(alpha) Ry(beta) Rz(gamma) acting on column vectors (x,y,z)."""
    return rot_z(alpha) @ rot_y(beta) @ rot_z(gamma)


def wigner_small_d(l: int, beta: float) -> np.ndarray:
    """d^l_{m' m}(beta), Wigner's closed form; rows m', columns m, both -l..l."""
    f = factorial
    c, s = np.cos(beta / 2), np.sin(beta / 2)
    d = np.zeros((2 * l + 1, 2 * l + 1))
    for mp in range(-l, l + 1):
        for m in range(-l, l + 1):
            pref = sqrt(f(l + mp) * f(l - mp) * f(l + m) * f(l - m))
            tot = 0.0
            for k in range(0, 2 * l + 1):
                a = (l + m - k, k, mp - m + k, l - mp - k)
                if min(a) < 0:
                    continue
                tot += (-1) ** ((mp - m + k) % 2) / (f(a[0]) * f(a[1]) * f(a[2]) * f(a[3])) \
                    * c ** (2 * l + m - mp - 2 * k) * s ** (mp - m + 2 * k)
            d[mp + l, m + l] = pref * tot
    return d


def wigner_D_complex(l: int, alpha: float, beta: float, gamma: float) -> np.ndarray:
    """D^l_{m' m} = e^{-i m' alpha} d^l_{m' m}(beta) e^{-i m gamma} (z-y-z Euler angles)."""
    m = np.arange(-l, l + 1)
    return np.exp(-1j * m[:, None] * alpha) * wigner_small_d(l, beta) * np.exp(-1j * m[None, :] * gamma)


def wigner_D_real(l: int, alpha: float, beta: float, gamma: float) -> np.ndarray:
    """Real orthogonal D with real_sh(l, R v) = D real_sh(l, v), R = euler_matrix(...).

    The complex harmonics obey Y(R v) = conj(D(R)) Y(v), hence D_real = U conj(D) U^dagger.
    """
    U = real_basis_matrix(l)
    D = U @ np.conj(wigner_D_complex(l, alpha, beta, gamma)) @ U.conj().T
    assert np.abs(D.imag).max() < 1e-12
    return D.real


def fitted_D_real(l: int, R: np.ndarray, rng: np.random.Generator, n: int = 64) -> np.ndarray:
    """The matrix D with real_sh(l, R v) = D real_sh(l, v), recovered by least squares from
    n random directions.  R may be improper (det -1).  Independent of the Euler-angle
    formulas above, which it serves to check."""
    v = rng.normal(size=(n, 3))
    A = real_sh(l, v)                # [n, 2l+1]
    B = real_sh(l, v @ R.T)          # [n, 2l+1]
    Dt, *_ = np.linalg.lstsq(A, B, rcond=None)
    return Dt.T


def block_diag_D(irreps, D_of_l, improper: bool = False) -> np.ndarray:
    """Block-diagonal representation matrix for a list of oracle.irreps.Irrep in the
    mul-major layout (index u*(2l+1)+m).  `D_of_l(l)` returns the proper-rotation block;
    if `improper`, odd-parity irreps pick up a factor -1 (inversion times the rotation)."""
    n = sum(ir.dim for ir in irreps)
    M = np.zeros((n, n))
    o = 0
    for ir in irreps:
        d = 2 * ir.l + 1
        blk = D_of_l(ir.l) * (ir.p if improper else 1)
        for u in range(ir.mul):
            M[o:o + d, o:o + d] = blk
            o += d
    return M
