"""Pins for oracle/so3.py: harmonics against explicit polynomials and norms, Wigner D against
the rotation matrix itself (degree 1), against a least-squares fit from the harmonics, and
against the group law."""
from math import sqrt

import numpy as np
import pytest

from oracle import so3

RNG = np.random.default_rng(11)


def test_sh_explicit_low_degrees():
    v = RNG.normal(size=(32, 3))
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    x, y, z = v.T
    assert np.abs(so3.real_sh(0, v)[:, 0] - 1.0).max() < 1e-14
    assert np.abs(so3.real_sh(1, v) - sqrt(3) * np.stack([y, z, x], 1)).max() < 1e-14
    y2 = np.stack([sqrt(15) * x * y, sqrt(15) * y * z, sqrt(5) / 2 * (3 * z * z - 1), sqrt(15) * x * z,
                   sqrt(15) / 2 * (x * x - y * y)], 1)
    assert np.abs(so3.real_sh(2, v) - y2).max() < 1e-13


@pytest.mark.parametrize("l", range(5))
def test_sh_norm_and_scale_invariance(l):
    v = RNG.normal(size=(50, 3))
    Y = so3.real_sh(l, v)
    assert np.abs((Y * Y).sum(1) - (2 * l + 1)).max() < 1e-12
    assert np.abs(so3.real_sh(l, 3.7 * v) - Y).max() < 1e-12
    assert np.abs(so3.real_sh(l, -v) - (-1) ** l * Y).max() < 1e-12      # parity (-1)^l


@pytest.mark.parametrize("l", range(5))
def test_sh_orthonormal_on_sphere(l):
    # Monte-Carlo-free check: Lebedev-like product quadrature (Gauss-Legendre x uniform phi)
    n = 12
    ct, wt = np.polynomial.legendre.leggauss(n)
    ph = np.arange(2 * n) * np.pi / n
    CT, PH = np.meshgrid(ct, ph, indexing="ij")
    st = np.sqrt(1 - CT ** 2)
    v = np.stack([st * np.cos(PH), st * np.sin(PH), CT], -1).reshape(-1, 3)
    w = np.repeat(wt, 2 * n) * (np.pi / n) / (4 * np.pi)
    Y = so3.real_sh(l, v)
    G = np.einsum("n,na,nb->ab", w, Y, Y)
    assert np.abs(G - np.eye(2 * l + 1)).max() < 1e-12


@pytest.mark.parametrize("l", range(5))
def test_wigner_D(l):
    a, b, g = RNG.uniform(0, 2 * np.pi, 3)
    R = so3.euler_matrix(a, b, g)
    assert abs(np.linalg.det(R) - 1) < 1e-14
    D = so3.wigner_D_real(l, a, b, g)
    assert np.abs(D @ D.T - np.eye(2 * l + 1)).max() < 1e-13
    v = RNG.normal(size=(20, 3))
    assert np.abs(so3.real_sh(l, v @ R.T) - so3.real_sh(l, v) @ D.T).max() < 1e-12
    assert np.abs(D - so3.fitted_D_real(l, R, RNG)).max() < 1e-11
    if l == 1:   # (y, z, x) ordering: D = P R P^T with P the cyclic permutation
        P = np.array([[0, 1, 0], [0, 0, 1], [1, 0, 0]], float)
        assert np.abs(D - P @ R @ P.T).max() < 1e-14
    # group law through the fitted matrices
    a2, b2, g2 = RNG.uniform(0, 2 * np.pi, 3)
    R2 = so3.euler_matrix(a2, b2, g2)
    D2 = so3.wigner_D_real(l, a2, b2, g2)
    assert np.abs(so3.fitted_D_real(l, R @ R2, RNG) - D @ D2).max() < 1e-11


def test_small_d_known_values():
    b = 0.83
    d1 = so3.wigner_small_d(1, b)
    assert abs(d1[1, 1] - np.cos(b)) < 1e-15                     # d^1_00
    assert abs(d1[2, 2] - (1 + np.cos(b)) / 2) < 1e-15           # d^1_11
    assert abs(d1[2, 1] + np.sin(b) / sqrt(2)) < 1e-15           # d^1_10
    assert abs(so3.wigner_small_d(2, b)[2, 2] - (3 * np.cos(b) ** 2 - 1) / 2) < 1e-15
