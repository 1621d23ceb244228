"""Pins for oracle/cg.py: the CG blocks are checked against things other than themselves.

 - Racah closed form vs sympy's Clebsch-Gordan routine and hand-known values
 - orthogonality / completeness of the real blocks (unitarity of the coupling)
 - nonzero-count table (tests/golden/cg_nnz_table.txt) and its permutation invariance
 - closed forms: identity for (0,l,l), dot product (1,1,0), cross product (1,1,1),
   magnitudes of (1,1,2), (2,2,2) (tests/golden/cg_closed_forms.txt)
 - sign convention (first nonzero positive)
 - Gaunt's formula: coupling two spherical harmonics of the same direction
"""
import os
from math import sqrt

import numpy as np
import pytest

from oracle import cg, so3

GOLD = os.path.join(os.path.dirname(__file__), "golden")
LMAX = 4
TRIPLES = [(a, b, c) for a in range(LMAX + 1) for b in range(LMAX + 1) for c in range(LMAX + 1)
           if abs(a - b) <= c <= a + b]


def test_racah_against_sympy():
    from sympy.physics.quantum.cg import CG
    for (j1, j2, j3) in [(1, 1, 0), (1, 1, 1), (1, 1, 2), (2, 1, 3), (2, 2, 2), (2, 3, 3), (3, 2, 1), (3, 3, 4)]:
        for m1 in range(-j1, j1 + 1):
            for m2 in range(-j2, j2 + 1):
                m3 = m1 + m2
                if abs(m3) > j3:
                    continue
                ref = float(CG(j1, m1, j2, m2, j3, m3).doit())
                assert abs(cg.su2_cg(j1, m1, j2, m2, j3, m3) - ref) < 1e-14


def test_racah_known_values():
    assert abs(cg.su2_cg(1, 0, 1, 0, 2, 0) - sqrt(2 / 3)) < 1e-15
    assert abs(cg.su2_cg(1, 1, 1, -1, 0, 0) - 1 / sqrt(3)) < 1e-15
    assert abs(cg.su2_cg(1, 0, 1, 0, 0, 0) + 1 / sqrt(3)) < 1e-15
    assert abs(cg.su2_cg(1, 1, 1, -1, 1, 0) - 1 / sqrt(2)) < 1e-15
    assert cg.su2_cg(1, 0, 1, 0, 1, 0) == 0.0            # antisymmetric coupling
    assert cg.su2_cg(1, 1, 1, 1, 2, 1) == 0.0            # m3 != m1 + m2
    assert abs(cg.wigner_3j(2, 2, 2, 0, 0, 0) + sqrt(2 / 35)) < 1e-15
    assert abs(cg.wigner_3j(1, 1, 2, 0, 0, 0) - sqrt(2 / 15)) < 1e-15


def test_real_basis_matrix_unitary():
    for l in range(LMAX + 1):
        U = cg.real_basis_matrix(l)
        assert np.abs(U @ U.conj().T - np.eye(2 * l + 1)).max() < 1e-15


@pytest.mark.parametrize("l1,l2,l3", TRIPLES)
def test_orthogonality(l1, l2, l3):
    C = cg.cg_block(l1, l2, l3)
    G = np.einsum("ijk,ijl->kl", C, C)
    assert np.abs(G - np.eye(2 * l3 + 1)).max() < 1e-13
    assert abs(np.sum(C * C) - (2 * l3 + 1)) < 1e-13


@pytest.mark.parametrize("l1,l2", [(a, b) for a in range(4) for b in range(4)])
def test_completeness(l1, l2):
    tot = np.zeros((2 * l1 + 1, 2 * l2 + 1, 2 * l1 + 1, 2 * l2 + 1))
    for l3 in range(abs(l1 - l2), l1 + l2 + 1):
        C = cg.cg_block(l1, l2, l3)
        tot += np.einsum("ijk,abk->ijab", C, C)
    eye = np.einsum("ia,jb->ijab", np.eye(2 * l1 + 1), np.eye(2 * l2 + 1))
    assert np.abs(tot - eye).max() < 1e-13


def test_nnz_table_golden():
    rows = [tuple(int(t) for t in ln.split()) for ln in open(os.path.join(GOLD, "cg_nnz_table.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 20
    for l1, l2, l3, n in rows:
        for (a, b, c) in {(l1, l2, l3), (l2, l1, l3), (l3, l2, l1), (l1, l3, l2), (l2, l3, l1), (l3, l1, l2)}:
            assert len(cg.cg_nonzeros(a, b, c)) == n, (a, b, c)


def test_closed_form_magnitudes_golden():
    want = {}
    for ln in open(os.path.join(GOLD, "cg_closed_forms.txt")):
        if ln.strip() and not ln.startswith("#"):
            l1, l2, l3, v, n = ln.split()
            want.setdefault((int(l1), int(l2), int(l3)), []).append((float(v), int(n)))
    for (l1, l2, l3), vals in want.items():
        w = np.abs(cg.cg_block(l1, l2, l3)) / sqrt(2 * l3 + 1)
        nz = w[w > 0]
        for v, n in vals:
            hit = np.sum(np.abs(nz - v) < 1e-13)
            assert hit > 0
            if n:
                assert hit == n
        assert all(min(abs(t - v) for v, _ in vals) < 1e-13 for t in nz)


def test_identity_dot_cross():
    for l in range(LMAX + 1):
        C = cg.cg_block(0, l, l)
        assert np.abs(C[0] - np.eye(2 * l + 1)).max() < 1e-14          # 0e x l -> l is the identity
        C = cg.cg_block(l, 0, l)
        assert np.abs(C[:, 0, :] - np.eye(2 * l + 1)).max() < 1e-14
    a, b = np.array([0.3, -1.2, 0.7]), np.array([1.1, 0.4, -0.5])     # components in (y, z, x) order
    dot = np.einsum("ijk,i,j->k", cg.cg_block(1, 1, 0), a, b)
    assert abs(dot[0] - a @ b / sqrt(3)) < 1e-14
    # cross product: vectors are stored (y, z, x); convert, cross in (x, y, z), convert back
    to_xyz = lambda t: np.array([t[2], t[0], t[1]])
    to_yzx = lambda t: np.array([t[1], t[2], t[0]])
    cr = np.einsum("ijk,i,j->k", cg.cg_block(1, 1, 1), a, b)
    assert np.abs(cr - to_yzx(np.cross(to_xyz(a), to_xyz(b))) / sqrt(2)).max() < 1e-14


@pytest.mark.parametrize("l1,l2,l3", TRIPLES)
def test_sign_convention(l1, l2, l3):
    C = cg.cg_block(l1, l2, l3)
    flat = C.ravel()
    nz = np.flatnonzero(flat)
    assert flat[nz[0]] > 0
    # nonzero list is the same data, lexicographic
    lst = cg.cg_nonzeros(l1, l2, l3)
    assert [(i, j, k) for i, j, k, _ in lst] == sorted((i, j, k) for i, j, k, _ in lst)
    D = np.zeros_like(C)
    for i, j, k, v in lst:
        D[i, j, k] = v
    assert np.array_equal(C, D)


@pytest.mark.parametrize("l1,l2,l3", [t for t in TRIPLES if max(t) <= 3])
def test_gaunt(l1, l2, l3):
    """sum_{m1 m2} w[m1,m2,k] Y_l1(v) Y_l2(v) = s * sqrt((2l1+1)(2l2+1)/(2l3+1)) * 3j(l1 l2 l3;000) * Y_l3(v)
    for component-normalised harmonics, s = +-1 the block's sign choice; zero for odd l1+l2+l3."""
    rng = np.random.default_rng(5)
    v = rng.normal(size=(16, 3))
    w = cg.cg_block(l1, l2, l3) / sqrt(2 * l3 + 1)
    lhs = np.einsum("ijk,ni,nj->nk", w, so3.real_sh(l1, v), so3.real_sh(l2, v))
    if (l1 + l2 + l3) % 2:
        assert np.abs(lhs).max() < 1e-12
        return
    coef = sqrt((2 * l1 + 1) * (2 * l2 + 1) / (2 * l3 + 1)) * cg.wigner_3j(l1, l2, l3, 0, 0, 0)
    rhs = coef * so3.real_sh(l3, v)
    s = np.sign(np.sum(lhs * rhs))
    assert np.abs(lhs - s * rhs).max() < 1e-12
    assert abs(coef) > 1e-3
