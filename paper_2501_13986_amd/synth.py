"""Seeded synthetic inputs with the shapes and distributions of the paper's workloads.

This module only *draws inputs*: Gaussian features and weights, unit vectors, the
spherical-harmonic edge attributes of those vectors, and radius-cutoff neighbour graphs in
a periodic box (the stand-in for the molecular graphs of the paper's Table 3, which are not
available).  It contains none of the tensor-product arithmetic, imports neither the HIP
library nor the CPU oracle, and is used by the tests and the benchmark to feed both.

Everything is generated in fp64 with numpy's PCG64 and cast by the caller.
"""
from __future__ import annotations

from math import pi, sqrt

import numpy as np

# the five benchmark configurations (irreps of x, y, z)
MACE_X = "128x0e+128x1o+128x2e"
MACE_Y = "1x0e+1x1o+1x2e+1x3o"
MACE_Z = "128x0e+128x1o+128x2e+128x3o"
NEQUIP_X = "32x0e+32x1o+32x2e"
NEQUIP_Y = "1x0e+1x1o+1x2e"
NEQUIP_Z = "32x0e+32x1o+32x2e"
# both parities of every degree up to 3 (a Nequip-like feature layout): 68 parity-allowed uvu paths
MANY_X = "+".join(f"8x{l}{p}" for l in range(4) for p in "eo")
MANY_Y = "1x0e+1x1o+1x2e+1x3o"
TINY_X = "4x0e+4x1o"
TINY_Y = "1x0e+1x1o"
TINY_Z = "4x0e+4x1o+4x1o+4x0e+4x1e+4x2e"       # one output segment per path, in path order
TINY_Z_MERGED = "4x0e+4x1o+4x1e+4x2e"


def normal(seed: int, shape, scale: float = 1.0) -> np.ndarray:
    return np.random.default_rng(seed).normal(size=shape) * scale


def unit_vectors(seed: int, n: int) -> np.ndarray:
    v = np.random.default_rng(seed).normal(size=(n, 3))
    return v / np.linalg.norm(v, axis=1, keepdims=True)


def sh_edge_attr(v: np.ndarray, lmax: int) -> np.ndarray:
    """Real spherical harmonics of unit vectors v[:, (x, y, z)] for l = 0..lmax (lmax <= 3),
    concatenated, ordered m = -l..l, scaled so that sum_m Y_lm^2 = 2l+1.  Explicit
    polynomials (degree 1 is sqrt3*(y, z, x))."""
    if not 0 <= lmax <= 3:
        raise ValueError("lmax must be in 0..3")
    x, y, z = v[:, 0], v[:, 1], v[:, 2]
    cols = [np.ones_like(x)]
    if lmax >= 1:
        s3 = sqrt(3.0)
        cols += [s3 * y, s3 * z, s3 * x]
    if lmax >= 2:
        s15 = sqrt(15.0)
        cols += [s15 * x * y, s15 * y * z, 0.5 * sqrt(5.0) * (3 * z * z - 1.0), s15 * x * z,
                 0.5 * s15 * (x * x - y * y)]
    if lmax >= 3:
        a, b, c = sqrt(70.0) / 4, sqrt(105.0), sqrt(42.0) / 4
        cols += [a * y * (3 * x * x - y * y), b * x * y * z, c * y * (5 * z * z - 1.0),
                 0.5 * sqrt(7.0) * z * (5 * z * z - 3.0), c * x * (5 * z * z - 1.0),
                 0.5 * b * z * (x * x - y * y), a * x * (x * x - 3 * y * y)]
    return np.stack(cols, axis=1)


def periodic_graph(seed: int, n_nodes: int, mean_degree: float, cutoff: float = 1.0, node_order: str = "random"):
    """n_nodes points uniform in a periodic cube sized so that a radius-`cutoff` ball holds
    `mean_degree` other points on average.  Returns (recv, send, unit) for every ordered
    pair within the cutoff under the minimum-image convention (both directions, no self
    loops), in a seeded random edge order; unit[e] = (r_send - r_recv)/|.|.
    node_order "random": node ids carry no spatial information (worst case for gathers);
    "cells": nodes numbered cell by cell on a grid of cutoff-sized cells, as a neighbour-list
    builder or a structure file ordered by residue leaves them (neighbours have nearby ids)."""
    from scipy.spatial import cKDTree

    rng = np.random.default_rng(seed)
    L = (n_nodes * (4.0 * pi / 3.0) * cutoff ** 3 / mean_degree) ** (1.0 / 3.0)
    if L <= 2 * cutoff:
        raise ValueError("box too small for the minimum-image convention")
    pos = rng.uniform(0.0, L, size=(n_nodes, 3))
    if node_order == "cells":
        nc = max(1, int(L / cutoff))
        c = np.minimum((pos / L * nc).astype(np.int64), nc - 1)
        pos = pos[np.lexsort((c[:, 2], c[:, 1], c[:, 0]))]
    elif node_order != "random":
        raise ValueError(node_order)
    pairs = cKDTree(pos, boxsize=L).query_pairs(cutoff, output_type="ndarray")
    recv = np.concatenate([pairs[:, 0], pairs[:, 1]]).astype(np.int64)
    send = np.concatenate([pairs[:, 1], pairs[:, 0]]).astype(np.int64)
    order = rng.permutation(recv.shape[0])
    recv, send = recv[order], send[order]
    d = pos[send] - pos[recv]
    d -= L * np.round(d / L)
    unit = d / np.linalg.norm(d, axis=1, keepdims=True)
    return recv, send, unit
