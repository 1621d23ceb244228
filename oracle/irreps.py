"""Irreps strings, segment offsets and path enumeration (oracle side).

Paper Sec. 2.1: a block-diagonal O(3) representation is written "3x1e + 1x2o": a list of
(multiplicity, degree l, parity) terms; a term with degree l occupies mul*(2l+1) words.
Paper Sec. 2.4 (Eq. 2): a problem is three such lists plus a list of
(x-segment, y-segment, z-segment, kernel kind) instructions.

Test infrastructure only; shares no code with the planner in the HIP library.
"""
from __future__ import annotations

import re
from dataclasses import dataclass
from typing import List, Sequence, Tuple

UVU = 0  # paper's sub-kernel B: diagonal weight tile, one weight per channel
UVW = 1  # paper's sub-kernel C: dense mul_x x mul_z weight tile


@dataclass(frozen=True)
class Irrep:
    mul: int
    l: int
    p: int  # +1 even, -1 odd

    @property
    def dim(self) -> int:
        return self.mul * (2 * self.l + 1)


_TERM = re.compile(r"^\s*(?:(\d+)\s*x\s*)?(\d+)\s*([eo])\s*$")


def parse_irreps(s: str) -> List[Irrep]:
    """Parse "128x0e+128x1o" into a list of Irrep.  A missing multiplicity means 1."""
    out = []
    if s.strip() == "":
        raise ValueError("empty irreps string")
    for term in s.split("+"):
        m = _TERM.match(term)
        if not m:
            raise ValueError(f"bad irreps term {term!r}")
        mul = int(m.group(1)) if m.group(1) is not None else 1
        if mul <= 0:
            raise ValueError(f"multiplicity must be positive in {term!r}")
        out.append(Irrep(mul, int(m.group(2)), +1 if m.group(3) == "e" else -1))
    return out


def offsets(irreps: Sequence[Irrep]) -> List[int]:
    """Start word of every segment, plus the total dimension as the last entry."""
    off = [0]
    for ir in irreps:
        off.append(off[-1] + ir.dim)
    return off


def dim(irreps: Sequence[Irrep]) -> int:
    return offsets(irreps)[-1]


def path_allowed(a: Irrep, b: Irrep, c: Irrep) -> bool:
    """Triangle rule |l1-l2| <= l3 <= l1+l2 and parity product rule p3 = p1*p2."""
    return abs(a.l - b.l) <= c.l <= a.l + b.l and c.p == a.p * b.p


def enumerate_paths(irx, iry, irz) -> List[Tuple[int, int, int]]:
    """Every allowed (ix, iy, iz) triple, in lexicographic order."""
    return [
        (ix, iy, iz)
        for ix, a in enumerate(irx)
        for iy, b in enumerate(iry)
        for iz, c in enumerate(irz)
        if path_allowed(a, b, c)
    ]


@dataclass(frozen=True)
class Path:
    ix: int
    iy: int
    iz: int
    mode: int = UVU
    coeff: float = 1.0


class TPSpec:
    """A CG tensor product problem (paper Eq. 2) with the weight layout of this project:
    paths sorted by (ix, iy, iz); a uvu path owns mul_x weights, a uvw path owns a
    row-major [mul_x, mul_z] tile; path blocks are concatenated in path order."""

    def __init__(self, irreps_x: str, irreps_y: str, irreps_z: str, paths=None,
                 mode: int = UVU, shared_weights: bool = False):
        self.irx = parse_irreps(irreps_x)
        self.iry = parse_irreps(irreps_y)
        self.irz = parse_irreps(irreps_z)
        if paths is None:
            paths = [Path(a, b, c, mode, 1.0) for (a, b, c) in enumerate_paths(self.irx, self.iry, self.irz)]
        paths = sorted(paths, key=lambda q: (q.ix, q.iy, q.iz))
        for q in paths:
            a, b, c = self.irx[q.ix], self.iry[q.iy], self.irz[q.iz]
            if not path_allowed(a, b, c):
                raise ValueError(f"path {q} violates the triangle or parity rule")
            if b.mul != 1:
                raise ValueError("y multiplicity must be 1")
            if q.mode == UVU and a.mul != c.mul:
                raise ValueError("uvu needs mul_x == mul_z")
        self.paths: List[Path] = paths
        self.shared_weights = shared_weights
        self.offx, self.offy, self.offz = offsets(self.irx), offsets(self.iry), offsets(self.irz)
        self.w_off = [0]
        for q in paths:
            n = self.irx[q.ix].mul * (1 if q.mode == UVU else self.irz[q.iz].mul)
            self.w_off.append(self.w_off[-1] + n)

    @property
    def dim_x(self): return self.offx[-1]
    @property
    def dim_y(self): return self.offy[-1]
    @property
    def dim_z(self): return self.offz[-1]
    @property
    def n_w(self): return self.w_off[-1]

    def ls(self, q: Path):
        return self.irx[q.ix].l, self.iry[q.iy].l, self.irz[q.iz].l
