"""The CG tensor product TP(P, x, y, W) and its gradients, as plain definitions (oracle).

Forward follows paper Eq. 1 specialised by the structure of Sec. 2.3 / Alg. 2: per path
(x segment, y segment, z segment) the block C = P^(l1,l2,l3) is contracted with the
rows X[u, :] of the x segment and with y, then multiplied by the path's weight tile
(diagonal "uvu" = kernel B, dense "uvw" = kernel C) and added into the z segment.
Backward is the three product-rule formulas of Sec. 3.3.  Double backward is the linear
combination of seven forward / backward calls of Sec. 3.4.

Shapes: x [B, dim_x], y [B, dim_y], W [B, n_w] (or [n_w] when shared), z [B, dim_z],
all fp64.  Inside a segment the index is u*(2l+1)+m.

`dense_reference` assembles the full tensor P and the structured matrix W explicitly and
evaluates einsum("ijk,i,j,kk'->k'") for one sample; it exists to pin `forward`.

Test infrastructure only; no blocking, fusion or reordering beyond the definitions.
"""
from __future__ import annotations

import numpy as np

from .cg import cg_block
from .irreps import TPSpec, UVU, UVW


def _seg(a: np.ndarray, off: int, mul: int, l: int) -> np.ndarray:
    return a[:, off:off + mul * (2 * l + 1)].reshape(a.shape[0], mul, 2 * l + 1)


def _weights(spec: TPSpec, W: np.ndarray, p: int, B: int) -> np.ndarray:
    """Weight tile of path p: [B or 1, mul_x] (uvu) or [B or 1, mul_x, mul_z] (uvw)."""
    q = spec.paths[p]
    w = W[..., spec.w_off[p]:spec.w_off[p + 1]]
    if w.ndim == 1:
        w = w[None, :]
    if q.mode == UVW:
        w = w.reshape(w.shape[0], spec.irx[q.ix].mul, spec.irz[q.iz].mul)
    return w


def forward(spec: TPSpec, x, y, W) -> np.ndarray:
    x, y, W = (np.asarray(a, dtype=np.float64) for a in (x, y, W))
    B = x.shape[0]
    z = np.zeros((B, spec.dim_z))
    for p, q in enumerate(spec.paths):
        l1, l2, l3 = spec.ls(q)
        C = cg_block(l1, l2, l3)
        X = _seg(x, spec.offx[q.ix], spec.irx[q.ix].mul, l1)          # [B, u, i]
        Y = y[:, spec.offy[q.iy]:spec.offy[q.iy] + 2 * l2 + 1]          # [B, j]
        Zp = np.einsum("ijk,bui,bj->buk", C, X, Y)                      # Alg. 2 inner loop
        w = _weights(spec, W, p, B)
        Zs = _seg(z, spec.offz[q.iz], spec.irz[q.iz].mul, l3)           # view into z
        if q.mode == UVU:
            Zs += q.coeff * w[:, :, None] * Zp
        else:
            Zs += q.coeff * np.einsum("buw,buk->bwk", np.broadcast_to(w, (B,) + w.shape[1:]), Zp)
    return z


def backward(spec: TPSpec, x, y, W, gz):
    """Returns (g_x, g_y, g_W) = gradients of E w.r.t. x, y, W given g_z = dE/dz.
    With shared weights g_W is summed over the batch."""
    x, y, W, gz = (np.asarray(a, dtype=np.float64) for a in (x, y, W, gz))
    B = x.shape[0]
    gx = np.zeros_like(x)
    gy = np.zeros_like(y)
    gW = np.zeros((B, spec.n_w))
    for p, q in enumerate(spec.paths):
        l1, l2, l3 = spec.ls(q)
        C = cg_block(l1, l2, l3)
        mx, mz = spec.irx[q.ix].mul, spec.irz[q.iz].mul
        X = _seg(x, spec.offx[q.ix], mx, l1)
        Y = y[:, spec.offy[q.iy]:spec.offy[q.iy] + 2 * l2 + 1]
        G = _seg(gz, spec.offz[q.iz], mz, l3)                           # [B, w, k]
        w = _weights(spec, W, p, B)
        # (W^T g_z) restricted to this path: G'[b, u, k]
        if q.mode == UVU:
            Gp = q.coeff * w[:, :, None] * G
        else:
            Gp = q.coeff * np.einsum("buw,bwk->buk", np.broadcast_to(w, (B,) + w.shape[1:]), G)
        _seg(gx, spec.offx[q.ix], mx, l1)[...] += np.einsum("ijk,bj,buk->bui", C, Y, Gp)
        gy[:, spec.offy[q.iy]:spec.offy[q.iy] + 2 * l2 + 1] += np.einsum("ijk,bui,buk->bj", C, X, Gp)
        Zp = np.einsum("ijk,bui,bj->buk", C, X, Y)
        if q.mode == UVU:
            gW[:, spec.w_off[p]:spec.w_off[p + 1]] = q.coeff * np.einsum("buk,buk->bu", G, Zp)
        else:
            gW[:, spec.w_off[p]:spec.w_off[p + 1]] = q.coeff * np.einsum("buk,bwk->buw", Zp, G).reshape(B, -1)
    if spec.shared_weights:
        gW = gW.sum(axis=0)
    return gx, gy, gW


def double_backward(spec: TPSpec, x, y, W, gz, La, Lb, LC):
    """Second-order pass of paper Sec. 3.4.  With (a, b, C) = backward(x, y, W, gz) and a scalar
    L(a, b, C), takes La = dL/da [B, dim_x], Lb = dL/db [B, dim_y], LC = dL/dC (shape of W) and
    returns (dL/dx, dL/dy, dL/dW, dL/dgz), as the paper's seven dispatches (op1 .. op7) of the
    forward and backward functions, combined as it states.  Per-sample weights only."""
    if spec.shared_weights:
        raise ValueError("double_backward: per-sample weights only")
    op1 = backward(spec, La, Lb, W, gz)
    op2 = backward(spec, x, y, LC, gz)
    op3 = forward(spec, La, y, W)
    op4 = backward(spec, La, y, W, gz)
    op5 = backward(spec, x, Lb, W, gz)
    op6 = forward(spec, x, Lb, W)
    op7 = forward(spec, x, y, LC)
    return op1[0] + op2[0], op1[1] + op2[1], op4[2] + op5[2], op3 + op6 + op7


def dense_reference(spec: TPSpec, x1, y1, W1) -> np.ndarray:
    """One sample of Eq. 1 with the sparse tensor and the weight matrix written out in full:
    P in R^{dim_x x dim_y x K}, W in R^{K x dim_z}, K = sum over paths of mul_x*(2 l3+1);
    z = einsum("ijk,i,j,kl->l").  Explicit Python loops, tiny inputs only."""
    K = sum(spec.irx[q.ix].mul * (2 * spec.ls(q)[2] + 1) for q in spec.paths)
    P = np.zeros((spec.dim_x, spec.dim_y, K))
    Wm = np.zeros((K, spec.dim_z))
    base = 0
    for p, q in enumerate(spec.paths):
        l1, l2, l3 = spec.ls(q)
        C = cg_block(l1, l2, l3)
        mx, mz = spec.irx[q.ix].mul, spec.irz[q.iz].mul
        wp = W1[spec.w_off[p]:spec.w_off[p + 1]]
        for u in range(mx):
            for k in range(2 * l3 + 1):
                row = base + u * (2 * l3 + 1) + k
                for i in range(2 * l1 + 1):
                    for j in range(2 * l2 + 1):
                        P[spec.offx[q.ix] + u * (2 * l1 + 1) + i, spec.offy[q.iy] + j, row] = C[i, j, k]
                if q.mode == UVU:
                    Wm[row, spec.offz[q.iz] + u * (2 * l3 + 1) + k] = q.coeff * wp[u]
                else:
                    for w in range(mz):
                        Wm[row, spec.offz[q.iz] + w * (2 * l3 + 1) + k] = q.coeff * wp[u * mz + w]
        base += mx * (2 * l3 + 1)
    return np.einsum("ijk,i,j,kl->l", P, x1, y1, Wm)


def flops_forward(spec: TPSpec) -> int:
    """Nonzero-FLOP count per sample: 2*nnz per channel for the contraction plus the
    weight multiply (2*(2 l3+1) per channel for uvu, 2*mul_x*mul_z*(2 l3+1) for uvw)."""
    tot = 0
    for q in spec.paths:
        l1, l2, l3 = spec.ls(q)
        nnz = int(np.count_nonzero(cg_block(l1, l2, l3)))
        mx, mz = spec.irx[q.ix].mul, spec.irz[q.iz].mul
        tot += 2 * nnz * mx
        tot += 2 * (2 * l3 + 1) * (mx if q.mode == UVU else mx * mz)
    return tot
