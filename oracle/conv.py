"""Graph convolution built on the CG tensor product (oracle side).

Paper Eq. 4: z_j = sum over edges e = (j, k) entering node j of TP(P, x_k, y_e, W_e).
Evaluated here exactly as the paper describes the unfused formulation (Sec. 3.5): gather
the sender rows of x, run the batched tensor product, scatter-sum by receiver.  The
gradients are the adjoint: g_z is gathered by receiver, the batched backward is run, and
g_x is scatter-summed by sender; g_y and g_W stay per edge.  The second-order pass is the paper's
seven-dispatch combination (Sec. 3.4) applied to the convolution, which is trilinear in
(x_nodes, y_edges, W_edges) like the product itself.

Graph convention: edges are stored in CSR order by receiver; `row_ptr[j]:row_ptr[j+1]` are
the edges entering node j and `col[e]` is the sender of edge e.  The transpose permutation
(needed by a fused backward, Sec. 3.5) lists CSR positions grouped by sender.

Test infrastructure only.
"""
from __future__ import annotations

import numpy as np

from . import tp
from .irreps import TPSpec


def csr_from_coo(recv, send, n_nodes: int):
    """Stable sort of COO edges by (receiver, sender, original index).

    Returns int64 arrays (row_ptr[V+1], col[E], perm[E], t_row_ptr[V+1], t_perm[E]):
      perm[e]      original index of the edge at CSR position e
      col[e]       sender of that edge
      t_perm[q]    CSR position of the q-th edge when CSR positions are stably re-sorted by
                   sender (ties keep CSR order, i.e. ascending receiver)
      t_row_ptr[k] number of edges whose sender is < k
    """
    recv = np.asarray(recv, dtype=np.int64)
    send = np.asarray(send, dtype=np.int64)
    E = recv.shape[0]
    perm = np.lexsort((np.arange(E), send, recv)).astype(np.int64)
    col = send[perm]
    row_ptr = np.zeros(n_nodes + 1, dtype=np.int64)
    np.add.at(row_ptr, recv + 1, 1)
    row_ptr = np.cumsum(row_ptr)
    t_perm = np.argsort(col, kind="stable").astype(np.int64)
    t_row_ptr = np.zeros(n_nodes + 1, dtype=np.int64)
    np.add.at(t_row_ptr, send + 1, 1)
    t_row_ptr = np.cumsum(t_row_ptr)
    return row_ptr, col, perm, t_row_ptr, t_perm


def rows_of_edges(row_ptr) -> np.ndarray:
    """Receiver of every CSR position."""
    row_ptr = np.asarray(row_ptr)
    return np.repeat(np.arange(row_ptr.shape[0] - 1, dtype=np.int64), np.diff(row_ptr))


def forward(spec: TPSpec, x_nodes, y_edges, W_edges, row_ptr, col) -> np.ndarray:
    x_nodes = np.asarray(x_nodes, dtype=np.float64)
    V = np.asarray(row_ptr).shape[0] - 1
    ze = tp.forward(spec, x_nodes[np.asarray(col)], y_edges, W_edges)   # one TP per edge
    z = np.zeros((V, spec.dim_z))
    np.add.at(z, rows_of_edges(row_ptr), ze)                             # sum over N(j)
    return z


def backward(spec: TPSpec, x_nodes, y_edges, W_edges, gz_nodes, row_ptr, col):
    """Returns (g_x [V, dim_x], g_y [E, dim_y], g_W [E, n_w])."""
    x_nodes = np.asarray(x_nodes, dtype=np.float64)
    gz_nodes = np.asarray(gz_nodes, dtype=np.float64)
    col = np.asarray(col)
    gxe, gy, gW = tp.backward(spec, x_nodes[col], y_edges, W_edges, gz_nodes[rows_of_edges(row_ptr)])
    gx = np.zeros_like(x_nodes)
    np.add.at(gx, col, gxe)
    return gx, gy, gW


def double_backward(spec: TPSpec, x_nodes, y_edges, W_edges, gz_nodes, La_nodes, Lb_edges, LC_edges, row_ptr, col):
    """Second-order pass of the convolution (paper Sec. 3.4 with the convolution in place of the
    product).  With (a, b, C) = backward(x, y, W, gz) and a scalar L(a, b, C): takes La = dL/da
    [V, dim_x], Lb = dL/db [E, dim_y], LC = dL/dC [E, n_w] and returns
    (dL/dx [V, dim_x], dL/dy [E, dim_y], dL/dW [E, n_w], dL/dgz [V, dim_z]) as the seven dispatches
    op1 .. op7 of the forward and backward functions, combined as the paper states."""
    f = lambda a, b, c: forward(spec, a, b, c, row_ptr, col)
    g = lambda a, b, c: backward(spec, a, b, c, gz_nodes, row_ptr, col)
    op1 = g(La_nodes, Lb_edges, W_edges)
    op2 = g(x_nodes, y_edges, LC_edges)
    op3 = f(La_nodes, y_edges, W_edges)
    op4 = g(La_nodes, y_edges, W_edges)
    op5 = g(x_nodes, Lb_edges, W_edges)
    op6 = f(x_nodes, Lb_edges, W_edges)
    op7 = f(x_nodes, y_edges, LC_edges)
    return op1[0] + op2[0], op1[1] + op2[1], op4[2] + op5[2], op3 + op6 + op7
