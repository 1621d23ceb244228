"""Pins for oracle/conv.py: CSR artefacts against their defining properties and a pure-Python
sort; the convolution of paper Eq. 4 against a node-by-node loop over single-sample tensor
products; its backward against the adjoint identity and finite differences; its second-order pass
against central differences through the backward (exact up to rounding: the scalar is linear in
every single entry) and against the batched second-order pass on a graph without shared nodes."""
import numpy as np

from oracle import conv, tp
from oracle.irreps import TPSpec
from paper_2501_13986_amd import synth

RNG = np.random.default_rng(77)


def small_graph(V=23, deg=6.0, seed=5):
    # small boxes violate L > 2r; draw a plain random multigraph-free edge set instead
    rng = np.random.default_rng(seed)
    E = int(V * deg)
    pairs = set()
    while len(pairs) < E:
        r, s = rng.integers(0, V, 2)
        if r != s and r != 3:           # node 3 receives nothing: an empty CSR row
            pairs.add((int(r), int(s)))
    pairs = list(pairs)
    rng.shuffle(pairs)
    recv = np.array([p[0] for p in pairs]); send = np.array([p[1] for p in pairs])
    return recv, send


def test_csr_properties_and_python_sort():
    V = 23
    recv, send = small_graph(V)
    E = recv.shape[0]
    row_ptr, col, perm, t_row_ptr, t_perm = conv.csr_from_coo(recv, send, V)
    assert all(a.dtype == np.int64 for a in (row_ptr, col, perm, t_row_ptr, t_perm))
    ref = sorted(range(E), key=lambda e: (recv[e], send[e], e))
    assert perm.tolist() == ref
    assert col.tolist() == [int(send[e]) for e in ref]
    assert row_ptr[0] == 0 and row_ptr[-1] == E and np.all(np.diff(row_ptr) >= 0)
    assert row_ptr[4] - row_ptr[3] == 0
    for j in range(V):
        assert np.all(recv[perm[row_ptr[j]:row_ptr[j + 1]]] == j)
        assert np.all(np.diff(col[row_ptr[j]:row_ptr[j + 1]]) >= 0)
    assert sorted(t_perm.tolist()) == list(range(E))
    rows = conv.rows_of_edges(row_ptr)
    tref = sorted(range(E), key=lambda e: (col[e], e))
    assert t_perm.tolist() == tref
    for k in range(V):
        seg = t_perm[t_row_ptr[k]:t_row_ptr[k + 1]]
        assert np.all(col[seg] == k)
        assert np.all(np.diff(rows[seg]) >= 0)
    assert t_row_ptr[-1] == E


def test_duplicate_edges_keep_original_order():
    recv = np.array([1, 0, 1, 1, 0]); send = np.array([2, 1, 2, 0, 1])
    row_ptr, col, perm, t_row_ptr, t_perm = conv.csr_from_coo(recv, send, 3)
    assert perm.tolist() == [1, 4, 3, 0, 2]
    assert row_ptr.tolist() == [0, 2, 5, 5]
    assert col.tolist() == [1, 1, 0, 2, 2]
    assert t_perm.tolist() == [2, 0, 1, 3, 4]
    assert t_row_ptr.tolist() == [0, 1, 3, 5]


def test_conv_forward_is_sum_over_neighbours():
    spec = TPSpec("2x0e+2x1o+2x2e", "1x0e+1x1o+1x2e", "2x0e+2x1o+2x2e+2x3o")
    V = 23
    recv, send = small_graph(V)
    row_ptr, col, perm, _, _ = conv.csr_from_coo(recv, send, V)
    E = col.shape[0]
    x = RNG.normal(size=(V, spec.dim_x)); y = RNG.normal(size=(E, spec.dim_y)); W = RNG.normal(size=(E, spec.n_w))
    z = conv.forward(spec, x, y, W, row_ptr, col)
    for j in range(V):
        acc = np.zeros(spec.dim_z)
        for e in range(row_ptr[j], row_ptr[j + 1]):
            acc += tp.dense_reference(spec, x[col[e]], y[e], W[e])
        assert np.abs(z[j] - acc).max() < 1e-12
    assert np.all(z[3] == 0.0)


def test_conv_backward_adjoint_and_fd():
    spec = TPSpec("2x0e+2x1o", "1x0e+1x1o+1x2e", "2x0e+2x1o+2x2e+2x1e")
    V = 11
    recv, send = small_graph(V, 4.0, seed=9)
    row_ptr, col, perm, _, _ = conv.csr_from_coo(recv, send, V)
    E = col.shape[0]
    x = RNG.normal(size=(V, spec.dim_x)); y = RNG.normal(size=(E, spec.dim_y)); W = RNG.normal(size=(E, spec.n_w))
    gz = RNG.normal(size=(V, spec.dim_z))
    gx, gy, gW = conv.backward(spec, x, y, W, gz, row_ptr, col)
    dx, dy, dW = RNG.normal(size=x.shape), RNG.normal(size=y.shape), RNG.normal(size=W.shape)
    f = lambda a, b, c: conv.forward(spec, a, b, c, row_ptr, col)
    assert abs(np.sum(gz * f(dx, y, W)) - np.sum(gx * dx)) < 1e-10
    assert abs(np.sum(gz * f(x, dy, W)) - np.sum(gy * dy)) < 1e-10
    assert abs(np.sum(gz * f(x, y, dW)) - np.sum(gW * dW)) < 1e-10
    h = 1e-5
    for arr, grad in ((x, gx), (y, gy), (W, gW)):
        flat = arr.reshape(-1)
        for t in RNG.choice(flat.size, size=8, replace=False):
            old = flat[t]
            flat[t] = old + h; ep = np.sum(gz * f(x, y, W))
            flat[t] = old - h; em = np.sum(gz * f(x, y, W))
            flat[t] = old
            fd = (ep - em) / (2 * h)
            assert abs(fd - grad.reshape(-1)[t]) < 1e-7 * max(1.0, abs(fd))


def test_conv_on_periodic_graph_matches_unfused_by_hand():
    spec = TPSpec("2x0e+2x1o", "1x0e+1x1o", "2x0e+2x1o")
    recv, send, unit = synth.periodic_graph(1, 600, 8.0)
    V = 600
    row_ptr, col, perm, t_row_ptr, t_perm = conv.csr_from_coo(recv, send, V)
    E = col.shape[0]
    y = synth.sh_edge_attr(unit[perm], 1)
    x = RNG.normal(size=(V, spec.dim_x)); W = RNG.normal(size=(E, spec.n_w))
    z = conv.forward(spec, x, y, W, row_ptr, col)
    ze = tp.forward(spec, x[send[perm]], y, W)
    ref = np.zeros_like(z)
    for e in range(E):
        ref[recv[perm[e]]] += ze[e]
    assert np.abs(z - ref).max() < 1e-12


def test_conv_double_backward_finite_differences():
    spec = TPSpec("2x0e+2x1o", "1x0e+1x1o+1x2e", "2x0e+2x1o+2x2e+2x1e")
    V = 9
    recv, send = small_graph(V, 3.0, seed=19)
    row_ptr, col, perm, _, _ = conv.csr_from_coo(recv, send, V)
    E = col.shape[0]
    x = RNG.normal(size=(V, spec.dim_x)); y = RNG.normal(size=(E, spec.dim_y)); W = RNG.normal(size=(E, spec.n_w))
    gz = RNG.normal(size=(V, spec.dim_z))
    La, Lb, LC = RNG.normal(size=x.shape), RNG.normal(size=y.shape), RNG.normal(size=W.shape)
    grads = conv.double_backward(spec, x, y, W, gz, La, Lb, LC, row_ptr, col)

    def L(x_, y_, W_, gz_):
        a, b, C = conv.backward(spec, x_, y_, W_, gz_, row_ptr, col)
        return float(np.sum(La * a) + np.sum(Lb * b) + np.sum(LC * C))
    args = [x, y, W, gz]
    h = 1e-3
    for which, (arr, grad) in enumerate(zip(args, grads)):
        assert grad.shape == arr.shape
        flat = arr.reshape(-1)
        for t in RNG.choice(flat.size, size=min(flat.size, 10), replace=False):
            old = flat[t]
            flat[t] = old + h; lp = L(*args)
            flat[t] = old - h; lm = L(*args)
            flat[t] = old
            fd = (lp - lm) / (2 * h)
            assert abs(fd - grad.reshape(-1)[t]) < 1e-9 * max(1.0, abs(fd)), (which, t)
        assert np.abs(grad).max() > 1e-3


def test_conv_double_backward_reduces_to_the_batched_one_on_disjoint_edges():
    """Every node is the sender or the receiver of exactly one edge: the convolution is then the batched
    product on relabelled rows, and so is its second-order pass."""
    spec = TPSpec("2x0e+2x1o", "1x0e+1x1o+1x2e", "2x0e+2x1o+2x2e+2x1e")
    E = 5
    V = 2 * E
    recv = np.arange(E, dtype=np.int64)           # edge e: node E+e -> node e
    send = np.arange(E, 2 * E, dtype=np.int64)
    row_ptr, col, perm, _, _ = conv.csr_from_coo(recv, send, V)
    assert np.array_equal(perm, np.arange(E))
    x = RNG.normal(size=(V, spec.dim_x)); y = RNG.normal(size=(E, spec.dim_y)); W = RNG.normal(size=(E, spec.n_w))
    gz = RNG.normal(size=(V, spec.dim_z))
    La, Lb, LC = RNG.normal(size=x.shape), RNG.normal(size=y.shape), RNG.normal(size=W.shape)
    Lx, Ly, LW, Lgz = conv.double_backward(spec, x, y, W, gz, La, Lb, LC, row_ptr, col)
    bx, by, bW, bgz = tp.double_backward(spec, x[E:], y, W, gz[:E], La[E:], Lb, LC)
    assert np.abs(Lx[E:] - bx).max() < 1e-12 and np.abs(Lx[:E]).max() == 0.0       # receivers send nothing
    assert np.abs(Ly - by).max() < 1e-12 and np.abs(LW - bW).max() < 1e-12
    assert np.abs(Lgz[:E] - bgz).max() < 1e-12 and np.abs(Lgz[E:]).max() == 0.0    # senders receive nothing
