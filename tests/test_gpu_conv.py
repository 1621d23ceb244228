"""GPU parity of the fused tensor product + graph convolution (forward, backward) and of the
CSR construction against the CPU oracle, through the C ABI.  Integer outputs must be bit-exact."""
import numpy as np
import pytest

from oracle import conv as oconv
from oracle.irreps import TPSpec
from paper_2501_13986_amd import synth
from tests._util import assert_close, memo

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _b():
    from paper_2501_13986_amd import binding
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


SPECS = {
    "mace": (synth.MACE_X, synth.MACE_Y, synth.MACE_Z),
    "small": ("4x0e+4x1o+4x2e", "1x0e+1x1o+1x2e", "4x0e+4x1o+4x2e+4x3o"),
    "mul96": ("96x0e+96x1o", "1x0e+1x1o", "96x0e+96x1o+96x1e"),
    "mul192": ("192x0e+192x1o", "1x0e+1x1o", "192x0e+192x1o"),
    "mul1": ("1x0e+1x1o+1x2e", "1x0e+1x1o+1x2e", "1x0e+1x1o+1x2e+1x3o"),   # 64 edge-range workers per wave
    "many_paths": (synth.MANY_X, synth.MANY_Y, synth.MANY_X),     # 68 paths: non-default schedules
}


def random_graph(seed, V, E, empty_rows=()):
    rng = np.random.default_rng(seed)
    recv = rng.integers(0, V, E)
    send = rng.integers(0, V, E)
    for r in empty_rows:
        recv[recv == r] = (r + 1) % V
        send[send == r] = (r + 1) % V
    return recv.astype(np.int64), send.astype(np.int64)


GRAPHS = {
    # name -> (V, E, empty rows): skewed shapes exercise rows split over many waves, rows shorter
    # than a chunk, empty rows at the start / middle / end, fewer edges than waves
    "typical": (200, 200 * 12, ()),
    "few_long_rows": (3, 2400, ()),
    "one_row": (1, 777, ()),
    "many_empty": (500, 40, ()),
    "empty_ends": (64, 2000, (0, 1, 30, 31, 62, 63)),
    "single_edge": (5, 1, ()),
}


def build(spec_name, graph_name, prec, seed=0):
    b = _b()
    ix, iy, iz = SPECS[spec_name]
    spec = TPSpec(ix, iy, iz)
    plan = b.Plan(ix, iy, iz, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0)
    V, E, empty = GRAPHS[graph_name]
    recv, send = random_graph(seed, V, E, empty)
    row_ptr, col, perm, t_row_ptr, t_perm = oconv.csr_from_coo(recv, send, V)
    npdt = np.float64 if prec == "f64" else np.float32
    x = synth.normal(seed + 1, (V, spec.dim_x)).astype(npdt)
    y = synth.normal(seed + 2, (E, spec.dim_y)).astype(npdt)
    W = synth.normal(seed + 3, (E, spec.n_w)).astype(npdt)
    gz = synth.normal(seed + 4, (V, spec.dim_z)).astype(npdt)
    return b, spec, plan, (x, y, W, gz), (row_ptr, col, perm, t_row_ptr, t_perm), (V, E)


@pytest.mark.parametrize("prec", ["f64", "f32"])
@pytest.mark.parametrize("graph", list(GRAPHS))
@pytest.mark.parametrize("spec_name", ["small", "mace"])
def test_conv_forward_parity(spec_name, graph, prec):
    b, spec, plan, (x, y, W, gz), (row_ptr, col, perm, t_row_ptr, t_perm), (V, E) = build(spec_name, graph, prec)
    print(f"spec={spec_name} graph={graph} prec={prec} V={V} E={E} entry=conv_forward", flush=True)
    tdt = torch.float64 if prec == "f64" else torch.float32
    z = torch.full((V, spec.dim_z), float("nan"), dtype=tdt, device="cuda")
    args = (plan, dev(x), dev(y), dev(W), z, dev(row_ptr), dev(col))
    b.conv_forward(*args)
    torch.cuda.synchronize()
    first = z.clone()
    ref = memo(oconv.forward, spec, x, y, W, row_ptr, col)
    assert_close(first.cpu().numpy(), ref, prec, "conv forward")
    empty = np.flatnonzero(np.diff(row_ptr) == 0)
    assert torch.all(first[torch.from_numpy(empty).cuda()] == 0)
    # deterministic: a second run is bit-identical
    z.fill_(float("nan"))
    b.conv_forward(*args)
    torch.cuda.synchronize()
    assert torch.equal(first, z)


@pytest.mark.parametrize("prec", ["f64", "f32"])
@pytest.mark.parametrize("graph", list(GRAPHS))
@pytest.mark.parametrize("spec_name", ["small", "mace"])
def test_conv_backward_parity(spec_name, graph, prec):
    b, spec, plan, (x, y, W, gz), (row_ptr, col, perm, t_row_ptr, t_perm), (V, E) = build(spec_name, graph, prec, seed=20)
    print(f"spec={spec_name} graph={graph} prec={prec} V={V} E={E} entry=conv_backward", flush=True)
    tdt = torch.float64 if prec == "f64" else torch.float32
    gx = torch.full((V, spec.dim_x), float("nan"), dtype=tdt, device="cuda")
    gy = torch.full((E, spec.dim_y), float("nan"), dtype=tdt, device="cuda")
    gW = torch.full((E, spec.n_w), float("nan"), dtype=tdt, device="cuda")
    args = (plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW, dev(row_ptr), dev(col), dev(t_row_ptr), dev(t_perm))
    b.conv_backward(*args)
    torch.cuda.synchronize()
    rx, ry, rW = memo(oconv.backward, spec, x, y, W, gz, row_ptr, col)
    assert_close(gx.cpu().numpy(), rx, prec, "conv gx")
    assert_close(gy.cpu().numpy(), ry, prec, "conv gy")
    assert_close(gW.cpu().numpy(), rW, prec, "conv gW")
    first = (gx.clone(), gy.clone(), gW.clone())
    for t in (gx, gy, gW):
        t.fill_(float("nan"))
    b.conv_backward(*args)
    torch.cuda.synchronize()
    assert all(torch.equal(a, c) for a, c in zip(first, (gx, gy, gW)))


@pytest.mark.parametrize("spec_name", ["mul96", "mul192", "many_paths", "mul1"])
def test_conv_channel_passes(spec_name):
    b, spec, plan, (x, y, W, gz), (row_ptr, col, perm, t_row_ptr, t_perm), (V, E) = build(spec_name, "typical", "f64", seed=3)
    print(f"spec={spec_name} graph=typical entry=conv_forward/conv_backward", flush=True)
    z = torch.full((V, spec.dim_z), float("nan"), dtype=torch.float64, device="cuda")
    b.conv_forward(plan, dev(x), dev(y), dev(W), z, dev(row_ptr), dev(col))
    gx = torch.full((V, spec.dim_x), float("nan"), dtype=torch.float64, device="cuda")
    gy = torch.full((E, spec.dim_y), float("nan"), dtype=torch.float64, device="cuda")
    gW = torch.full((E, spec.n_w), float("nan"), dtype=torch.float64, device="cuda")
    b.conv_backward(plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW, dev(row_ptr), dev(col), dev(t_row_ptr), dev(t_perm))
    torch.cuda.synchronize()
    assert_close(z.cpu().numpy(), memo(oconv.forward, spec, x, y, W, row_ptr, col), "f64", "z")
    rx, ry, rW = memo(oconv.backward, spec, x, y, W, gz, row_ptr, col)
    assert_close(gx.cpu().numpy(), rx, "f64", "gx")
    assert_close(gy.cpu().numpy(), ry, "f64", "gy")
    assert_close(gW.cpu().numpy(), rW, "f64", "gW")


def test_conv_no_edges_zero_fills():
    b = _b()
    plan = b.Plan(*SPECS["small"], dtype=b.CGTP_F64, device=0)
    V = 7
    z = torch.full((V, plan.dim_z), 3.0, dtype=torch.float64, device="cuda")
    e0 = torch.zeros((0, 1), dtype=torch.float64, device="cuda")
    row_ptr = torch.zeros(V + 1, dtype=torch.int64, device="cuda")
    st = b.lib().conv_forward(plan._h, None, None, None, z.data_ptr(), V, 0, row_ptr.data_ptr(), None, None)
    torch.cuda.synchronize()
    assert st == 0 and torch.all(z == 0)


# 65 536 nodes is the last size whose keys recv * V + send fit 32 bits; 70 001 takes the 64-bit keys
@pytest.mark.parametrize("V,E,seed", [(23, 140, 0), (1000, 33000, 1), (5, 0, 2), (4, 9, 3), (65536, 50000, 4), (70001, 50000, 5)])
def test_csr_from_coo_bit_exact(V, E, seed):
    b = _b()
    print(f"V={V} E={E} entry=cgtp_csr_from_coo", flush=True)
    rng = np.random.default_rng(seed)
    recv = rng.integers(0, V, E).astype(np.int64)
    send = rng.integers(0, V, E).astype(np.int64)
    if E >= 9:
        recv[:4] = recv[4:8]        # duplicates: ties must keep the original order
        send[:4] = send[4:8]
    ref = oconv.csr_from_coo(recv, send, V)
    got = b.cgtp_csr_from_coo(dev(recv), dev(send), V)
    names = ("row_ptr", "col", "perm", "t_row_ptr", "t_perm")
    for n, g, r in zip(names, got, ref):
        assert g.dtype == torch.int64
        assert np.array_equal(g.cpu().numpy(), r), n


@pytest.mark.parametrize("V,E,seed", [(1, 1, 0), (7, 50, 1), (300, 7000, 2), (5000, 160001, 3), (50, 0, 4), (65536, 40000, 5), (70001, 40000, 6)])
def test_csr_from_coo_async_bit_exact(V, E, seed):
    """The asynchronous variant on a caller-owned workspace: the same arrays bit for bit, with and without the transpose
    (whose outputs must then stay untouched), the range-check flag on the device, and refusal of a short workspace."""
    b = _b()
    print(f"V={V} E={E} entry=cgtp_csr_from_coo_async", flush=True)
    rng = np.random.default_rng(seed)
    recv = rng.integers(0, V, E).astype(np.int64)
    send = rng.integers(0, V, E).astype(np.int64)
    if E >= 9:
        recv[:4] = recv[4:8]
        send[:4] = send[4:8]
    ref = oconv.csr_from_coo(recv, send, V)
    need = b.cgtp_csr_workspace_bytes(E, V)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    flag = torch.full((1,), 7, dtype=torch.int32, device="cuda")
    mk = lambda: (torch.full((V + 1,), -5, dtype=torch.int64, device="cuda"), torch.full((E,), -5, dtype=torch.int64, device="cuda"),
                  torch.full((E,), -5, dtype=torch.int64, device="cuda"), torch.full((V + 1,), -5, dtype=torch.int64, device="cuda"),
                  torch.full((E,), -5, dtype=torch.int64, device="cuda"))
    d_recv, d_send = dev(recv) if E else torch.zeros(1, dtype=torch.int64, device="cuda")[:0], dev(send) if E else torch.zeros(1, dtype=torch.int64, device="cuda")[:0]
    got = b.cgtp_csr_from_coo_async(d_recv, d_send, V, mk(), ws, flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    for n, g, r in zip(("row_ptr", "col", "perm", "t_row_ptr", "t_perm"), got, ref):
        assert np.array_equal(g.cpu().numpy(), r), n
    fwd_only = b.cgtp_csr_from_coo_async(d_recv, d_send, V, mk(), ws, None, transpose=False)
    torch.cuda.synchronize()
    for n, g, r in zip(("row_ptr", "col", "perm"), fwd_only, ref):
        assert np.array_equal(g.cpu().numpy(), r), n
    assert torch.all(fwd_only[3] == -5) and torch.all(fwd_only[4] == -5)
    if E > 0:
        with pytest.raises(b.CgtpError):
            b.cgtp_csr_from_coo_async(d_recv, d_send, V, mk(), ws[: need - 256], flag)
        bad = recv.copy(); bad[E // 2] = V           # one receiver out of range: flagged on the device, no exception
        b.cgtp_csr_from_coo_async(dev(bad), d_send, V, mk(), ws, flag)
        torch.cuda.synchronize()
        assert int(flag.item()) == 1


def test_csr_rejects_out_of_range_indices():
    b = _b()
    recv = dev(np.array([0, 1, 9], dtype=np.int64)); send = dev(np.array([1, 0, 1], dtype=np.int64))
    with pytest.raises(b.CgtpError):
        b.cgtp_csr_from_coo(recv, send, 3)


def test_conv_on_periodic_box_with_device_csr():
    """End to end at a reduced size of the benchmark recipe: periodic box, harmonics of the
    edge directions, CSR built on the device, convolution forward and backward."""
    b = _b()
    V, deg = 300, 24.0
    recv, send, unit = synth.periodic_graph(4, V, deg)
    spec = TPSpec(*SPECS["mace"])
    plan = b.Plan(*SPECS["mace"], dtype=b.CGTP_F32, device=0)
    row_ptr, col, perm, t_row_ptr, t_perm = b.cgtp_csr_from_coo(dev(recv), dev(send), V)
    ref_csr = oconv.csr_from_coo(recv, send, V)
    for g, r in zip((row_ptr, col, perm, t_row_ptr, t_perm), ref_csr):
        assert np.array_equal(g.cpu().numpy(), r)
    E = recv.shape[0]
    print(f"V={V} E={E} entry=conv_forward/backward periodic box", flush=True)
    y = synth.sh_edge_attr(unit[ref_csr[2]], 3).astype(np.float32)
    x = synth.normal(1, (V, spec.dim_x)).astype(np.float32)
    W = synth.normal(2, (E, spec.n_w)).astype(np.float32)
    gz = synth.normal(3, (V, spec.dim_z)).astype(np.float32)
    z = torch.empty((V, spec.dim_z), dtype=torch.float32, device="cuda")
    b.conv_forward(plan, dev(x), dev(y), dev(W), z, row_ptr, col)
    gx = torch.empty((V, spec.dim_x), dtype=torch.float32, device="cuda")
    gy = torch.empty((E, spec.dim_y), dtype=torch.float32, device="cuda")
    gW = torch.empty((E, spec.n_w), dtype=torch.float32, device="cuda")
    b.conv_backward(plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW, row_ptr, col, t_row_ptr, t_perm)
    torch.cuda.synchronize()
    assert_close(z.cpu().numpy(), memo(oconv.forward, spec, x, y, W, ref_csr[0], ref_csr[1]), "f32", "z")
    rx, ry, rW = memo(oconv.backward, spec, x, y, W, gz, ref_csr[0], ref_csr[1])
    assert_close(gx.cpu().numpy(), rx, "f32", "gx")
    assert_close(gy.cpu().numpy(), ry, "f32", "gy")
    assert_close(gW.cpu().numpy(), rW, "f32", "gW")


@pytest.mark.parametrize("prec", ["f64", "f32"])
@pytest.mark.parametrize("graph", ["typical", "few_long_rows", "many_empty", "single_edge"])
@pytest.mark.parametrize("order", ["as_generated", "by_receiver", "by_sender"])
@pytest.mark.parametrize("spec_name", ["small", "mace"])
def test_conv_atomic_unsorted_edges(spec_name, order, graph, prec):
    """Nondeterministic variant: edges in their original (unsorted) order, results equal to the
    oracle's within the tolerance (sum order differs from run to run)."""
    b = _b()
    ix, iy, iz = SPECS[spec_name]
    spec = TPSpec(ix, iy, iz)
    plan = b.Plan(ix, iy, iz, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0)
    V, E, empty = GRAPHS[graph]
    recv, send = random_graph(31, V, E, empty)
    if order != "as_generated":      # long runs of equal receivers (resp. senders) exercise the run-combining path
        o = np.argsort(recv if order == "by_receiver" else send, kind="stable")
        recv, send = recv[o], send[o]
    print(f"spec={spec_name} graph={graph} order={order} prec={prec} V={V} E={E} entry=conv_forward_atomic/conv_backward_atomic", flush=True)
    npdt = np.float64 if prec == "f64" else np.float32
    tdt = torch.float64 if prec == "f64" else torch.float32
    # edge data is drawn in CSR order and scattered to the order the kernels are given (so that the reference
    # is the same for every input order)
    row_ptr, col, perm, _, _ = oconv.csr_from_coo(recv, send, V)
    x = synth.normal(32, (V, spec.dim_x)).astype(npdt)
    y_csr = synth.normal(33, (E, spec.dim_y)).astype(npdt)
    W_csr = synth.normal(34, (E, spec.n_w)).astype(npdt)
    y = np.empty_like(y_csr); y[perm] = y_csr                   # rows in the original edge order
    W = np.empty_like(W_csr); W[perm] = W_csr
    gz = synth.normal(35, (V, spec.dim_z)).astype(npdt)
    z = torch.full((V, spec.dim_z), float("nan"), dtype=tdt, device="cuda")
    gx = torch.full((V, spec.dim_x), float("nan"), dtype=tdt, device="cuda")
    gy = torch.full((E, spec.dim_y), float("nan"), dtype=tdt, device="cuda")
    gW = torch.full((E, spec.n_w), float("nan"), dtype=tdt, device="cuda")
    b.conv_forward_atomic(plan, dev(x), dev(y), dev(W), z, dev(recv), dev(send))
    b.conv_backward_atomic(plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW, dev(recv), dev(send))
    torch.cuda.synchronize()
    # oracle on the sorted graph; map per-edge quantities through perm (original index of each CSR position)
    assert_close(z.cpu().numpy(), memo(oconv.forward, spec, x, y_csr, W_csr, row_ptr, col), prec, "atomic z")
    rx, ry, rW = memo(oconv.backward, spec, x, y_csr, W_csr, gz, row_ptr, col)
    assert_close(gx.cpu().numpy(), rx, prec, "atomic gx")
    assert_close(gy.cpu().numpy()[perm], ry, prec, "atomic gy")
    assert_close(gW.cpu().numpy()[perm], rW, prec, "atomic gW")


@pytest.mark.parametrize("prec", ["f64", "f32"])
@pytest.mark.parametrize("graph", ["typical", "few_long_rows", "many_empty"])
@pytest.mark.parametrize("spec_name", ["small", "mace"])
def test_conv_with_compensated_row_sums(spec_name, graph, prec):
    """Plans created with kahan_conv compute the same convolution (forward, backward, atomic forward)."""
    b = _b()
    ix, iy, iz = SPECS[spec_name]
    spec = TPSpec(ix, iy, iz)
    plan = b.Plan(ix, iy, iz, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0, kahan_conv=True)
    V, E, empty = GRAPHS[graph]
    recv, send = random_graph(41, V, E, empty)
    print(f"spec={spec_name} graph={graph} prec={prec} kahan entry=conv_forward/conv_backward/conv_forward_atomic", flush=True)
    npdt = np.float64 if prec == "f64" else np.float32
    tdt = torch.float64 if prec == "f64" else torch.float32
    row_ptr, col, perm, t_row_ptr, t_perm = oconv.csr_from_coo(recv, send, V)
    x = synth.normal(42, (V, spec.dim_x)).astype(npdt)
    y = synth.normal(43, (E, spec.dim_y)).astype(npdt)
    W = synth.normal(44, (E, spec.n_w)).astype(npdt)
    gz = synth.normal(45, (V, spec.dim_z)).astype(npdt)
    z = torch.full((V, spec.dim_z), float("nan"), dtype=tdt, device="cuda")
    za = torch.full((V, spec.dim_z), float("nan"), dtype=tdt, device="cuda")
    gx = torch.full((V, spec.dim_x), float("nan"), dtype=tdt, device="cuda")
    gy = torch.full((E, spec.dim_y), float("nan"), dtype=tdt, device="cuda")
    gW = torch.full((E, spec.n_w), float("nan"), dtype=tdt, device="cuda")
    b.conv_forward(plan, dev(x), dev(y), dev(W), z, dev(row_ptr), dev(col))
    b.conv_backward(plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW, dev(row_ptr), dev(col), dev(t_row_ptr), dev(t_perm))
    b.conv_forward_atomic(plan, dev(x), dev(y), dev(W), za, dev(oconv.rows_of_edges(row_ptr)), dev(col))
    torch.cuda.synchronize()
    ref = memo(oconv.forward, spec, x, y, W, row_ptr, col)
    assert_close(z.cpu().numpy(), ref, prec, "z")
    assert_close(za.cpu().numpy(), ref, prec, "z (atomic)")
    rx, ry, rW = memo(oconv.backward, spec, x, y, W, gz, row_ptr, col)
    assert_close(gx.cpu().numpy(), rx, prec, "gx")
    assert_close(gy.cpu().numpy(), ry, prec, "gy")
    assert_close(gW.cpu().numpy(), rW, prec, "gW")


def test_compensated_row_sums_are_more_accurate_on_long_rows():
    """fp32, a few rows with tens of thousands of edges each: the error against the fp64 oracle must drop
    clearly when the plan uses compensated sums (forward: sums over a receiver's edges; backward: over a
    sender's edges)."""
    b = _b()
    ix, iy, iz = "32x0e+32x1o+32x2e", synth.MACE_Y, "32x0e+32x1o+32x2e+32x3o"
    spec = TPSpec(ix, iy, iz)
    V, E = 6, 36000
    rng = np.random.default_rng(7)
    recv = rng.integers(0, 3, E).astype(np.int64)          # three receivers take all edges
    send = rng.integers(3, 6, E).astype(np.int64)          # three senders emit all edges
    row_ptr, col, perm, t_row_ptr, t_perm = oconv.csr_from_coo(recv, send, V)
    print(f"spec=32-channel V={V} E={E} entry=conv_forward/conv_backward plain vs kahan", flush=True)
    x = synth.normal(52, (V, spec.dim_x)).astype(np.float32)
    y = synth.normal(53, (E, spec.dim_y)).astype(np.float32)
    W = synth.normal(54, (E, spec.n_w)).astype(np.float32)
    gz = synth.normal(55, (V, spec.dim_z)).astype(np.float32)
    # reference on a channel subset (the full oracle at this size is slow): segment-wise slices keep whole channels
    errs = {}
    dx, dy, dW, dgz = dev(x), dev(y), dev(W), dev(gz)
    drp, dcol, dtrp, dtp = dev(row_ptr), dev(col), dev(t_row_ptr), dev(t_perm)
    zs, gxs = {}, {}
    for kahan in (False, True):
        plan = b.Plan(ix, iy, iz, dtype=b.CGTP_F32, device=0, kahan_conv=kahan)
        z = torch.empty((V, spec.dim_z), dtype=torch.float32, device="cuda")
        gx = torch.empty((V, spec.dim_x), dtype=torch.float32, device="cuda")
        gy = torch.empty((E, spec.dim_y), dtype=torch.float32, device="cuda")
        gW = torch.empty((E, spec.n_w), dtype=torch.float32, device="cuda")
        b.conv_forward(plan, dx, dy, dW, z, drp, dcol)
        b.conv_backward(plan, dx, dy, dW, dgz, gx, gy, gW, drp, dcol, dtrp, dtp)
        torch.cuda.synchronize()
        zs[kahan], gxs[kahan] = z.cpu().numpy().astype(np.float64), gx.cpu().numpy().astype(np.float64)
    # fp64 reference in slabs of edges (memory), summed in fp64
    ref_z = np.zeros((V, spec.dim_z)); ref_gx = np.zeros((V, spec.dim_x))
    recv_of = oconv.rows_of_edges(row_ptr)
    from oracle import tp as otp
    for a in range(0, E, 9000):
        e = np.arange(a, min(E, a + 9000))
        ze = otp.forward(spec, x[col[e]], y[e], W[e])
        np.add.at(ref_z, recv_of[e], ze)
        rx, _, _ = otp.backward(spec, x[col[e]], y[e], W[e], gz[recv_of[e]])
        np.add.at(ref_gx, col[e], rx)
    for name, got, ref in (("z", zs, ref_z), ("gx", gxs, ref_gx)):
        scale = np.sqrt(np.mean(ref[np.abs(ref).sum(axis=1) > 0] ** 2))
        e_plain = np.abs(got[False] - ref).max() / scale
        e_kahan = np.abs(got[True] - ref).max() / scale
        print(f"{name}: max error / rms  plain {e_plain:.3e}  compensated {e_kahan:.3e}", flush=True)
        assert e_kahan < 1e-4 and e_plain < 1e-4
        assert e_kahan < 0.5 * e_plain, (name, e_plain, e_kahan)


@pytest.mark.parametrize("env", [{"CGTP_PHASES_CONV_FWD": "2"},
                                 {"CGTP_PHASES_CONV_FWD": "3", "CGTP_PREFETCH_CONV_FWD": "0", "CGTP_FRESH_Y": "1"},
                                 {"CGTP_PHASES_CONV_BWD": "2"},
                                 {"CGTP_PHASES_CONV_BWD": "3", "CGTP_PIN_PER_PATH": "2", "CGTP_FRESH_Y": "1"}])
@pytest.mark.parametrize("graph", ["typical", "few_long_rows", "many_empty"])
@pytest.mark.parametrize("spec_name", ["mace", "small", "mul192"])
def test_conv_phased_schedules_give_the_same_results(spec_name, graph, env, monkeypatch):
    """Phases over output segments (forward) and over x segments (backward): every phase walks the edge range
    again with part of the accumulators; results must not change."""
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    b, spec, plan, (x, y, W, gz), (row_ptr, col, perm, t_row_ptr, t_perm), (V, E) = build(spec_name, graph, "f64", seed=9)
    print(f"spec={spec_name} graph={graph} env={env} entry=conv_forward/conv_forward_atomic/conv_backward", flush=True)
    z = torch.full((V, spec.dim_z), float("nan"), dtype=torch.float64, device="cuda")
    za = torch.full((V, spec.dim_z), float("nan"), dtype=torch.float64, device="cuda")
    gx = torch.full((V, spec.dim_x), float("nan"), dtype=torch.float64, device="cuda")
    gy = torch.full((E, spec.dim_y), float("nan"), dtype=torch.float64, device="cuda")
    gW = torch.full((E, spec.n_w), float("nan"), dtype=torch.float64, device="cuda")
    b.conv_forward(plan, dev(x), dev(y), dev(W), z, dev(row_ptr), dev(col))
    b.conv_forward_atomic(plan, dev(x), dev(y), dev(W), za, dev(oconv.rows_of_edges(row_ptr)), dev(col))
    b.conv_backward(plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW, dev(row_ptr), dev(col), dev(t_row_ptr), dev(t_perm))
    torch.cuda.synchronize()
    ref = memo(oconv.forward, spec, x, y, W, row_ptr, col)
    assert_close(z.cpu().numpy(), ref, "f64", "z")
    assert_close(za.cpu().numpy(), ref, "f64", "z (atomic)")
    rx, ry, rW = memo(oconv.backward, spec, x, y, W, gz, row_ptr, col)
    assert_close(gx.cpu().numpy(), rx, "f64", "gx")
    assert_close(gy.cpu().numpy(), ry, "f64", "gy")
    assert_close(gW.cpu().numpy(), rW, "f64", "gW")


@pytest.mark.parametrize("prec", ["f64", "f32"])
@pytest.mark.parametrize("graph", ["typical", "few_long_rows", "many_empty", "single_edge"])
@pytest.mark.parametrize("spec_name", ["small", "mace", "mul192"])
def test_conv_on_unsorted_edge_data_through_the_edge_permutation(spec_name, graph, prec):
    """Edge tensors stay in the caller's (unsorted) order; the kernels walk the CSR built by the library and
    reach the rows through `perm`.  Deterministic, equal to the oracle on the sorted data."""
    b = _b()
    ix, iy, iz = SPECS[spec_name]
    spec = TPSpec(ix, iy, iz)
    plan = b.Plan(ix, iy, iz, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0)
    V, E, empty = GRAPHS[graph]
    recv, send = random_graph(71, V, E, empty)
    print(f"spec={spec_name} graph={graph} prec={prec} V={V} E={E} entry=conv_forward_perm/conv_backward_perm", flush=True)
    npdt = np.float64 if prec == "f64" else np.float32
    tdt = torch.float64 if prec == "f64" else torch.float32
    x = synth.normal(72, (V, spec.dim_x)).astype(npdt)
    y = synth.normal(73, (E, spec.dim_y)).astype(npdt)          # rows in the original edge order
    W = synth.normal(74, (E, spec.n_w)).astype(npdt)
    gz = synth.normal(75, (V, spec.dim_z)).astype(npdt)
    row_ptr, col, perm, t_row_ptr, t_perm = b.cgtp_csr_from_coo(dev(recv), dev(send), V)
    z = torch.full((V, spec.dim_z), float("nan"), dtype=tdt, device="cuda")
    gx = torch.full((V, spec.dim_x), float("nan"), dtype=tdt, device="cuda")
    gy = torch.full((E, spec.dim_y), float("nan"), dtype=tdt, device="cuda")
    gW = torch.full((E, spec.n_w), float("nan"), dtype=tdt, device="cuda")
    b.conv_forward_perm(plan, dev(x), dev(y), dev(W), z, row_ptr, col, perm)
    b.conv_backward_perm(plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW, row_ptr, col, t_row_ptr, t_perm, perm)
    torch.cuda.synchronize()
    rp, cl, pm, _, _ = oconv.csr_from_coo(recv, send, V)
    assert_close(z.cpu().numpy(), memo(oconv.forward, spec, x, y[pm], W[pm], rp, cl), prec, "z")
    rx, ry, rW = memo(oconv.backward, spec, x, y[pm], W[pm], gz, rp, cl)
    assert_close(gx.cpu().numpy(), rx, prec, "gx")
    assert_close(gy.cpu().numpy()[pm], ry, prec, "gy")
    assert_close(gW.cpu().numpy()[pm], rW, prec, "gW")
