"""GPU parity at the full benchmark sizes (configs 2-5), in the launch configuration bench.py times.
The oracle cannot run these sizes in seconds, so sampled outputs are recomputed one by one:
sampled batch rows (configs 2, 3), sampled receiver rows (config 4), sampled sender rows and
sampled edges (config 5).  Large N(0,1) tensors are drawn on the device with torch's seeded
generator (plumbing only) and the sampled rows are copied to the host for the oracle."""
import numpy as np
import pytest

from oracle import conv as oconv, tp as otp
from oracle.irreps import TPSpec, UVW
from paper_2501_13986_amd import synth
from tests._util import assert_close

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def gauss(seed, shape, dt):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return torch.randn(shape, generator=g, device="cuda", dtype=dt)


def tdt(prec):
    return torch.float64 if prec == "f64" else torch.float32


def host(t, idx=None):
    return (t if idx is None else t[torch.as_tensor(idx, device=t.device)]).cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("prec", ["f32", "f64"])
def test_config2_mace_batched_forward_backward(prec):
    from paper_2501_13986_amd import binding as b
    irr = (synth.MACE_X, synth.MACE_Y, synth.MACE_Z)
    spec = TPSpec(*irr)
    plan = b.Plan(*irr, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0)
    B, dt = 50000, tdt(prec)
    print(f"config 2 prec={prec} B={B} entry=tp_forward/tp_backward", flush=True)
    x = gauss(2000, (B, spec.dim_x), dt); W = gauss(2002, (B, spec.n_w), dt); gz = gauss(2003, (B, spec.dim_z), dt)
    y = torch.from_numpy(synth.sh_edge_attr(synth.unit_vectors(2001, B), 3)).to("cuda", dt)
    z = torch.empty((B, spec.dim_z), device="cuda", dtype=dt)
    gx = torch.empty_like(x); gy = torch.empty_like(y); gW = torch.empty_like(W)
    b.tp_forward(plan, x, y, W, z)
    b.tp_backward(plan, x, y, W, gz, gx, gy, gW)
    torch.cuda.synchronize()
    idx = np.unique(np.concatenate([[0, 1, 63, 64, B - 2, B - 1], np.random.default_rng(0).integers(0, B, 58)]))
    xs, ys, Ws, gzs = host(x, idx), host(y, idx), host(W, idx), host(gz, idx)
    assert_close(host(z, idx), otp.forward(spec, xs, ys, Ws), prec, "z")
    rx, ry, rW = otp.backward(spec, xs, ys, Ws, gzs)
    assert_close(host(gx, idx), rx, prec, "gx")
    assert_close(host(gy, idx), ry, prec, "gy")
    assert_close(host(gW, idx), rW, prec, "gW")
    for t in (z, gx, gy, gW):
        assert bool(torch.isfinite(t).all())


def test_config3_nequip_uvw_forward():
    from paper_2501_13986_amd import binding as b
    irr = (synth.NEQUIP_X, synth.NEQUIP_Y, synth.NEQUIP_Z)
    spec = TPSpec(*irr, mode=UVW, shared_weights=True)
    plan = b.Plan(*irr, mode=b.CGTP_UVW, shared_weights=True, dtype=b.CGTP_F32, device=0)
    B = 100000
    print(f"config 3 B={B} entry=tp_forward (uvw)", flush=True)
    x = gauss(3000, (B, spec.dim_x), torch.float32)
    y = torch.from_numpy(synth.sh_edge_attr(synth.unit_vectors(3001, B), 2)).to("cuda", torch.float32)
    W = gauss(3002, (spec.n_w,), torch.float32) / np.sqrt(32.0)
    z = torch.empty((B, spec.dim_z), device="cuda", dtype=torch.float32)
    b.tp_forward(plan, x, y, W, z)
    torch.cuda.synchronize()
    idx = np.unique(np.concatenate([[0, 15, 16, B - 17, B - 16, B - 1], np.random.default_rng(1).integers(0, B, 58)]))
    assert_close(host(z, idx), otp.forward(spec, host(x, idx), host(y, idx), host(W)), "f32", "z")
    assert bool(torch.isfinite(z).all())


def test_config3_shape_uvw_backward():
    """Shared weights, B = 100000.  gx and gy are per row: sampled rows against the oracle.  gW is a sum over the
    whole batch: with gz zero outside the sampled rows the other rows contribute exact zeros, so the oracle on the
    sampled rows alone gives the expected sum while the kernel walks all 100000 rows."""
    from paper_2501_13986_amd import binding as b
    irr = (synth.NEQUIP_X, synth.NEQUIP_Y, synth.NEQUIP_Z)
    spec = TPSpec(*irr, mode=UVW, shared_weights=True)
    plan = b.Plan(*irr, mode=b.CGTP_UVW, shared_weights=True, dtype=b.CGTP_F32, device=0)
    B = 100000
    print(f"config 3 shape B={B} entry=tp_backward (uvw, shared weights)", flush=True)
    x = gauss(3100, (B, spec.dim_x), torch.float32)
    y = torch.from_numpy(synth.sh_edge_attr(synth.unit_vectors(3101, B), 2)).to("cuda", torch.float32)
    W = gauss(3102, (spec.n_w,), torch.float32) / np.sqrt(32.0)
    gz = gauss(3103, (B, spec.dim_z), torch.float32)
    gx = torch.empty_like(x); gy = torch.empty_like(y); gW = torch.empty_like(W)
    idx = np.unique(np.concatenate([[0, 15, 16, 63, 64, B - 65, B - 17, B - 16, B - 1], np.random.default_rng(2).integers(0, B, 55)]))
    b.tp_backward(plan, x, y, W, gz, gx, gy, gW)
    torch.cuda.synchronize()
    rx, ry, _ = otp.backward(spec, host(x, idx), host(y, idx), host(W), host(gz, idx))
    assert_close(host(gx, idx), rx, "f32", "gx")
    assert_close(host(gy, idx), ry, "f32", "gy")
    assert bool(torch.isfinite(gW).all()) and bool(torch.isfinite(gx).all()) and bool(torch.isfinite(gy).all())
    keep = torch.zeros((B, 1), device="cuda", dtype=torch.float32)
    keep[torch.as_tensor(idx, device="cuda")] = 1.0
    gz0 = gz * keep
    b.tp_backward(plan, x, y, W, gz0, gx, gy, gW)
    torch.cuda.synchronize()
    rx, ry, rW = otp.backward(spec, host(x, idx), host(y, idx), host(W), host(gz0, idx))
    assert_close(host(gW), rW, "f32", "gW (sum over the batch)")
    assert_close(host(gx, idx), rx, "f32", "gx")
    off = torch.ones(B, dtype=torch.bool, device="cuda"); off[torch.as_tensor(idx, device="cuda")] = False
    assert bool((gx[off] == 0).all()) and bool((gy[off] == 0).all())


@pytest.mark.parametrize("prec", ["f32", "f64"])
def test_diffdock_shape_uvw_per_sample_weights(prec):
    from paper_2501_13986_amd import binding as b
    irr = ("48x0e+10x1o+10x1e+48x0o", synth.NEQUIP_Y, "48x0e+10x1o+10x1e+48x0o")
    spec = TPSpec(*irr, mode=UVW, shared_weights=False)
    plan = b.Plan(*irr, mode=b.CGTP_UVW, shared_weights=False, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0)
    B, dt = 50000, tdt(prec)
    print(f"DiffDock shape prec={prec} B={B} entry=tp_forward/tp_backward (uvw, per-sample weights)", flush=True)
    x = gauss(6100, (B, spec.dim_x), dt); W = gauss(6102, (B, spec.n_w), dt) / np.sqrt(48.0); gz = gauss(6103, (B, spec.dim_z), dt)
    y = torch.from_numpy(synth.sh_edge_attr(synth.unit_vectors(6101, B), 2)).to("cuda", dt)
    z = torch.empty((B, spec.dim_z), device="cuda", dtype=dt)
    gx = torch.empty_like(x); gy = torch.empty_like(y); gW = torch.empty_like(W)
    b.tp_forward(plan, x, y, W, z)
    b.tp_backward(plan, x, y, W, gz, gx, gy, gW)
    torch.cuda.synchronize()
    idx = np.unique(np.concatenate([[0, 1, 3, 4, B - 5, B - 1], np.random.default_rng(3).integers(0, B, 40)]))
    xs, ys, Ws, gzs = host(x, idx), host(y, idx), host(W, idx), host(gz, idx)
    assert_close(host(z, idx), otp.forward(spec, xs, ys, Ws), prec, "z")
    rx, ry, rW = otp.backward(spec, xs, ys, Ws, gzs)
    assert_close(host(gx, idx), rx, prec, "gx")
    assert_close(host(gy, idx), ry, prec, "gy")
    assert_close(host(gW, idx), rW, prec, "gW")
    for t in (z, gx, gy, gW):
        assert bool(torch.isfinite(t).all())


def split_rows(plan, kernel, ptr, E, count, seed):
    """Rows of a CSR-like offset array that are cut by the edge ranges of a convolution launch: the launch gives every
    wave resident on the GPU one range [w*E/n, (w+1)*E/n) of the sorted edge list (n = resident waves, at most E); a row
    holding a range boundary strictly inside is assembled from pieces of two or more waves by the row-merge kernel."""
    info = plan.kernel_info(kernel)
    n = min(E, info["blocks_per_cu"] * torch.cuda.get_device_properties(0).multi_processor_count * (info["wg"] // 64))
    bounds = (np.arange(1, n, dtype=np.int64) * E) // n
    rows = np.searchsorted(ptr, bounds, side="right") - 1            # row holding edge position `bound`
    cut = rows[ptr[rows] < bounds]                                   # boundary strictly inside the row
    cut = np.unique(cut)
    assert cut.size > 0, "no split row in this launch"
    pick = np.random.default_rng(seed).choice(cut, size=min(count, cut.size), replace=False)
    return np.unique(np.concatenate([pick, cut[:1], cut[-1:]]))


class Box:
    def __init__(self, seed, V, deg):
        from paper_2501_13986_amd import binding as b
        recv, send, unit = synth.periodic_graph(seed, V, deg)
        self.V, self.E = V, recv.shape[0]
        self.dev = b.cgtp_csr_from_coo(torch.from_numpy(recv).cuda(), torch.from_numpy(send).cuda(), V)
        self.ref = oconv.csr_from_coo(recv, send, V)
        for g, r in zip(self.dev, self.ref):
            assert np.array_equal(g.cpu().numpy(), r), "CSR arrays must be bit-exact"
        self.y = synth.sh_edge_attr(unit[self.ref[2]], 3)      # CSR order, fp64, host


@pytest.mark.parametrize("prec", ["f32", "f64"])
def test_config4_conv_forward(prec):
    from paper_2501_13986_amd import binding as b
    irr = (synth.MACE_X, synth.MACE_Y, synth.MACE_Z)
    spec = TPSpec(*irr)
    plan = b.Plan(*irr, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0)
    g, dt = Box(4001, 5000, 32.0), tdt(prec)
    print(f"config 4 prec={prec} V={g.V} E={g.E} entry=conv_forward", flush=True)
    row_ptr, col = g.ref[0], g.ref[1]
    x = gauss(4000, (g.V, spec.dim_x), dt); W = gauss(4002, (g.E, spec.n_w), dt)
    y = torch.from_numpy(g.y).to("cuda", dt)
    z = torch.full((g.V, spec.dim_z), float("nan"), device="cuda", dtype=dt)
    b.conv_forward(plan, x, y, W, z, g.dev[0], g.dev[1])
    torch.cuda.synchronize()
    assert bool(torch.isfinite(z).all())
    rows = np.unique(np.concatenate([[0, 1, g.V - 1], np.random.default_rng(2).integers(0, g.V, 21),
                                     split_rows(plan, b.K_CONV_FWD, row_ptr, g.E, 10, 12)]))   # incl. rows cut by the edge ranges
    xh = host(x)
    for j in rows:
        e = np.arange(row_ptr[j], row_ptr[j + 1])
        ref = otp.forward(spec, xh[col[e]], host(y, e), host(W, e)).sum(axis=0) if e.size else np.zeros(spec.dim_z)
        assert_close(host(z, [j])[0], ref, prec, f"z row {j}")


@pytest.mark.parametrize("prec", ["f32", "f64"])
def test_config5_conv_backward(prec):
    from paper_2501_13986_amd import binding as b
    irr = (synth.MACE_X, synth.MACE_Y, synth.MACE_Z)
    spec = TPSpec(*irr)
    plan = b.Plan(*irr, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0)
    g, dt = Box(5001, 20000, 40.0), tdt(prec)
    print(f"config 5 prec={prec} V={g.V} E={g.E} entry=conv_backward", flush=True)
    row_ptr, col, perm, t_row_ptr, t_perm = g.ref
    recv_of = oconv.rows_of_edges(row_ptr)
    x = gauss(4000, (g.V, spec.dim_x), dt); W = gauss(4002, (g.E, spec.n_w), dt); gz = gauss(4003, (g.V, spec.dim_z), dt)
    y = torch.from_numpy(g.y).to("cuda", dt)
    gx = torch.full((g.V, spec.dim_x), float("nan"), device="cuda", dtype=dt)
    gy = torch.full((g.E, spec.dim_y), float("nan"), device="cuda", dtype=dt)
    gW = torch.full((g.E, spec.n_w), float("nan"), device="cuda", dtype=dt)
    b.conv_backward(plan, x, y, W, gz, gx, gy, gW, *g.dev[:2], *g.dev[3:])
    torch.cuda.synchronize()
    for t in (gx, gy, gW):
        assert bool(torch.isfinite(t).all())
    xh, gzh = host(x), host(gz)
    # sampled edges: gy and gW are per edge
    e = np.unique(np.concatenate([[0, 1, g.E - 1], np.random.default_rng(3).integers(0, g.E, 61)]))
    rx, ry, rW = otp.backward(spec, xh[col[e]], host(y, e), host(W, e), gzh[recv_of[e]])
    assert_close(host(gy, e), ry, prec, "gy (sampled edges)")
    assert_close(host(gW, e), rW, prec, "gW (sampled edges)")
    # sampled sender rows: gx sums over the edges leaving the node
    for k in np.unique(np.concatenate([[0, g.V - 1], np.random.default_rng(4).integers(0, g.V, 8),
                                       split_rows(plan, b.K_CONV_BWD, t_row_ptr, g.E, 8, 14)])):   # incl. sender rows cut by the ranges
        ek = t_perm[t_row_ptr[k]:t_row_ptr[k + 1]]
        if ek.size:
            rxk, _, _ = otp.backward(spec, np.repeat(xh[k][None], ek.size, 0), host(y, ek), host(W, ek), gzh[recv_of[ek]])
            ref = rxk.sum(axis=0)
        else:
            ref = np.zeros(spec.dim_x)
        assert_close(host(gx, [k])[0], ref, prec, f"gx row {k}")


@pytest.mark.parametrize("prec", ["f32", "f64"])
def test_config2_shape_double_backward(prec):
    """Fused second-order pass at the benchmark batch (B = 50000), sampled rows against the oracle."""
    from paper_2501_13986_amd import binding as b
    irr = (synth.MACE_X, synth.MACE_Y, synth.MACE_Z)
    spec = TPSpec(*irr)
    plan = b.Plan(*irr, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0)
    B, dt = 50000, tdt(prec)
    print(f"config 2 shape prec={prec} B={B} entry=tp_double_backward", flush=True)
    x = gauss(2000, (B, spec.dim_x), dt); W = gauss(2002, (B, spec.n_w), dt); gz = gauss(2003, (B, spec.dim_z), dt)
    y = torch.from_numpy(synth.sh_edge_attr(synth.unit_vectors(2001, B), 3)).to("cuda", dt)
    La = gauss(2004, (B, spec.dim_x), dt); LC = gauss(2006, (B, spec.n_w), dt)
    Lb = torch.from_numpy(synth.sh_edge_attr(synth.unit_vectors(2005, B), 3)).to("cuda", dt)
    outs = [torch.full((B, d), float("nan"), device="cuda", dtype=dt) for d in (spec.dim_x, spec.dim_y, spec.n_w, spec.dim_z)]
    b.tp_double_backward(plan, x, y, W, gz, La, Lb, LC, *outs)
    torch.cuda.synchronize()
    idx = np.unique(np.concatenate([[0, 1, 63, 64, B - 2, B - 1], np.random.default_rng(5).integers(0, B, 40)]))
    ref = otp.double_backward(spec, *(host(t, idx) for t in (x, y, W, gz, La, Lb, LC)))
    for got, r, what in zip(outs, ref, ("dL/dx", "dL/dy", "dL/dW", "dL/dgz")):
        assert_close(host(got, idx), r, prec, what)
        assert bool(torch.isfinite(got).all())


@pytest.mark.parametrize("prec", ["f32", "f64"])
def test_config4_shape_atomic_conv_on_unsorted_edges(prec):
    """Atomic forward and backward on the 5000-node graph with its edges in generator (unsorted) order:
    sampled receiver rows of z, sampled sender rows of gx, sampled edges of gy and gW."""
    from paper_2501_13986_amd import binding as b
    irr = (synth.MACE_X, synth.MACE_Y, synth.MACE_Z)
    spec = TPSpec(*irr)
    plan = b.Plan(*irr, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0)
    dt = tdt(prec)
    recv, send, unit = synth.periodic_graph(4001, 5000, 32.0)
    V, E = 5000, recv.shape[0]
    print(f"config 4 shape prec={prec} V={V} E={E} entry=conv_forward_atomic/conv_backward_atomic", flush=True)
    x = gauss(4000, (V, spec.dim_x), dt); W = gauss(4002, (E, spec.n_w), dt); gz = gauss(4003, (V, spec.dim_z), dt)
    y = torch.from_numpy(synth.sh_edge_attr(unit, 3)).to("cuda", dt)       # rows in the unsorted edge order
    rd, sd = torch.from_numpy(recv).cuda(), torch.from_numpy(send).cuda()
    z = torch.full((V, spec.dim_z), float("nan"), device="cuda", dtype=dt)
    gx = torch.full((V, spec.dim_x), float("nan"), device="cuda", dtype=dt)
    gy = torch.full((E, spec.dim_y), float("nan"), device="cuda", dtype=dt)
    gW = torch.full((E, spec.n_w), float("nan"), device="cuda", dtype=dt)
    b.conv_forward_atomic(plan, x, y, W, z, rd, sd)
    b.conv_backward_atomic(plan, x, y, W, gz, gx, gy, gW, rd, sd)
    torch.cuda.synchronize()
    for t in (z, gx, gy, gW):
        assert bool(torch.isfinite(t).all())
    xh, gzh = host(x), host(gz)
    rng = np.random.default_rng(6)
    for j in np.unique(np.concatenate([[0, V - 1], rng.integers(0, V, 14)])):
        e = np.nonzero(recv == j)[0]
        ref = otp.forward(spec, xh[send[e]], host(y, e), host(W, e)).sum(axis=0) if e.size else np.zeros(spec.dim_z)
        assert_close(host(z, [j])[0], ref, prec, f"z row {j}")
    e = np.unique(np.concatenate([[0, E - 1], rng.integers(0, E, 46)]))
    _, ry, rW = otp.backward(spec, xh[send[e]], host(y, e), host(W, e), gzh[recv[e]])
    assert_close(host(gy, e), ry, prec, "gy (sampled edges)")
    assert_close(host(gW, e), rW, prec, "gW (sampled edges)")
    for k in np.unique(np.concatenate([[0, V - 1], rng.integers(0, V, 10)])):
        ek = np.nonzero(send == k)[0]
        if ek.size:
            rxk, _, _ = otp.backward(spec, np.repeat(xh[k][None], ek.size, 0), host(y, ek), host(W, ek), gzh[recv[ek]])
            ref = rxk.sum(axis=0)
        else:
            ref = np.zeros(spec.dim_x)
        assert_close(host(gx, [k])[0], ref, prec, f"gx row {k}")


@pytest.mark.parametrize("prec", ["f32", "f64"])
def test_config4_shape_conv_double_backward(prec):
    """Second-order pass of the convolution on the 5000-node graph: sampled edges (dL/dy, dL/dW), sampled receiver
    rows (dL/dgz) and sampled sender rows (dL/dx), each recomputed as the gather / scatter of the oracle's
    per-edge second-order pass."""
    from paper_2501_13986_amd import binding as b
    irr = (synth.MACE_X, synth.MACE_Y, synth.MACE_Z)
    spec = TPSpec(*irr)
    plan = b.Plan(*irr, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0)
    g, dt = Box(4001, 5000, 32.0), tdt(prec)
    print(f"config 4 shape prec={prec} V={g.V} E={g.E} entry=conv_double_backward", flush=True)
    row_ptr, col, perm, t_row_ptr, t_perm = g.ref
    recv_of = oconv.rows_of_edges(row_ptr)
    x = gauss(4000, (g.V, spec.dim_x), dt); W = gauss(4002, (g.E, spec.n_w), dt); gz = gauss(4003, (g.V, spec.dim_z), dt)
    La = gauss(4004, (g.V, spec.dim_x), dt); LC = gauss(4006, (g.E, spec.n_w), dt)
    y = torch.from_numpy(g.y).to("cuda", dt)
    Lb = gauss(4005, (g.E, spec.dim_y), dt)
    Lx = torch.full((g.V, spec.dim_x), float("nan"), device="cuda", dtype=dt)
    Ly = torch.full((g.E, spec.dim_y), float("nan"), device="cuda", dtype=dt)
    LW = torch.full((g.E, spec.n_w), float("nan"), device="cuda", dtype=dt)
    Lgz = torch.full((g.V, spec.dim_z), float("nan"), device="cuda", dtype=dt)
    b.conv_double_backward(plan, x, y, W, gz, La, Lb, LC, Lx, Ly, LW, Lgz, g.dev[0], g.dev[1], g.dev[3], g.dev[4])
    torch.cuda.synchronize()
    for t in (Lx, Ly, LW, Lgz):
        assert bool(torch.isfinite(t).all())
    xh, gzh, Lah = host(x), host(gz), host(La)

    def per_edge(e):
        return otp.double_backward(spec, xh[col[e]], host(y, e), host(W, e), gzh[recv_of[e]], Lah[col[e]], host(Lb, e), host(LC, e))
    rng = np.random.default_rng(8)
    e = np.unique(np.concatenate([[0, g.E - 1], rng.integers(0, g.E, 30)]))
    _, ry, rW, _ = per_edge(e)
    assert_close(host(Ly, e), ry, prec, "dL/dy (sampled edges)")
    assert_close(host(LW, e), rW, prec, "dL/dW (sampled edges)")
    for j in np.unique(np.concatenate([[0, g.V - 1], rng.integers(0, g.V, 8)])):
        ej = np.arange(row_ptr[j], row_ptr[j + 1])
        ref = per_edge(ej)[3].sum(axis=0) if ej.size else np.zeros(spec.dim_z)
        assert_close(host(Lgz, [j])[0], ref, prec, f"dL/dgz row {j}")
    for k in np.unique(np.concatenate([[0, g.V - 1], rng.integers(0, g.V, 8)])):
        ek = t_perm[t_row_ptr[k]:t_row_ptr[k + 1]]
        ref = per_edge(ek)[0].sum(axis=0) if ek.size else np.zeros(spec.dim_x)
        assert_close(host(Lx, [k])[0], ref, prec, f"dL/dx row {k}")
