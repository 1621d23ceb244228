"""GPU parity on seeded random uvu problems (paper Eq. 2, kernel B): irreps lists, multiplicities, degrees, path
subsets and path coefficients drawn at random, every entry point of the batched product and of the fused convolution
against the CPU oracle through the C ABI.  The fixed cases elsewhere were chosen by hand; these are not."""
import numpy as np
import pytest

from oracle import conv as oconv
from oracle import tp as otp
from oracle.irreps import TPSpec, Path, parse_irreps, path_allowed
from tests._util import assert_close

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

MULS = [1, 2, 3, 4, 5, 8, 12, 16, 24, 32, 48, 64, 96]


def random_uvu_problem(seed):
    """x: 1-4 segments (degree <= 3, either parity, a multiplicity from MULS); y: 1-3 distinct irreps of multiplicity 1;
    z: 1-5 segments, each reachable from one (x, y) pair and of that x segment's multiplicity.  Paths: every allowed
    triple with equal multiplicities, each dropped with probability 1/4 (at least one kept), a third of them with a
    coefficient other than 1."""
    rng = np.random.default_rng(seed)
    par = lambda: "eo"[int(rng.integers(0, 2))]
    xs = [(int(rng.choice(MULS)), int(rng.integers(0, 4)), par()) for _ in range(int(rng.integers(1, 5)))]
    ys = list(dict.fromkeys((1, int(rng.integers(0, 4)), par()) for _ in range(int(rng.integers(1, 4)))))
    zs = []
    for _ in range(int(rng.integers(1, 6))):
        m, l1, p1 = xs[int(rng.integers(0, len(xs)))]
        _, l2, p2 = ys[int(rng.integers(0, len(ys)))]
        l3 = int(rng.integers(abs(l1 - l2), l1 + l2 + 1))
        zs.append((m, l3, "e" if p1 == p2 else "o"))
    fmt = lambda seg: "+".join(f"{m}x{l}{p}" for m, l, p in seg)
    ix, iy, iz = fmt(xs), fmt(ys), fmt(zs)
    irx, iry, irz = parse_irreps(ix), parse_irreps(iy), parse_irreps(iz)
    allowed = [(a, b, c) for a, ia in enumerate(irx) for b, ib in enumerate(iry) for c, ic in enumerate(irz)
               if path_allowed(ia, ib, ic) and ia.mul == ic.mul]
    keep = [t for t in allowed if rng.random() >= 0.25] or allowed[:1]
    paths = [(a, b, c, 0, float(np.round(rng.uniform(-2, 2), 3)) if rng.random() < 1 / 3 else 1.0) for a, b, c in keep]
    return ix, iy, iz, paths


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("prec", ["f64", "f32"])
@pytest.mark.parametrize("seed", list(range(200, 224)))
def test_random_uvu_problems(seed, prec):
    from paper_2501_13986_amd import binding as b
    ix, iy, iz, paths = random_uvu_problem(seed)
    spec = TPSpec(ix, iy, iz, paths=[Path(p[0], p[1], p[2], 0, p[4]) for p in paths])
    plan = b.Plan(ix, iy, iz, paths=paths, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0)
    assert (plan.dim_x, plan.dim_y, plan.dim_z, plan.n_w) == (spec.dim_x, spec.dim_y, spec.dim_z, spec.n_w)
    npdt, tdt = (np.float64, torch.float64) if prec == "f64" else (np.float32, torch.float32)
    rng = np.random.default_rng(seed + 5000)
    B = 131
    print(f"seed={seed} prec={prec} ({ix}) x ({iy}) -> ({iz}) paths={paths} B={B}", flush=True)

    def out(n, d):
        return torch.full((n + 1, d), 7.0, dtype=tdt, device="cuda")     # one guard row

    # batched product: forward, backward, second-order pass
    x, y, gz = (rng.normal(size=(B, d)).astype(npdt) for d in (spec.dim_x, spec.dim_y, spec.dim_z))
    W, LC = (rng.normal(size=(B, spec.n_w)).astype(npdt) for _ in range(2))
    La, Lb = (rng.normal(size=(B, d)).astype(npdt) for d in (spec.dim_x, spec.dim_y))
    print("  entry=tp_forward", flush=True)
    z = out(B, spec.dim_z); b.tp_forward(plan, dev(x), dev(y), dev(W), z, B=B)
    print("  entry=tp_backward", flush=True)
    gx, gy, gW = out(B, spec.dim_x), out(B, spec.dim_y), out(B, spec.n_w)
    b.tp_backward(plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW, B=B)
    print("  entry=tp_double_backward", flush=True)
    Lx, Ly, LW, Lgz = out(B, spec.dim_x), out(B, spec.dim_y), out(B, spec.n_w), out(B, spec.dim_z)
    b.tp_double_backward(plan, dev(x), dev(y), dev(W), dev(gz), dev(La), dev(Lb), dev(LC), Lx, Ly, LW, Lgz, B=B)
    torch.cuda.synchronize()
    for t in (z, gx, gy, gW, Lx, Ly, LW, Lgz):
        assert torch.all(t[B:] == 7.0)
    assert_close(z[:B].cpu().numpy(), otp.forward(spec, x, y, W), prec, "z")
    for g, r, what in zip((gx, gy, gW), otp.backward(spec, x, y, W, gz), ("gx", "gy", "gW")):
        assert_close(g[:B].cpu().numpy(), r, prec, what)
    for g, r, what in zip((Lx, Ly, LW, Lgz), otp.double_backward(spec, x, y, W, gz, La, Lb, LC), ("dL/dx", "dL/dy", "dL/dW", "dL/dgz")):
        assert_close(g[:B].cpu().numpy(), r, prec, what)

    # fused convolution on a small random graph with a few empty rows: CSR-sorted forward / backward (the second-order
    # pass and the atomic variants follow below)
    V, E = 23, 260
    recv, send = rng.integers(0, V, E).astype(np.int64), rng.integers(0, V, E).astype(np.int64)
    recv[recv == 7] = 8; recv[recv == V - 1] = 0
    row_ptr, col, perm, t_row_ptr, t_perm = oconv.csr_from_coo(recv, send, V)
    xn, gzn = rng.normal(size=(V, spec.dim_x)).astype(npdt), rng.normal(size=(V, spec.dim_z)).astype(npdt)
    ye, We = rng.normal(size=(E, spec.dim_y)).astype(npdt), rng.normal(size=(E, spec.n_w)).astype(npdt)
    print(f"  entry=conv_forward V={V} E={E}", flush=True)
    zn = torch.full((V, spec.dim_z), 7.0, dtype=tdt, device="cuda")
    b.conv_forward(plan, dev(xn), dev(ye), dev(We), zn, dev(row_ptr), dev(col))
    print("  entry=conv_backward", flush=True)
    gxn = torch.full((V, spec.dim_x), 7.0, dtype=tdt, device="cuda")
    gye, gWe = torch.full((E, spec.dim_y), 7.0, dtype=tdt, device="cuda"), torch.full((E, spec.n_w), 7.0, dtype=tdt, device="cuda")
    b.conv_backward(plan, dev(xn), dev(ye), dev(We), dev(gzn), gxn, gye, gWe, dev(row_ptr), dev(col), dev(t_row_ptr), dev(t_perm))
    torch.cuda.synchronize()
    assert_close(zn.cpu().numpy(), oconv.forward(spec, xn, ye, We, row_ptr, col), prec, "conv z")
    for g, r, what in zip((gxn, gye, gWe), oconv.backward(spec, xn, ye, We, gzn, row_ptr, col), ("conv gx", "conv gy", "conv gW")):
        assert_close(g.cpu().numpy(), r, prec, what)

    # second-order pass of the convolution, and the atomic variants on the unsorted edge list
    Lan, Lbe, LCe = (rng.normal(size=s_).astype(npdt) for s_ in ((V, spec.dim_x), (E, spec.dim_y), (E, spec.n_w)))
    print("  entry=conv_double_backward", flush=True)
    Lxn, Lgzn = torch.full((V, spec.dim_x), 7.0, dtype=tdt, device="cuda"), torch.full((V, spec.dim_z), 7.0, dtype=tdt, device="cuda")
    Lye, LWe = torch.full((E, spec.dim_y), 7.0, dtype=tdt, device="cuda"), torch.full((E, spec.n_w), 7.0, dtype=tdt, device="cuda")
    b.conv_double_backward(plan, dev(xn), dev(ye), dev(We), dev(gzn), dev(Lan), dev(Lbe), dev(LCe), Lxn, Lye, LWe, Lgzn,
                           dev(row_ptr), dev(col), dev(t_row_ptr), dev(t_perm))
    print("  entry=conv_forward_atomic/conv_backward_atomic", flush=True)
    y_orig = np.empty_like(ye); y_orig[perm] = ye           # rows in the original (unsorted) edge order
    W_orig = np.empty_like(We); W_orig[perm] = We
    za = torch.full((V, spec.dim_z), 7.0, dtype=tdt, device="cuda")
    gxa = torch.full((V, spec.dim_x), 7.0, dtype=tdt, device="cuda")
    gya, gWa = torch.full((E, spec.dim_y), 7.0, dtype=tdt, device="cuda"), torch.full((E, spec.n_w), 7.0, dtype=tdt, device="cuda")
    b.conv_forward_atomic(plan, dev(xn), dev(y_orig), dev(W_orig), za, dev(recv), dev(send))
    b.conv_backward_atomic(plan, dev(xn), dev(y_orig), dev(W_orig), dev(gzn), gxa, gya, gWa, dev(recv), dev(send))
    torch.cuda.synchronize()
    ref2 = oconv.double_backward(spec, xn, ye, We, gzn, Lan, Lbe, LCe, row_ptr, col)
    for g, r, what in zip((Lxn, Lye, LWe, Lgzn), ref2, ("conv dL/dx", "conv dL/dy", "conv dL/dW", "conv dL/dgz")):
        assert_close(g.cpu().numpy(), r, prec, what)
    assert_close(za.cpu().numpy(), oconv.forward(spec, xn, ye, We, row_ptr, col), prec, "atomic z")
    rx, ry, rW = oconv.backward(spec, xn, ye, We, gzn, row_ptr, col)
    assert_close(gxa.cpu().numpy(), rx, prec, "atomic gx")
    assert_close(gya.cpu().numpy()[perm], ry, prec, "atomic gy")
    assert_close(gWa.cpu().numpy()[perm], rW, prec, "atomic gW")
