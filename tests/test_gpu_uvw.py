"""GPU parity of the fully connected ("uvw") tensor product against the CPU oracle, through the C ABI:
shared weights (the weight contraction runs on the matrix cores in fp32) and per-sample weights (a stream of
weight tiles, fp32 and fp64)."""
import numpy as np
import pytest

from oracle import tp as otp
from oracle.irreps import TPSpec, Path, UVW
from paper_2501_13986_amd import synth
from tests._util import assert_close

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

CASES = {
    "nequip": (synth.NEQUIP_X, synth.NEQUIP_Y, synth.NEQUIP_Z, None),
    "small": ("4x0e+4x1o", "1x0e+1x1o", "16x0e+16x1o+16x1e", None),
    "mixed_mul": ("8x0e+4x1o+12x2e", "1x0e+1x1o+1x2e", "16x0e+32x1o+16x2e", None),
    "unused_and_coeff": ("4x0e+8x1o", "1x0e+1x1o", "16x1o+5x3e+16x0e", [(0, 1, 0, 1, 0.5), (1, 1, 2, 1, -2.0)]),
}


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("B", [1, 15, 16, 17, 64, 1000])
@pytest.mark.parametrize("name", list(CASES))
def test_uvw_forward_parity(name, B):
    from paper_2501_13986_amd import binding as b
    ix, iy, iz, paths = CASES[name]
    spec = TPSpec(ix, iy, iz, mode=UVW, shared_weights=True,
                  paths=None if paths is None else [Path(p[0], p[1], p[2], UVW, p[4]) for p in paths])
    plan = b.Plan(ix, iy, iz, paths=paths, mode=b.CGTP_UVW, shared_weights=True, dtype=b.CGTP_F32, device=0)
    assert (plan.dim_x, plan.dim_y, plan.dim_z, plan.n_w) == (spec.dim_x, spec.dim_y, spec.dim_z, spec.n_w)
    print(f"case={name} B={B} entry=tp_forward (uvw)", flush=True)
    x = synth.normal(1, (B, spec.dim_x)).astype(np.float32)
    y = synth.normal(2, (B, spec.dim_y)).astype(np.float32)
    mulx = max(ir.mul for ir in spec.irx)
    W = synth.normal(3, (spec.n_w,), scale=1.0 / np.sqrt(mulx)).astype(np.float32)
    z = torch.full((B + 1, spec.dim_z), 7.0, dtype=torch.float32, device="cuda")
    b.tp_forward(plan, dev(x), dev(y), dev(W), z, B=B)
    torch.cuda.synchronize()
    assert torch.all(z[B:] == 7.0)
    ref = otp.forward(spec, x, y, W)
    assert_close(z[:B].cpu().numpy(), ref, "f32", f"{name} uvw forward")


BWD_CASES = {
    "nequip": (synth.NEQUIP_X, synth.NEQUIP_Y, synth.NEQUIP_Z, None),
    "mul16": ("16x0e+16x1o", "1x0e+1x1o", "16x0e+16x1o+16x1e", None),
    "mixed_mul": ("32x0e+16x1o+16x2e", "1x0e+1x1o+1x2e", "16x0e+32x1o+16x2e", None),
    "unused_and_coeff": ("16x0e+16x1o+16x2e", "1x0e+1x1o", "16x1o+5x3e+16x0e", [(0, 1, 0, 1, 0.5), (1, 1, 2, 1, -2.0)]),
    "one_block": ("16x1o", "1x0e+1x1o", "16x1o+16x0e", None),        # a single (segment, channel half) block per tile
    "wide": ("48x0e+16x1o", "1x0e+1x1o+1x2e", "48x0e+16x1o+32x2e", None),   # three channel blocks, unequal multiplicities
}


@pytest.mark.parametrize("B", [1, 17, 64, 1000, 5003, 70001])
@pytest.mark.parametrize("name", list(BWD_CASES))
def test_uvw_backward_parity(name, B):
    from paper_2501_13986_amd import binding as b
    ix, iy, iz, paths = BWD_CASES[name]
    spec = TPSpec(ix, iy, iz, mode=UVW, shared_weights=True,
                  paths=None if paths is None else [Path(p[0], p[1], p[2], UVW, p[4]) for p in paths])
    plan = b.Plan(ix, iy, iz, paths=paths, mode=b.CGTP_UVW, shared_weights=True, dtype=b.CGTP_F32, device=0)
    print(f"case={name} B={B} entry=tp_backward (uvw)", flush=True)
    x = synth.normal(11, (B, spec.dim_x)).astype(np.float32)
    y = synth.normal(12, (B, spec.dim_y)).astype(np.float32)
    mulx = max(ir.mul for ir in spec.irx)
    W = synth.normal(13, (spec.n_w,), scale=1.0 / np.sqrt(mulx)).astype(np.float32)
    gz = synth.normal(14, (B, spec.dim_z)).astype(np.float32)
    gx = torch.full((B + 1, spec.dim_x), 7.0, dtype=torch.float32, device="cuda")
    gy = torch.full((B + 1, spec.dim_y), 7.0, dtype=torch.float32, device="cuda")
    gW = torch.full((spec.n_w,), float("nan"), dtype=torch.float32, device="cuda")
    b.tp_backward(plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW, B=B)
    torch.cuda.synchronize()
    assert torch.all(gx[B:] == 7.0) and torch.all(gy[B:] == 7.0)
    rx, ry, rW = otp.backward(spec, x, y, W, gz)
    assert rW.shape == (spec.n_w,)
    assert_close(gx[:B].cpu().numpy(), rx, "f32", f"{name} uvw gx")
    assert_close(gy[:B].cpu().numpy(), ry, "f32", f"{name} uvw gy")
    assert_close(gW.cpu().numpy(), rW, "f32", f"{name} uvw gW")
    # deterministic: fixed-order reduction of the per-wave partial sums
    gW2 = torch.empty_like(gW)
    b.tp_backward(plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW2, B=B)
    torch.cuda.synchronize()
    assert torch.equal(gW, gW2)


def _random_shared_spec(seed):
    """Seeded random irreps for the shared-weight kernels: 1-3 segments per side, degrees up to 2 (z up to 3),
    multiplicities from {16, 32, 48, 64} (what the backward's tiles cover), y of multiplicity 1."""
    rng = np.random.default_rng(seed)
    par = lambda: "eo"[int(rng.integers(0, 2))]
    mul = lambda: int(rng.choice([16, 32, 48, 64]))
    ix = "+".join(f"{mul()}x{int(rng.integers(0, 3))}{par()}" for _ in range(int(rng.integers(1, 4))))
    iy = "+".join(dict.fromkeys(f"1x{int(rng.integers(0, 3))}{par()}" for _ in range(int(rng.integers(1, 4)))))
    iz = "+".join(f"{mul()}x{int(rng.integers(0, 4))}{par()}" for _ in range(int(rng.integers(1, 4))))
    return ix, iy, iz


@pytest.mark.parametrize("seed", list(range(300, 324)))
def test_uvw_shared_weights_random_specs(seed):
    """Forward and backward of the shared-weight kernels on seeded random irreps; plans beyond the documented
    limits (weights + tiles above 160 KB of LDS) must be refused at plan creation, not run."""
    from oracle.irreps import enumerate_paths, parse_irreps
    from paper_2501_13986_amd import binding as b
    ix, iy, iz = _random_shared_spec(seed)
    if not enumerate_paths(parse_irreps(ix), parse_irreps(iy), parse_irreps(iz)):
        pytest.skip(f"no allowed path for {ix} x {iy} -> {iz}")
    spec = TPSpec(ix, iy, iz, mode=UVW, shared_weights=True)
    try:
        plan = b.Plan(ix, iy, iz, mode=b.CGTP_UVW, shared_weights=True, dtype=b.CGTP_F32, device=0)
    except b.CgtpError as e:
        assert e.status == 2 and spec.n_w * 4 > 100 * 1024, (e.status, spec.n_w)      # CGTP_EUNSUPPORTED, and only for large weight sets
        pytest.skip(f"refused: {spec.n_w} weights")
    B = 333
    print(f"seed={seed} spec=({ix}) x ({iy}) -> ({iz}) paths={len(spec.paths)} n_w={spec.n_w} B={B} entry=tp_forward/tp_backward (uvw, shared weights)", flush=True)
    rng = np.random.default_rng(seed + 1000)
    x, y, gz = (rng.normal(size=(B, d)).astype(np.float32) for d in (spec.dim_x, spec.dim_y, spec.dim_z))
    W = (rng.normal(size=(spec.n_w,)) / 8).astype(np.float32)
    z = torch.full((B + 1, spec.dim_z), 7.0, dtype=torch.float32, device="cuda")
    b.tp_forward(plan, dev(x), dev(y), dev(W), z, B=B)
    torch.cuda.synchronize()
    assert torch.all(z[B:] == 7.0)
    assert_close(z[:B].cpu().numpy(), otp.forward(spec, x, y, W), "f32", "uvw z")
    gx, gy = (torch.full((B + 1, d), 7.0, dtype=torch.float32, device="cuda") for d in (spec.dim_x, spec.dim_y))
    gW = torch.full((spec.n_w,), 7.0, dtype=torch.float32, device="cuda")
    try:
        b.tp_backward(plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW, B=B)
    except b.CgtpError as e:
        assert e.status == 2
        pytest.skip(f"forward-only plan: {e}")
    torch.cuda.synchronize()
    assert torch.all(gx[B:] == 7.0) and torch.all(gy[B:] == 7.0)
    for g, r, what in zip((gx[:B], gy[:B], gW), otp.backward(spec, x, y, W, gz), ("uvw gx", "uvw gy", "uvw gW")):
        assert_close(g.cpu().numpy(), r, "f32", what)


# per-sample weights: W [B, n_w].  Multiplicities that divide 64, that do not, above 32 (one row of the tile per
# load) and below (several), unused segments, coefficients.
PS_CASES = {
    "diffdock_shaped": ("48x0e+10x1o+10x1e+48x0o", "1x0e+1x1o+1x2e", "48x0e+10x1o+10x1e+48x0o", None),
    "tetris_shaped": ("1x0e+1x1o+1x2e+1x3o", "1x0e+1x1o+1x2e+1x3o", "1x0o+6x0e", None),
    "odd_muls": ("3x0e+5x1o+7x2e", "1x0e+1x1o+1x2e", "9x0e+2x1o+33x2e", None),
    "wide": ("64x0e+64x1o", "1x0e+1x1o", "64x0e+64x1o", None),
    "unused_and_coeff": ("4x0e+8x1o+2x2e", "1x0e+1x1o", "16x1o+5x3e+6x0e", [(0, 1, 0, 1, 0.5), (1, 1, 2, 1, -2.0)]),
    "many_paths": ("4x0e+4x1o+4x2e+4x3o+4x4e", "1x0e+1x1o+1x2e+1x3o+1x4e", "4x0e+4x1o+4x2e+4x3o+4x4e", None),   # 42 paths, l <= 4
}


@pytest.mark.parametrize("prec", ["f32", "f64"])
@pytest.mark.parametrize("B", [1, 5, 203])
@pytest.mark.parametrize("name", list(PS_CASES))
def test_uvw_per_sample_parity(name, B, prec):
    from paper_2501_13986_amd import binding as b
    ix, iy, iz, paths = PS_CASES[name]
    spec = TPSpec(ix, iy, iz, mode=UVW, shared_weights=False,
                  paths=None if paths is None else [Path(p[0], p[1], p[2], UVW, p[4]) for p in paths])
    plan = b.Plan(ix, iy, iz, paths=paths, mode=b.CGTP_UVW, shared_weights=False,
                  dtype=b.CGTP_F32 if prec == "f32" else b.CGTP_F64, device=0)
    assert (plan.dim_x, plan.dim_y, plan.dim_z, plan.n_w) == (spec.dim_x, spec.dim_y, spec.dim_z, spec.n_w)
    print(f"case={name} B={B} {prec} entry=tp_forward/tp_backward (uvw, per-sample weights)", flush=True)
    npdt = np.float32 if prec == "f32" else np.float64
    tdt = torch.float32 if prec == "f32" else torch.float64
    x = synth.normal(21, (B, spec.dim_x)).astype(npdt)
    y = synth.normal(22, (B, spec.dim_y)).astype(npdt)
    mulx = max(ir.mul for ir in spec.irx)
    W = synth.normal(23, (B, spec.n_w), scale=1.0 / np.sqrt(mulx)).astype(npdt)
    gz = synth.normal(24, (B, spec.dim_z)).astype(npdt)
    z = torch.full((B + 1, spec.dim_z), 7.0, dtype=tdt, device="cuda")
    b.tp_forward(plan, dev(x), dev(y), dev(W), z, B=B)
    torch.cuda.synchronize()
    assert torch.all(z[B:] == 7.0)
    assert_close(z[:B].cpu().numpy(), otp.forward(spec, x, y, W), prec, f"{name} uvw per-sample forward")
    gx = torch.full((B + 1, spec.dim_x), 7.0, dtype=tdt, device="cuda")
    gy = torch.full((B + 1, spec.dim_y), 7.0, dtype=tdt, device="cuda")
    gW = torch.full((B + 1, spec.n_w), 7.0, dtype=tdt, device="cuda")
    b.tp_backward(plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW, B=B)
    torch.cuda.synchronize()
    assert torch.all(gx[B:] == 7.0) and torch.all(gy[B:] == 7.0) and torch.all(gW[B:] == 7.0)
    rx, ry, rW = otp.backward(spec, x, y, W, gz)
    assert_close(gx[:B].cpu().numpy(), rx, prec, f"{name} uvw per-sample gx")
    assert_close(gy[:B].cpu().numpy(), ry, prec, f"{name} uvw per-sample gy")
    assert_close(gW[:B].cpu().numpy(), rW, prec, f"{name} uvw per-sample gW")


def _random_spec(seed):
    """Seeded random irreps lists: 1-4 segments per side, degrees up to 3, multiplicities 1..64 (biased to small),
    both parities; y has multiplicity 1."""
    rng = np.random.default_rng(seed)
    def side(n, muls):
        out = []
        for _ in range(n):
            out.append(f"{int(rng.choice(muls))}x{int(rng.integers(0, 4))}{'eo'[int(rng.integers(0, 2))]}")
        return "+".join(out)
    muls = [1, 2, 3, 5, 8, 10, 13, 16, 21, 32, 33, 48, 64]
    ix, iz = side(int(rng.integers(1, 5)), muls), side(int(rng.integers(1, 5)), muls)
    iy = "+".join(dict.fromkeys(f"1x{int(rng.integers(0, 4))}{'eo'[int(rng.integers(0, 2))]}" for _ in range(int(rng.integers(1, 4)))))
    return ix, iy, iz


@pytest.mark.parametrize("seed", list(range(100, 132)))
def test_uvw_per_sample_random_specs(seed):
    """Forward, backward and second-order pass (one fused kernel) on seeded random irreps (fp64: any wrong index
    shows at 1e-10)."""
    from oracle.irreps import enumerate_paths, parse_irreps
    from paper_2501_13986_amd import binding as b
    ix, iy, iz = _random_spec(seed)
    if not enumerate_paths(parse_irreps(ix), parse_irreps(iy), parse_irreps(iz)):
        pytest.skip(f"no allowed path for {ix} x {iy} -> {iz}")
    spec = TPSpec(ix, iy, iz, mode=UVW, shared_weights=False)
    plan = b.Plan(ix, iy, iz, mode=b.CGTP_UVW, shared_weights=False, dtype=b.CGTP_F64, device=0)
    B = 37
    print(f"seed={seed} spec=({ix}) x ({iy}) -> ({iz}) paths={len(spec.paths)} B={B} entry=tp_forward/backward/double_backward (uvw per-sample)", flush=True)
    rng = np.random.default_rng(seed + 1000)
    x, y, gz = rng.normal(size=(B, spec.dim_x)), rng.normal(size=(B, spec.dim_y)), rng.normal(size=(B, spec.dim_z))
    W, La, Lb, LC = rng.normal(size=(B, spec.n_w)), rng.normal(size=(B, spec.dim_x)), rng.normal(size=(B, spec.dim_y)), rng.normal(size=(B, spec.n_w))
    def out(d):
        return torch.full((B + 1, d), 7.0, dtype=torch.float64, device="cuda")
    z = out(spec.dim_z); b.tp_forward(plan, dev(x), dev(y), dev(W), z, B=B)
    gx, gy, gW = out(spec.dim_x), out(spec.dim_y), out(spec.n_w)
    b.tp_backward(plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW, B=B)
    Lx, Ly, LW, Lgz = out(spec.dim_x), out(spec.dim_y), out(spec.n_w), out(spec.dim_z)
    b.tp_double_backward(plan, dev(x), dev(y), dev(W), dev(gz), dev(La), dev(Lb), dev(LC), Lx, Ly, LW, Lgz, B=B)
    torch.cuda.synchronize()
    for t in (z, gx, gy, gW, Lx, Ly, LW, Lgz):
        assert torch.all(t[B:] == 7.0)
    assert_close(z[:B].cpu().numpy(), otp.forward(spec, x, y, W), "f64", "z")
    for g, r, what in zip((gx, gy, gW), otp.backward(spec, x, y, W, gz), ("gx", "gy", "gW")):
        assert_close(g[:B].cpu().numpy(), r, "f64", what)
    for g, r, what in zip((Lx, Ly, LW, Lgz), otp.double_backward(spec, x, y, W, gz, La, Lb, LC), ("dL/dx", "dL/dy", "dL/dW", "dL/dgz")):
        assert_close(g[:B].cpu().numpy(), r, "f64", what)


def test_uvw_empty_batches():
    """B = 0: nothing is read or written (shared weights: gW is the empty sum, zero)."""
    from paper_2501_13986_amd import binding as b
    for shared in (True, False):
        plan = b.Plan("16x0e+16x1o", "1x0e+1x1o", "16x0e+16x1o+16x1e", mode=b.CGTP_UVW, shared_weights=shared, device=0)
        x = torch.zeros((0, plan.dim_x), device="cuda"); y = torch.zeros((0, plan.dim_y), device="cuda")
        W = torch.ones((plan.n_w,) if shared else (1, plan.n_w), device="cuda")
        z = torch.full((1, plan.dim_z), 7.0, device="cuda")
        b.tp_forward(plan, x, y, W, z, B=0)
        gx = torch.full((1, plan.dim_x), 7.0, device="cuda"); gy = torch.full((1, plan.dim_y), 7.0, device="cuda")
        gW = torch.full((plan.n_w,) if shared else (1, plan.n_w), 7.0, device="cuda")
        b.tp_backward(plan, x, y, W, z, gx, gy, gW, B=0)
        torch.cuda.synchronize()
        assert torch.all(z == 7.0) and torch.all(gx == 7.0) and torch.all(gy == 7.0)
        assert torch.all(gW == (0.0 if shared else 7.0))


def test_uvw_unsupported_cases_are_reported():
    from paper_2501_13986_amd import binding as b
    for args, kw in [(("6x0e", "1x0e", "16x0e"), {}),                 # mul_x not a multiple of 4
                     (("4x0e", "1x0e", "8x0e"), {}),                  # mul_z not a multiple of 16
                     ((synth.NEQUIP_X, synth.NEQUIP_Y, synth.NEQUIP_Z), {"dtype": b.CGTP_F64}),
                     (("128x0e", "1x0e", "16x0e"), {"shared_weights": False})]:   # per-sample weights: multiplicity above 64
        with pytest.raises(b.CgtpError) as e:
            b.Plan(*args, mode=b.CGTP_UVW, device=-1, **{"shared_weights": True, **kw})
        assert e.value.status == 2
    plan = b.Plan("4x0e+4x1o", "1x0e+1x1o", "16x0e+16x1o+16x1e", mode=b.CGTP_UVW, shared_weights=True, device=0)
    assert b.lib().tp_backward(plan._h, 16, 16, 16, 16, 16, 16, 16, 4, None) == 2   # backward needs mul_x % 16 == 0
