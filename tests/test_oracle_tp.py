"""Pins for oracle/tp.py.

 - brute force: the dense einsum of paper Eq. 1 with P and W assembled entry by entry
 - equivariance under random proper and improper rotations (paper Sec. 2.1), <= 1e-10
 - backward: adjoint identities (exact, TP is multilinear) and central finite differences
 - double backward (paper Sec. 3.4): central finite differences of L(a, b, C) through `backward`
   (exact up to rounding: L is linear in each argument), and a planted-mistake check
 - special cases with a textbook answer: scalar x scalar, vector cross product
 - FLOP model against the figures quoted for the benchmark shapes
"""
import numpy as np
import pytest

from oracle import so3, tp
from oracle.irreps import TPSpec, Path, UVU, UVW, parse_irreps, enumerate_paths
from paper_2501_13986_amd import synth

RNG = np.random.default_rng(2024)

SPECS = {
    "tiny_sep": lambda: TPSpec(synth.TINY_X, synth.TINY_Y, synth.TINY_Z,
                               paths=[Path(ix, iy, iz) for iz, (ix, iy) in
                                      enumerate([(0, 0), (0, 1), (1, 0), (1, 1), (1, 1), (1, 1)])]),
    "tiny_merged": lambda: TPSpec(synth.TINY_X, synth.TINY_Y, synth.TINY_Z_MERGED),
    "small_uvu": lambda: TPSpec("3x0e+3x1o+3x2e", "1x0e+1x1o+1x2e+1x3o", "3x0e+3x1o+3x2e+3x3o+3x1e"),
    "small_uvw": lambda: TPSpec("3x0e+2x1o+4x2e", "1x0e+1x1o+1x2e", "2x0e+3x1o+2x2e", mode=UVW, shared_weights=True),
    "uvw_per_sample": lambda: TPSpec("2x1o+3x2e", "1x1o+1x2e", "2x1e+3x1o", mode=UVW),
    "coeff": lambda: TPSpec("2x1o", "1x1o", "2x0e+2x2e", paths=[Path(0, 0, 0, UVU, 0.5), Path(0, 0, 1, UVU, -2.0)]),
}


def draw(spec, B, rng=RNG):
    x = rng.normal(size=(B, spec.dim_x))
    y = rng.normal(size=(B, spec.dim_y))
    W = rng.normal(size=(spec.n_w,) if spec.shared_weights else (B, spec.n_w))
    return x, y, W


def test_parse_and_paths():
    ir = parse_irreps("128x0e + 128x1o+ 2e")
    assert [(t.mul, t.l, t.p) for t in ir] == [(128, 0, 1), (128, 1, -1), (1, 2, 1)]
    with pytest.raises(ValueError):
        parse_irreps("3x1q")
    with pytest.raises(ValueError):
        parse_irreps("0x1e")
    mace = TPSpec(synth.MACE_X, synth.MACE_Y, synth.MACE_Z)
    assert (mace.dim_x, mace.dim_y, mace.dim_z, mace.n_w, len(mace.paths)) == (1152, 16, 2048, 2176, 17)
    neq = TPSpec(synth.NEQUIP_X, synth.NEQUIP_Y, synth.NEQUIP_Z, mode=UVW, shared_weights=True)
    assert (neq.dim_x, neq.dim_y, neq.dim_z, neq.n_w, len(neq.paths)) == (288, 9, 288, 11264, 11)
    tiny = SPECS["tiny_sep"]()
    assert (tiny.dim_x, tiny.dim_y, tiny.dim_z, tiny.n_w) == (16, 4, 64, 24)
    assert [tiny.ls(q) for q in tiny.paths] == [(0, 0, 0), (0, 1, 1), (1, 0, 1), (1, 1, 0), (1, 1, 1), (1, 1, 2)]
    merged = SPECS["tiny_merged"]()
    assert merged.dim_z == 48 and len(merged.paths) == 6
    # 1o x 1o -> 1o is parity-forbidden, 1o x 1o -> 1e is allowed
    assert (1, 1, 1) not in enumerate_paths(parse_irreps("0e+1o"), parse_irreps("0e+1o"), parse_irreps("0e+1o"))
    with pytest.raises(ValueError):
        TPSpec("2x1o", "1x1o", "2x1o", paths=[Path(0, 0, 0)])
    with pytest.raises(ValueError):
        TPSpec("2x1o", "2x1o", "2x1e")


def test_flop_model():
    assert tp.flops_forward(TPSpec(synth.MACE_X, synth.MACE_Y, synth.MACE_Z)) == 73216
    assert tp.flops_forward(TPSpec(synth.NEQUIP_X, synth.NEQUIP_Y, synth.NEQUIP_Z, mode=UVW)) == 76992
    assert tp.flops_forward(SPECS["tiny_sep"]()) == 344


@pytest.mark.parametrize("name", list(SPECS))
def test_forward_equals_dense_einsum(name):
    spec = SPECS[name]()
    x, y, W = draw(spec, 3)
    z = tp.forward(spec, x, y, W)
    for b in range(3):
        ref = tp.dense_reference(spec, x[b], y[b], W if spec.shared_weights else W[b])
        assert np.abs(z[b] - ref).max() < 1e-12


def test_textbook_special_cases():
    # scalar x scalar -> scalar with one channel is the plain product w*x*y
    s = TPSpec("1x0e", "1x0e", "1x0e")
    assert np.allclose(tp.forward(s, [[2.0]], [[3.0]], [[5.0]]), [[30.0]], atol=1e-15)
    # 1o x 1o -> 1e is the cross product / sqrt2, components stored (y, z, x)
    c = TPSpec("1x1o", "1x1o", "1x1e")
    a, b = RNG.normal(size=3), RNG.normal(size=3)                      # xyz
    yzx = lambda t: np.array([t[1], t[2], t[0]])
    out = tp.forward(c, yzx(a)[None], yzx(b)[None], [[1.0]])[0]
    assert np.abs(out - yzx(np.cross(a, b)) / np.sqrt(2)).max() < 1e-14
    # two paths into one output segment add up
    m = TPSpec("1x0e+1x0e", "1x0e", "1x0e", paths=[Path(0, 0, 0), Path(1, 0, 0)])
    assert np.allclose(tp.forward(m, [[2.0, 7.0]], [[3.0]], [[5.0, 11.0]]), [[2 * 3 * 5 + 7 * 3 * 11.0]])


@pytest.mark.parametrize("name", list(SPECS))
@pytest.mark.parametrize("improper", [False, True])
def test_equivariance(name, improper):
    spec = SPECS[name]()
    x, y, W = draw(spec, 4)
    a, b, g = RNG.uniform(0, 2 * np.pi, 3)
    Dl = lambda l: so3.wigner_D_real(l, a, b, g)
    Dx, Dy, Dz = (so3.block_diag_D(ir, Dl, improper) for ir in (spec.irx, spec.iry, spec.irz))
    lhs = tp.forward(spec, x @ Dx.T, y @ Dy.T, W)
    rhs = tp.forward(spec, x, y, W) @ Dz.T
    assert np.abs(lhs - rhs).max() < 1e-10 * max(1.0, np.abs(rhs).max())
    assert np.abs(rhs).max() > 0.1


@pytest.mark.parametrize("name", list(SPECS))
def test_backward_adjoint_identities(name):
    spec = SPECS[name]()
    B = 4
    x, y, W = draw(spec, B)
    gz = RNG.normal(size=(B, spec.dim_z))
    gx, gy, gW = tp.backward(spec, x, y, W, gz)
    dx, dy, dW = draw(spec, B)
    assert abs(np.sum(gz * tp.forward(spec, dx, y, W)) - np.sum(gx * dx)) < 1e-10
    assert abs(np.sum(gz * tp.forward(spec, x, dy, W)) - np.sum(gy * dy)) < 1e-10
    assert abs(np.sum(gz * tp.forward(spec, x, y, dW)) - np.sum(gW * dW)) < 1e-10
    assert gW.shape == W.shape


@pytest.mark.parametrize("name", ["tiny_sep", "small_uvu", "small_uvw", "uvw_per_sample"])
def test_backward_finite_differences(name):
    spec = SPECS[name]()
    B = 2
    x, y, W = draw(spec, B)
    gz = RNG.normal(size=(B, spec.dim_z))
    gx, gy, gW = tp.backward(spec, x, y, W, gz)
    E = lambda x_, y_, W_: float(np.sum(gz * tp.forward(spec, x_, y_, W_)))
    h = 1e-5
    for arr, grad, which in ((x, gx, 0), (y, gy, 1), (W, gW, 2)):
        flat = arr.reshape(-1)
        idx = RNG.choice(flat.size, size=min(flat.size, 12), replace=False)
        for t in idx:
            old = flat[t]
            flat[t] = old + h; ep = E(x, y, W)
            flat[t] = old - h; em = E(x, y, W)
            flat[t] = old
            fd = (ep - em) / (2 * h)
            assert abs(fd - grad.reshape(-1)[t]) < 1e-7 * max(1.0, abs(fd)), (which, t)


def _scalar_L(spec, x, y, W, gz, La, Lb, LC):
    a, b, C = tp.backward(spec, x, y, W, gz)
    return float(np.sum(La * a) + np.sum(Lb * b) + np.sum(LC * C))


@pytest.mark.parametrize("name", ["tiny_sep", "tiny_merged", "small_uvu", "uvw_per_sample", "coeff"])
def test_double_backward_finite_differences(name):
    """dL/d(x, y, W, gz) of L = <La, a> + <Lb, b> + <LC, C>, (a, b, C) = backward(x, y, W, gz),
    against central differences of L evaluated through the (pinned) backward."""
    spec = SPECS[name]()
    B = 2
    x, y, W = draw(spec, B)
    gz = RNG.normal(size=(B, spec.dim_z))
    La, Lb, LC = draw(spec, B)
    grads = tp.double_backward(spec, x, y, W, gz, La, Lb, LC)
    args = [x, y, W, gz]
    h = 1e-3     # L is linear in each single entry, so the step only has to beat rounding
    for which, (arr, grad) in enumerate(zip(args, grads)):
        assert grad.shape == arr.shape
        flat = arr.reshape(-1)
        idx = RNG.choice(flat.size, size=min(flat.size, 16), replace=False)
        for t in idx:
            old = flat[t]
            flat[t] = old + h; lp = _scalar_L(spec, *args, La, Lb, LC)
            flat[t] = old - h; lm = _scalar_L(spec, *args, La, Lb, LC)
            flat[t] = old
            fd = (lp - lm) / (2 * h)
            assert abs(fd - grad.reshape(-1)[t]) < 1e-9 * max(1.0, abs(fd)), (which, t, fd, grad.reshape(-1)[t])
        assert np.abs(grad).max() > 1e-3


def test_double_backward_each_input_matters():
    """Every one of the three incoming gradients reaches every output it should (a dropped
    dispatch would leave a zero block): the Jacobian structure of paper Sec. 3.4."""
    spec = SPECS["small_uvu"]()
    B = 3
    x, y, W = draw(spec, B)
    gz = RNG.normal(size=(B, spec.dim_z))
    La, Lb, LC = draw(spec, B)
    z0 = [np.zeros_like(La), np.zeros_like(Lb), np.zeros_like(LC)]
    for t, inc in enumerate((La, Lb, LC)):
        only = list(z0)
        only[t] = inc
        gx, gy, gW, ggz = tp.double_backward(spec, x, y, W, gz, *only)
        nz = [np.abs(g).max() > 1e-6 for g in (gx, gy, gW, ggz)]
        # a = dE/dx does not depend on x, b not on y, C not on W: that block is exactly zero
        expect = [True, True, True, True]
        expect[t] = False
        assert nz == expect, (t, nz)
    # symmetry of second derivatives: d<La,a>/dy contracted with Lb equals d<Lb,b>/dx contracted with La
    g1 = tp.double_backward(spec, x, y, W, gz, La, z0[1], z0[2])
    g2 = tp.double_backward(spec, x, y, W, gz, z0[0], Lb, z0[2])
    assert abs(np.sum(g1[1] * Lb) - np.sum(g2[0] * La)) < 1e-10
