"""GPU parity of the transposed segment layout (plan flag CGTP_IR_MUL: index (m+l)*mul + u inside a segment, the
alternative the paper's Sec. 4 "data layout" discusses) against the CPU oracle.  The oracle works in the default layout;
the test carries x, gz and the incoming second-order gradients into the transposed layout with an index array and the
results back, so every entry point of a uvu plan is compared element by element."""
import numpy as np
import pytest

from oracle import conv as oconv, tp as otp
from oracle.irreps import TPSpec, Path
from paper_2501_13986_amd import synth
from tests._util import assert_close, ir_mul_index
from tests.test_gpu_tp import CASES

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _b():
    from paper_2501_13986_amd import binding
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def make(name, prec):
    b = _b()
    ix, iy, iz, paths = CASES[name]
    spec = TPSpec(ix, iy, iz, paths=None if paths is None else
                  [Path(p[0], p[1], p[2], 0, p[4] if len(p) > 4 else 1.0) for p in paths])
    plan = b.Plan(ix, iy, iz, paths=paths, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0, flags=b.CGTP_IR_MUL)
    return b, spec, plan, ir_mul_index(spec.irx), ir_mul_index(spec.irz)


def back(t, idx):
    """A result in the transposed layout, as a numpy array in the default layout."""
    a = t.cpu().numpy()
    out = np.empty_like(a)
    out[:, idx] = a
    return out


@pytest.mark.parametrize("prec", ["f64", "f32"])
@pytest.mark.parametrize("name", ["mace", "mixed_mul", "mul3_odd", "mul192_two_passes", "unused_segments", "mul2", "l4"])
def test_batched_forward_backward_ir_mul(name, prec):
    B = 133
    b, spec, plan, px, pz = make(name, prec)
    print(f"case={name} prec={prec} B={B} layout=IR_MUL entry=tp_forward/tp_backward", flush=True)
    npdt, tdt = (np.float64, torch.float64) if prec == "f64" else (np.float32, torch.float32)
    x = synth.normal(21, (B, spec.dim_x)).astype(npdt); y = synth.normal(22, (B, spec.dim_y)).astype(npdt)
    W = synth.normal(23, (B, spec.n_w)).astype(npdt); gz = synth.normal(24, (B, spec.dim_z)).astype(npdt)
    z = torch.full((B, spec.dim_z), float("nan"), dtype=tdt, device="cuda")
    gx = torch.full((B, spec.dim_x), float("nan"), dtype=tdt, device="cuda")
    gy = torch.full((B, spec.dim_y), float("nan"), dtype=tdt, device="cuda")
    gW = torch.full((B, spec.n_w), float("nan"), dtype=tdt, device="cuda")
    b.tp_forward(plan, dev(x[:, px]), dev(y), dev(W), z)
    b.tp_backward(plan, dev(x[:, px]), dev(y), dev(W), dev(gz[:, pz]), gx, gy, gW)
    torch.cuda.synchronize()
    assert_close(back(z, pz), otp.forward(spec, x, y, W), prec, "z")
    rx, ry, rW = otp.backward(spec, x, y, W, gz)
    assert_close(back(gx, px), rx, prec, "gx")
    assert_close(gy.cpu().numpy(), ry, prec, "gy")
    assert_close(gW.cpu().numpy(), rW, prec, "gW")


@pytest.mark.parametrize("name", ["mace", "mixed_mul"])
def test_double_backward_ir_mul(name):
    B, prec = 67, "f64"
    b, spec, plan, px, pz = make(name, prec)
    print(f"case={name} B={B} layout=IR_MUL entry=tp_double_backward", flush=True)
    x = synth.normal(31, (B, spec.dim_x)); y = synth.normal(32, (B, spec.dim_y)); W = synth.normal(33, (B, spec.n_w))
    gz = synth.normal(34, (B, spec.dim_z)); La = synth.normal(35, (B, spec.dim_x)); Lb = synth.normal(36, (B, spec.dim_y))
    LC = synth.normal(37, (B, spec.n_w))
    Lx = torch.full((B, spec.dim_x), float("nan"), dtype=torch.float64, device="cuda")
    Ly = torch.full((B, spec.dim_y), float("nan"), dtype=torch.float64, device="cuda")
    LW = torch.full((B, spec.n_w), float("nan"), dtype=torch.float64, device="cuda")
    Lgz = torch.full((B, spec.dim_z), float("nan"), dtype=torch.float64, device="cuda")
    b.tp_double_backward(plan, dev(x[:, px]), dev(y), dev(W), dev(gz[:, pz]), dev(La[:, px]), dev(Lb), dev(LC), Lx, Ly, LW, Lgz)
    torch.cuda.synchronize()
    rx, ry, rW, rgz = otp.double_backward(spec, x, y, W, gz, La, Lb, LC)
    assert_close(back(Lx, px), rx, prec, "Lx")
    assert_close(Ly.cpu().numpy(), ry, prec, "Ly")
    assert_close(LW.cpu().numpy(), rW, prec, "LW")
    assert_close(back(Lgz, pz), rgz, prec, "Lgz")


@pytest.mark.parametrize("prec", ["f64", "f32"])
@pytest.mark.parametrize("name", ["mace", "mixed_mul"])
def test_convolution_ir_mul(name, prec):
    """Fused convolution forward and backward (deterministic and atomic variants) in the transposed layout, on a
    small skewed graph with split and empty rows."""
    b, spec, plan, px, pz = make(name, prec)
    V = 150
    recv, send, unit = synth.periodic_graph(41, V, 11.0)
    keep = recv % 7 != 3                      # some nodes receive nothing
    recv, send = recv[keep], send[keep]
    row_ptr, col, perm, t_row_ptr, t_perm = oconv.csr_from_coo(recv, send, V)
    E = col.shape[0]
    print(f"case={name} prec={prec} V={V} E={E} layout=IR_MUL entry=conv_forward/conv_backward(+atomic)", flush=True)
    npdt, tdt = (np.float64, torch.float64) if prec == "f64" else (np.float32, torch.float32)
    x = synth.normal(42, (V, spec.dim_x)).astype(npdt); y = synth.normal(43, (E, spec.dim_y)).astype(npdt)
    W = synth.normal(44, (E, spec.n_w)).astype(npdt); gz = synth.normal(45, (V, spec.dim_z)).astype(npdt)
    z = torch.full((V, spec.dim_z), float("nan"), dtype=tdt, device="cuda")
    gx = torch.full((V, spec.dim_x), float("nan"), dtype=tdt, device="cuda")
    gy = torch.full((E, spec.dim_y), float("nan"), dtype=tdt, device="cuda")
    gW = torch.full((E, spec.n_w), float("nan"), dtype=tdt, device="cuda")
    g = [dev(a) for a in (row_ptr, col, t_row_ptr, t_perm)]
    dx, dy, dW, dgz = dev(x[:, px]), dev(y), dev(W), dev(gz[:, pz])
    ref = oconv.forward(spec, x, y, W, row_ptr, col)
    rx, ry, rW = oconv.backward(spec, x, y, W, gz, row_ptr, col)
    b.conv_forward(plan, dx, dy, dW, z, g[0], g[1])
    b.conv_backward(plan, dx, dy, dW, dgz, gx, gy, gW, g[0], g[1], g[2], g[3])
    torch.cuda.synchronize()
    assert_close(back(z, pz), ref, prec, "z")
    assert_close(back(gx, px), rx, prec, "gx")
    assert_close(gy.cpu().numpy(), ry, prec, "gy")
    assert_close(gW.cpu().numpy(), rW, prec, "gW")
    # the variant for unsorted edge lists: CSR order is one valid edge order, receivers / senders given per edge
    rows = oconv.rows_of_edges(row_ptr)
    z.fill_(float("nan")); gx.fill_(float("nan")); gy.fill_(float("nan")); gW.fill_(float("nan"))
    b.conv_forward_atomic(plan, dx, dy, dW, z, dev(rows), g[1])
    b.conv_backward_atomic(plan, dx, dy, dW, dgz, gx, gy, gW, dev(rows), g[1])
    torch.cuda.synchronize()
    assert_close(back(z, pz), ref, prec, "z atomic")
    assert_close(back(gx, px), rx, prec, "gx atomic")
    assert_close(gy.cpu().numpy(), ry, prec, "gy atomic")
    assert_close(gW.cpu().numpy(), rW, prec, "gW atomic")
