"""conv_forward_static, the entry point that allocates nothing (its side buffer is a static device array of the
library), against conv_forward through the C ABI: bit-identical results (same kernels, same edge ranges) and parity
with the CPU oracle, on two calls in a row of which the second has the smaller input; the size limit is an error."""
import numpy as np
import pytest

from oracle import conv as oconv
from oracle.irreps import TPSpec
from paper_2501_13986_amd import synth
from tests._util import assert_close

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("prec", ["f32", "f64"])
def test_conv_forward_static_matches_conv_forward(prec):
    from paper_2501_13986_amd import binding as b
    irr = (synth.MACE_X, synth.MACE_Y, synth.MACE_Z)
    spec = TPSpec(*irr)
    plan = b.Plan(*irr, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0)
    npdt, tdt = (np.float64, torch.float64) if prec == "f64" else (np.float32, torch.float32)
    for call, (V, deg, seed) in enumerate([(900, 30.0, 61), (260, 12.0, 62)]):     # second call: smaller input
        recv, send, unit = synth.periodic_graph(seed, V, deg)
        row_ptr, col, perm, _, _ = oconv.csr_from_coo(recv, send, V)
        E = col.shape[0]
        print(f"prec={prec} call={call} V={V} E={E} entry=conv_forward_static", flush=True)
        x = synth.normal(seed + 1, (V, spec.dim_x)).astype(npdt)
        y = synth.sh_edge_attr(unit[perm], 3).astype(npdt)
        W = synth.normal(seed + 2, (E, spec.n_w)).astype(npdt)
        dx, dy, dW, drp, dcol = dev(x), dev(y), dev(W), dev(row_ptr), dev(col)
        z_ref = torch.full((V, spec.dim_z), float("nan"), dtype=tdt, device="cuda")
        z = torch.full((V, spec.dim_z), float("nan"), dtype=tdt, device="cuda")
        b.conv_forward(plan, dx, dy, dW, z_ref, drp, dcol)
        torch.cuda.synchronize()
        before, free_before = torch.cuda.memory_allocated(), torch.cuda.mem_get_info()[0]
        b.conv_forward_static(plan, dx, dy, dW, z, drp, dcol)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        if call > 0:     # (the very first use of the library on a GPU loads its code, and with it the static array)
            assert torch.cuda.mem_get_info()[0] >= free_before, "device memory was allocated"
        assert torch.equal(z, z_ref), "conv_forward_static differs from conv_forward"
        assert_close(z.cpu().numpy(), oconv.forward(spec, x, y, W, row_ptr, col), prec, "z")


def test_conv_forward_static_refuses_what_does_not_fit():
    """A plan with 256 channels needs 64 MiB of side buffer on a full GPU: more than the static array holds."""
    from paper_2501_13986_amd import binding as b
    irr = ("256x0e+256x1o+256x2e", synth.MACE_Y, "256x0e+256x1o+256x2e+256x3o")
    plan = b.Plan(*irr, dtype=b.CGTP_F32, device=0)
    V = 4000
    recv, send, unit = synth.periodic_graph(63, V, 8.0)
    row_ptr, col, perm, _, _ = oconv.csr_from_coo(recv, send, V)
    E = col.shape[0]
    print(f"V={V} E={E} entry=conv_forward_static (too large)", flush=True)
    x = torch.zeros((V, plan.dim_x), device="cuda"); y = torch.zeros((E, plan.dim_y), device="cuda")
    W = torch.zeros((E, plan.n_w), device="cuda"); z = torch.zeros((V, plan.dim_z), device="cuda")
    with pytest.raises(b.CgtpError) as ei:
        b.conv_forward_static(plan, x, y, W, z, dev(row_ptr), dev(col))
    assert ei.value.status == 1 and "static buffer holds" in str(ei.value)
    b.conv_forward(plan, x, y, W, z, dev(row_ptr), dev(col))      # the ordinary entry point takes it
    torch.cuda.synchronize()
    assert torch.all(z == 0)
