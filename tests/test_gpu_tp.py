"""GPU parity of the batched tensor product (forward and backward) against the CPU oracle,
element by element on the same seeded inputs, through the C ABI."""
import numpy as np
import pytest

from oracle import tp as otp
from oracle.irreps import TPSpec, Path
from paper_2501_13986_amd import synth
from tests._util import assert_close

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _b():
    from paper_2501_13986_amd import binding
    return binding


TINY_PATHS = [(0, 0, 0), (0, 1, 1), (1, 0, 2), (1, 1, 3), (1, 1, 4), (1, 1, 5)]

# name -> (irreps x, y, z, explicit paths or None)
CASES = {
    "tiny_separate": (synth.TINY_X, synth.TINY_Y, synth.TINY_Z, TINY_PATHS),
    "tiny_merged": (synth.TINY_X, synth.TINY_Y, synth.TINY_Z_MERGED, None),
    "mace": (synth.MACE_X, synth.MACE_Y, synth.MACE_Z, None),
    "mul3_odd": ("3x0e+3x1o+3x2e", "1x0e+1x1o+1x2e+1x3o", "3x0e+3x1o+3x2e+3x3o+3x1e", None),
    "mixed_mul": ("8x0e+4x1o+2x2e", "1x0e+1x1o+1x2e", "8x0e+4x1o+2x2e+4x1e+4x2e",
                  [(0, 0, 0), (1, 0, 1), (1, 1, 3), (1, 1, 4), (1, 2, 1), (2, 0, 2), (2, 2, 2)]),
    "mul96": ("96x0e+96x1o", "1x0e+1x1o+1x2e", "96x0e+96x1o+96x2e", None),
    "mul192_two_passes": ("192x0e+192x1o", "1x0e+1x1o", "192x0e+192x1o+192x1e", None),
    "l4": ("2x4e+2x3o", "1x2e+1x4e", "2x4e+2x2e+2x3o+2x5o", None),
    "coeff": ("6x1o", "1x1o", "6x0e+6x2e", [(0, 0, 0, 0, 0.5), (0, 0, 1, 0, -2.0)]),
    "unused_segments": ("4x0e+4x1o+4x2e", "1x0e+1x1o", "4x3o+4x0e+4x1o", [(1, 1, 1), (0, 1, 2)]),
    # one and two channels: a wave holds 64 / 32 samples, the cross-lane sums degenerate
    "mul1": ("1x0e+1x1o+1x2e", "1x0e+1x1o+1x2e", "1x0e+1x1o+1x2e+1x3o", None),
    "mul2": ("2x0e+2x1o", "1x0e+1x1o", "2x0e+2x1o+2x1e+2x2e", None),
    # 68 paths: the planner has to leave its default schedule to keep the kernels out of private memory
    "many_paths": (synth.MANY_X, synth.MANY_Y, synth.MANY_X, None),
}


def make(name, prec, B, seed=0):
    b = _b()
    ix, iy, iz, paths = CASES[name]
    spec = TPSpec(ix, iy, iz, paths=None if paths is None else
                  [Path(p[0], p[1], p[2], 0, p[4] if len(p) > 4 else 1.0) for p in paths])
    plan = b.Plan(ix, iy, iz, paths=paths, dtype=b.CGTP_F64 if prec == "f64" else b.CGTP_F32, device=0)
    assert (plan.dim_x, plan.dim_y, plan.dim_z, plan.n_w) == (spec.dim_x, spec.dim_y, spec.dim_z, spec.n_w)
    npdt = np.float64 if prec == "f64" else np.float32
    x = synth.normal(seed + 1, (B, spec.dim_x)).astype(npdt)
    y = synth.normal(seed + 2, (B, spec.dim_y)).astype(npdt)
    W = synth.normal(seed + 3, (B, spec.n_w)).astype(npdt)
    gz = synth.normal(seed + 4, (B, spec.dim_z)).astype(npdt)
    return b, spec, plan, (x, y, W, gz)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("prec", ["f64", "f32"])
@pytest.mark.parametrize("name", list(CASES))
def test_forward_parity(name, prec):
    B = 1000 if name.startswith("tiny") else 261
    b, spec, plan, (x, y, W, gz) = make(name, prec, B)
    print(f"case={name} prec={prec} B={B} entry=tp_forward", flush=True)
    z = torch.full((B, spec.dim_z), float("nan"), dtype=torch.float64 if prec == "f64" else torch.float32, device="cuda")
    b.tp_forward(plan, dev(x), dev(y), dev(W), z)
    torch.cuda.synchronize()
    ref = otp.forward(spec, x, y, W)      # oracle in fp64 on the same (possibly fp32-rounded) inputs
    assert_close(z.cpu().numpy(), ref, prec, f"{name} forward")


@pytest.mark.parametrize("prec", ["f64", "f32"])
@pytest.mark.parametrize("name", list(CASES))
def test_backward_parity(name, prec):
    B = 1000 if name.startswith("tiny") else 261
    b, spec, plan, (x, y, W, gz) = make(name, prec, B, seed=10)
    print(f"case={name} prec={prec} B={B} entry=tp_backward", flush=True)
    tdt = torch.float64 if prec == "f64" else torch.float32
    gx = torch.full((B, spec.dim_x), float("nan"), dtype=tdt, device="cuda")
    gy = torch.full((B, spec.dim_y), float("nan"), dtype=tdt, device="cuda")
    gW = torch.full((B, spec.n_w), float("nan"), dtype=tdt, device="cuda")
    b.tp_backward(plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW)
    torch.cuda.synchronize()
    rx, ry, rW = otp.backward(spec, x, y, W, gz)
    # segments of x / y that no path reads have zero gradient in the oracle; the library writes
    # zeros for unused x segments and leaves unused y words untouched only if there are none
    assert_close(gx.cpu().numpy(), rx, prec, f"{name} gx")
    assert_close(gW.cpu().numpy(), rW, prec, f"{name} gW")
    assert_close(gy.cpu().numpy(), ry, prec, f"{name} gy")


@pytest.mark.parametrize("B", [0, 1, 3, 64, 65])
def test_ragged_and_empty_batches(B):
    b, spec, plan, (x, y, W, gz) = make("mixed_mul", "f64", max(B, 1))
    print(f"case=mixed_mul B={B} entry=tp_forward/tp_backward", flush=True)
    x, y, W, gz = x[:B], y[:B], W[:B], gz[:B]
    z = torch.full((max(B, 1) + 1, spec.dim_z), 7.0, dtype=torch.float64, device="cuda")   # one guard row
    gx = torch.full((max(B, 1) + 1, spec.dim_x), 7.0, dtype=torch.float64, device="cuda")
    gy = torch.full((max(B, 1) + 1, spec.dim_y), 7.0, dtype=torch.float64, device="cuda")
    gW = torch.full((max(B, 1) + 1, spec.n_w), 7.0, dtype=torch.float64, device="cuda")
    dx, dy, dW, dgz = (dev(a) if B else torch.zeros((1, a.shape[1]), dtype=torch.float64, device="cuda") for a in (x, y, W, gz))
    b.tp_forward(plan, dx, dy, dW, z, B=B)
    b.tp_backward(plan, dx, dy, dW, dgz, gx, gy, gW, B=B)
    torch.cuda.synchronize()
    for t in (z, gx, gy, gW):
        assert torch.all(t[B:] == 7.0)          # nothing written past the batch
    if B:
        assert_close(z[:B].cpu().numpy(), otp.forward(spec, x, y, W), "f64", "forward")
        rx, ry, rW = otp.backward(spec, x, y, W, gz)
        assert_close(gx[:B].cpu().numpy(), rx, "f64", "gx")
        assert_close(gy[:B].cpu().numpy(), ry, "f64", "gy")
        assert_close(gW[:B].cpu().numpy(), rW, "f64", "gW")


def test_bad_arguments():
    b, spec, plan, (x, y, W, gz) = make("tiny_merged", "f64", 4)
    L = b.lib()
    assert L.tp_forward(plan._h, None, None, None, None, 4, None) == 1
    assert L.tp_forward(plan._h, None, None, None, None, -1, None) == 1
    dx = dev(x)
    assert L.tp_forward(plan._h, dx.data_ptr() + 8, dx.data_ptr(), dx.data_ptr(), dx.data_ptr(), 1, None) == 1
    assert L.tp_forward(None, 16, 16, 16, 16, 4, None) == 1


def test_kernel_info_reports_no_spills():
    b, spec, plan, _ = make("mace", "f32", 1)
    for k in range(4):
        info = plan.kernel_info(k)
        assert info["scratch"] == 0, (k, info)
        assert info["blocks_per_cu"] >= 1


@pytest.mark.parametrize("env", [{"CGTP_PHASES_TP_BWD": "3", "CGTP_PIN_PER_PATH": "2", "CGTP_FRESH_Y": "1", "CGTP_UPFRONT_TP_BWD": "0"},
                                 {"CGTP_PHASES_TP_BWD": "2"}, {"CGTP_W_UPFRONT_FWD": "0", "CGTP_FRESH_Y": "1"}])
@pytest.mark.parametrize("name", ["mace", "unused_segments", "mixed_mul"])
def test_forced_schedules_give_the_same_results(name, env, monkeypatch):
    """Every code-generation choice the planner can make (phases over x segments, per-path accumulator
    updates, per-path y products, load placement) computes the same thing."""
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    B = 130
    b, spec, plan, (x, y, W, gz) = make(name, "f64", B, seed=50)
    print(f"case={name} env={env} B={B} entry=tp_forward/tp_backward", flush=True)
    z = torch.full((B, spec.dim_z), float("nan"), dtype=torch.float64, device="cuda")
    gx = torch.full((B, spec.dim_x), float("nan"), dtype=torch.float64, device="cuda")
    gy = torch.full((B, spec.dim_y), float("nan"), dtype=torch.float64, device="cuda")
    gW = torch.full((B, spec.n_w), float("nan"), dtype=torch.float64, device="cuda")
    b.tp_forward(plan, dev(x), dev(y), dev(W), z)
    b.tp_backward(plan, dev(x), dev(y), dev(W), dev(gz), gx, gy, gW)
    torch.cuda.synchronize()
    assert_close(z.cpu().numpy(), otp.forward(spec, x, y, W), "f64", "z")
    rx, ry, rW = otp.backward(spec, x, y, W, gz)
    assert_close(gx.cpu().numpy(), rx, "f64", "gx")
    assert_close(gy.cpu().numpy(), ry, "f64", "gy")
    assert_close(gW.cpu().numpy(), rW, "f64", "gW")
