"""The entry points are plain asynchronous launches on the caller's stream, so a whole step can be
recorded into a HIP graph and replayed.  Checked here: every replay reproduces the eager results
bit for bit (the kernels are deterministic), with eager work and synchronisations between replays."""
import numpy as np
import pytest

from paper_2501_13986_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_step_replays_from_a_hip_graph():
    from paper_2501_13986_amd import binding as b
    irr = (synth.MACE_X, synth.MACE_Y, synth.MACE_Z)
    plan = b.Plan(*irr, dtype=b.CGTP_F32, device=0)
    DX, DY, DZ, NW = plan.dim_x, plan.dim_y, plan.dim_z, plan.n_w
    B, V = 777, 300
    recv, send, unit = synth.periodic_graph(11, V, 20.0)
    E = recv.shape[0]
    print(f"graph capture: B={B} V={V} E={E} entries=tp_forward/tp_backward/conv_forward/conv_backward", flush=True)
    dev = "cuda"
    row_ptr, col, perm, t_row_ptr, t_perm = b.cgtp_csr_from_coo(torch.from_numpy(recv).to(dev), torch.from_numpy(send).to(dev), V)
    g = torch.Generator(device=dev)
    g.manual_seed(5)
    rnd = lambda *shape: torch.randn(shape, generator=g, device=dev, dtype=torch.float32)
    x, y, W, gz = rnd(B, DX), rnd(B, DY), rnd(B, NW), rnd(B, DZ)
    xn, ye, We, gzn = rnd(V, DX), rnd(E, DY), rnd(E, NW), rnd(V, DZ)
    outs = {"z": torch.empty(B, DZ, device=dev), "gx": torch.empty(B, DX, device=dev), "gy": torch.empty(B, DY, device=dev),
            "gW": torch.empty(B, NW, device=dev), "zn": torch.empty(V, DZ, device=dev), "gxn": torch.empty(V, DX, device=dev),
            "gye": torch.empty(E, DY, device=dev), "gWe": torch.empty(E, NW, device=dev)}

    def step():
        b.tp_forward(plan, x, y, W, outs["z"])
        b.tp_backward(plan, x, y, W, gz, outs["gx"], outs["gy"], outs["gW"])
        b.conv_forward(plan, xn, ye, We, outs["zn"], row_ptr, col)
        b.conv_backward(plan, xn, ye, We, gzn, outs["gxn"], outs["gye"], outs["gWe"], row_ptr, col, t_row_ptr, t_perm)

    step()                       # eager: also sizes the plan's workspace, which must not grow during capture
    torch.cuda.synchronize()
    eager = {k: v.clone() for k, v in outs.items()}
    side = torch.cuda.Stream()   # default priority
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                   # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(3):
        for v in outs.values():
            v.fill_(float("nan"))            # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in outs:
            assert torch.equal(outs[k], eager[k]), (rep, k)
