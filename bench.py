"""Benchmark of the CG tensor product hot path on one MI355X.

One "step" runs the whole hot path once on the MACE-shaped problem (x 128x0e+128x1o+128x2e,
y 1x0e+..+1x3o, 17 uvu paths), inputs resident in HBM: batched forward and backward on 50 000
samples (config 2), then the fused convolution forward and backward on the largest graph of the
benchmark set, 20 000 nodes / ~800 000 edges (config 5).  The step is timed in fp32 (`value`,
`ms_per_step`, `roofline`) and then again in fp64 (`step_f64`, `roofline_f64`).  After the timed
regions the same kernels are timed one by one on the 5 000-node / ~160 000-edge graph (config 4,
both precisions) and the fully connected uvw product of config 3 (fp32, matrix cores); every
configuration is a row of "kernels" with its time (HIP events on the launch stream), GFLOP/s of
nonzero flops, edges/s and the fraction of the roofline that binds it.  --extra adds the variants
(double backward, atomic and unsorted-edge convolution, compensated sums, per-sample uvw, ...).
The CPU oracle is timed on a bounded sample of the same step.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--extra] [--no-cpu] [--calib-copy] [--step-only]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
VALU_PEAK_TFLOPS = {"f32": 78.6, "f64": 78.6}   # 256 CU x 4 SIMD x 16 lanes x 2 flop x 2.4 GHz, plain (unpacked) FMA
MFMA_F32_PEAK_TFLOPS = 157.3
TRAFFIC_FILE = {"f32": "hbm_traffic_step_f32.txt", "f64": "hbm_traffic_step_f64.txt"}


def measured_traffic(kernel: str, prec: str):
    """HBM bytes per launch of `kernel` in the step of precision `prec`, from the committed rocprofv3 counter summary
    of this same command (profiles/hbm_traffic_step_<prec>.txt, lines "kernel fetch_bytes write_bytes"; two --pmc runs,
    FETCH_SIZE and WRITE_SIZE, scaled by the 1 GiB device copy of --calib-copy), or None.  Not measured in this run:
    counters need the profiler."""
    path = os.path.join(ROOT, "profiles", TRAFFIC_FILE[prec])
    try:
        for ln in open(path):
            t = ln.split()
            if len(t) >= 3 and t[0] == kernel:
                return int(float(t[1]) + float(t[2]))
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--extra", action="store_true", help="also time every configuration (fp32/fp64, both graphs)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--calib-copy", action="store_true", help="also run one 1 GiB device copy (counter calibration)")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay timing of the step")
    ap.add_argument("--only", default="", help="comma list of extra rows to run, e.g. cfg5_f32 (default all)")
    ap.add_argument("--step-only", action="store_true", help="time the fp32 step only (for per-kernel profiles of the step)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2501_13986_amd import binding as b, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    irr = (synth.MACE_X, synth.MACE_Y, synth.MACE_Z)

    def tdt(prec):
        return torch.float32 if prec == "f32" else torch.float64

    def esz(prec):
        return 4 if prec == "f32" else 8

    def gauss(seed, shape, prec):
        g = torch.Generator(device=dev)
        g.manual_seed(seed)
        return torch.randn(shape, generator=g, device=dev, dtype=tdt(prec))

    def sh_of_units(seed, n, prec):
        return torch.from_numpy(synth.sh_edge_attr(synth.unit_vectors(seed, n), 3)).to(dev, tdt(prec))

    class Graph:
        def __init__(self, seed, V, deg, node_order="random"):
            recv, send, unit = synth.periodic_graph(seed, V, deg, node_order=node_order)
            self.V, self.E = V, recv.shape[0]
            r = torch.from_numpy(recv).to(dev)
            s = torch.from_numpy(send).to(dev)
            self.recv, self.send = r, s           # generator's edge order (not sorted by receiver)
            self.row_ptr, self.col, self.perm, self.t_row_ptr, self.t_perm = b.cgtp_csr_from_coo(r, s, V)
            self.y64 = torch.from_numpy(synth.sh_edge_attr(unit, 3)).to(dev)[self.perm]

    plans = {}

    def plan(prec):
        if prec not in plans:
            plans[prec] = b.Plan(*irr, dtype=b.CGTP_F32 if prec == "f32" else b.CGTP_F64, device=0)
        return plans[prec]

    P32 = plan("f32")
    F_FWD, F_BWD = P32.flops(0), P32.flops(1)
    DX, DY, DZ, NW = P32.dim_x, P32.dim_y, P32.dim_z, P32.n_w

    def bytes_model(kind, prec, n, V=0):
        s = esz(prec)
        if kind == "tp_fwd":
            return n * (DX + DY + NW + DZ) * s
        if kind == "tp_bwd":
            return n * (2 * DX + 2 * DY + 2 * NW + DZ) * s
        if kind == "conv_fwd":
            return n * (DY + NW) * s + V * (DX + DZ) * s
        if kind == "conv_bwd":
            return n * (2 * DY + 2 * NW) * s + V * (2 * DX + DZ) * s
        raise ValueError(kind)

    def row(name, kind, prec, ms, n, V=0):
        atomic = kind.endswith("_atomic")
        kind = kind.replace("_atomic", "")
        fl = n * (F_FWD if kind.endswith("fwd") else F_BWD)
        by = bytes_model(kind, prec, n, V)
        gbs = by / ms / 1e6
        tfl = fl / ms / 1e9
        t_hbm = by / (HBM_PEAK_GBS * 1e9) * 1e3
        t_alu = fl / (VALU_PEAK_TFLOPS[prec] * 1e12) * 1e3
        r = {"name": name, "kernel": kind + ("_atomic" if atomic else ""), "dtype": prec, "units": n, "ms": round(ms, 4),
             "gflops": round(tfl * 1e3, 1), "alg_gbs": round(gbs, 1),
             "frac_hbm": round(gbs / HBM_PEAK_GBS, 4), "frac_valu": round(tfl / VALU_PEAK_TFLOPS[prec], 4),
             "binding": "hbm" if t_hbm >= t_alu else "alu",
             "frac_binding": round(max(t_hbm, t_alu) / ms, 4)}
        if kind.startswith("conv"):
            r["edges_per_s"] = round(n / ms * 1e3, 1)
            r["nodes"] = V
            # "no-cache" byte model: every gathered row (x[sender] forward, gz[receiver] backward) is fetched
            # per edge instead of once per node; on a randomly ordered graph the gathers miss the per-XCD L2
            gather = n * (DX if kind == "conv_fwd" else DZ) * esz(prec)
            r["nocache_gbs"] = round((by + gather) / ms / 1e6, 1)
            r["frac_hbm_nocache"] = round((by + gather) / ms / 1e6 / HBM_PEAK_GBS, 4)
        return r

    def timed(fn, warm, iters):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
        ev[0].record()
        for i in range(iters):
            fn()
            ev[i + 1].record()
        torch.cuda.synchronize()
        ts = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(iters))
        return ts[len(ts) // 2], sum(ts) / len(ts)

    # ---------------------------------------------------------------- the timed step, fp32 then fp64
    B = 50000
    g5 = Graph(5001, 20000, 40.0)      # config 5: the largest graph of the benchmark set
    g4 = Graph(4001, 5000, 32.0)       # config 4

    def roofline_of(kind, prec, n, V, ms):
        """The roofline that binds a launch (the one with the larger minimum time) and both fractions."""
        dbytes = bytes_model(kind, prec, n, V)
        dflops = n * (F_FWD if kind.endswith("fwd") else F_BWD)
        hbm_frac = dbytes / ms / 1e6 / HBM_PEAK_GBS
        alu_frac = dflops / ms / 1e9 / VALU_PEAK_TFLOPS[prec]
        if alu_frac > hbm_frac:
            r = {"bound": "alu", "kernel": "cgtp_" + kind, "achieved": round(dflops / ms / 1e9, 2),
                 "peak": VALU_PEAK_TFLOPS[prec], "unit": "TFLOP/s", "frac": round(alu_frac, 4)}
        else:
            r = {"bound": "hbm", "kernel": "cgtp_" + kind, "achieved": round(dbytes / ms / 1e6, 1),
                 "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(hbm_frac, 4)}
        r.update({"traffic": measured_traffic("cgtp_" + kind, prec), "traffic_source": "profiles/" + TRAFFIC_FILE[prec],
                  "dtype": prec, "alg_bytes_per_launch": dbytes, "alg_flops_per_launch": dflops, "avg_ms": round(ms, 4),
                  "frac_hbm": round(hbm_frac, 4), "frac_alu": round(alu_frac, 4)})
        return r

    def run_step(prec, tag, with_graph):
        P = plan(prec)
        x = gauss(2000, (B, DX), prec); W = gauss(2002, (B, NW), prec); gz = gauss(2003, (B, DZ), prec)
        y = sh_of_units(2001, B, prec)
        z = torch.empty((B, DZ), device=dev, dtype=tdt(prec))
        gx = torch.empty_like(x); gy = torch.empty_like(y); gW = torch.empty_like(W)
        g = g5
        xn = gauss(4000, (g.V, DX), prec); We = gauss(4002, (g.E, NW), prec); gzn = gauss(4003, (g.V, DZ), prec)
        ye = g.y64.to(tdt(prec))
        zn = torch.empty((g.V, DZ), device=dev, dtype=tdt(prec))
        gxn = torch.empty_like(xn); gye = torch.empty_like(ye); gWe = torch.empty_like(We)

        def k_tp_fwd(): b.tp_forward(P, x, y, W, z)
        def k_tp_bwd(): b.tp_backward(P, x, y, W, gz, gx, gy, gW)
        def k_conv_fwd(): b.conv_forward(P, xn, ye, We, zn, g.row_ptr, g.col)
        def k_conv_bwd(): b.conv_backward(P, xn, ye, We, gzn, gxn, gye, gWe, g.row_ptr, g.col, g.t_row_ptr, g.t_perm)
        step_kernels = [("tp_fwd", k_tp_fwd, B, 0), ("tp_bwd", k_tp_bwd, B, 0),
                        ("conv_fwd", k_conv_fwd, g.E, g.V), ("conv_bwd", k_conv_bwd, g.E, g.V)]
        for _ in range(a.warmup):
            for _, fn, _, _ in step_kernels:
                fn()
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(step_kernels) + 1)] for _ in range(a.steps)]
        t0 = time.perf_counter()
        for s_ in range(a.steps):
            evs[s_][0].record()
            for i, (_, fn, _, _) in enumerate(step_kernels):
                fn()
                evs[s_][i + 1].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / a.steps
        avg_ms = [sum(evs[s_][i].elapsed_time(evs[s_][i + 1]) for s_ in range(a.steps)) / a.steps for i in range(len(step_kernels))]
        step_flops = B * (F_FWD + F_BWD) + g.E * (F_FWD + F_BWD)
        step_rows = [row(tag + "/" + k, k, prec, avg_ms[i], n, V) for i, (k, _, n, V) in enumerate(step_kernels)]
        dom = max(range(len(step_kernels)), key=lambda i: avg_ms[i])
        dk, _, dn, dV = step_kernels[dom]
        roof = roofline_of(dk, prec, dn, dV, avg_ms[dom])
        # the same step recorded once into a HIP graph and replayed (one launch per step instead of ten)
        graph_ms = None
        if with_graph:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            cg = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                for _, fn, _, _ in step_kernels:
                    fn()
                torch.cuda.synchronize()
                with torch.cuda.graph(cg, stream=side):
                    for _, fn, _, _ in step_kernels:
                        fn()
            torch.cuda.current_stream().wait_stream(side)
            for _ in range(a.warmup):
                cg.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(a.steps):
                cg.replay()
            torch.cuda.synchronize()
            graph_ms = (time.perf_counter() - t0) * 1e3 / a.steps
            del cg
        out = {
        "metric": "CG TP nonzero GFLOP/s (MACE uvu: batched fwd+bwd B=50000 and fused conv fwd+bwd on 20000 nodes / ~800k edges)",
        "value": round(value, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config 2 (MACE uvu, 17 paths, batch 50000) forward+backward, plus the fused convolution "
                               "forward+backward on the config 5 graph (20000 nodes, mean degree 40), the largest "
                               "single-GPU configuration; fp32 in the headline, the same step in fp64 under step_f64",
                   "batch": B, "nodes": g5.V, "edges": g5.E, "flops_per_step": step_flops},
        "roofline": roofline, "roofline_f64": roofline_f64, "step_f64": step_f64,
        "edges_per_s": {"conv_fwd_f32": head["edges_per_s_conv_fwd"], "conv_bwd_f32": head["edges_per_s_conv_bwd"],
                        "conv_fwd_f64": None if step_f64 is None else step_f64["edges_per_s_conv_fwd"],
                        "conv_bwd_f64": None if step_f64 is None else step_f64["edges_per_s_conv_bwd"]},
        "cpu_baseline": cpu,
        "graph_replay_ms_per_step": None if graph_ms is None else round(graph_ms, 4), "kernels": rows,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
