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

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--extra] [--no-cpu] [--calib-copy] [--step-only [--dtype f64]]
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
    ap.add_argument("--step-only", action="store_true", help="time one step only (for per-kernel profiles of the step)")
    ap.add_argument("--dtype", default="f32", choices=["f32", "f64"], help="precision of the step with --step-only")
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
        out = {"dtype": prec, "ms_per_step": round(ms_per_step, 4), "value": round(step_flops / ms_per_step / 1e6, 1),
               "unit": "GFLOP/s", "flops_per_step": step_flops, "edges_per_s_conv_fwd": round(g.E / avg_ms[2] * 1e3, 1),
               "edges_per_s_conv_bwd": round(g.E / avg_ms[3] * 1e3, 1)}
        del x, W, gz, y, z, gx, gy, gW, xn, We, gzn, ye, zn, gxn, gye, gWe
        torch.cuda.empty_cache()
        return out, step_rows, roof, graph_ms

    def conv_rows(prec, g, tag):
        P = plan(prec)
        xn = gauss(4000, (g.V, DX), prec); We = gauss(4002, (g.E, NW), prec); gzn = gauss(4003, (g.V, DZ), prec)
        ye = g.y64.to(tdt(prec))
        zn = torch.empty((g.V, DZ), device=dev, dtype=tdt(prec))
        gxn = torch.empty_like(xn); gye = torch.empty_like(ye); gWe = torch.empty_like(We)
        _, avg = timed(lambda: b.conv_forward(P, xn, ye, We, zn, g.row_ptr, g.col), a.warmup, a.steps)
        r = [row(f"{tag} conv fwd V={g.V} E={g.E}", "conv_fwd", prec, avg, g.E, g.V)]
        _, avg = timed(lambda: b.conv_backward(P, xn, ye, We, gzn, gxn, gye, gWe, g.row_ptr, g.col, g.t_row_ptr, g.t_perm), a.warmup, a.steps)
        r.append(row(f"{tag} conv bwd V={g.V} E={g.E}", "conv_bwd", prec, avg, g.E, g.V))
        return r

    def uvw_rows():
        # config 3, NequIP-shaped fully connected TP: shared 11 x 32 x 32 weights, matrix-core bound
        P3 = b.Plan(synth.NEQUIP_X, synth.NEQUIP_Y, synth.NEQUIP_Z, mode=b.CGTP_UVW, shared_weights=True,
                    dtype=b.CGTP_F32, device=0)
        B3 = 100000
        sets = []
        for t in range(3):   # rotate buffer sets: one set (234 MB) would sit in the 256 MB Infinity Cache
            x3 = gauss(3000 + 10 * t, (B3, P3.dim_x), "f32")
            y3 = torch.from_numpy(synth.sh_edge_attr(synth.unit_vectors(3001 + 10 * t, B3), 2)).to(dev, torch.float32)
            sets.append((x3, y3, torch.empty((B3, P3.dim_z), device=dev, dtype=torch.float32)))
        W3 = gauss(3002, (P3.n_w,), "f32") / (32.0 ** 0.5)
        it = [0]

        def k3():
            xs, ys, zs = sets[it[0] % 3]
            it[0] += 1
            b.tp_forward(P3, xs, ys, W3, zs)
        med, _ = timed(k3, 3, 12)
        fl = B3 * P3.flops(0)
        by = B3 * (P3.dim_x + P3.dim_y + P3.dim_z) * 4 + P3.n_w * 4
        r = [{"name": "cfg3 NequIP uvw TP fwd B=100000", "kernel": "tp_fwd_uvw", "dtype": "f32", "units": B3,
              "ms": round(med, 4), "gflops": round(fl / med / 1e6, 1), "alg_gbs": round(by / med / 1e6, 1),
              "frac_hbm": round(by / med / 1e6 / HBM_PEAK_GBS, 4), "frac_mfma": round(fl / med / 1e9 / MFMA_F32_PEAK_TFLOPS, 4),
              "binding": "mfma", "frac_binding": round(fl / med / 1e9 / MFMA_F32_PEAK_TFLOPS, 4)}]
        gz3 = gauss(3003, (B3, P3.dim_z), "f32")
        gx3 = torch.empty((B3, P3.dim_x), device=dev, dtype=torch.float32)
        gy3 = torch.empty((B3, P3.dim_y), device=dev, dtype=torch.float32)
        gW3 = torch.empty((P3.n_w,), device=dev, dtype=torch.float32)

        def k3b():
            xs, ys, _ = sets[it[0] % 3]
            it[0] += 1
            b.tp_backward(P3, xs, ys, W3, gz3, gx3, gy3, gW3)
        med, _ = timed(k3b, 3, 12)
        fl = B3 * P3.flops(1)
        by = B3 * (2 * P3.dim_x + 2 * P3.dim_y + P3.dim_z) * 4 + 2 * P3.n_w * 4
        r.append({"name": "cfg3-shaped NequIP uvw TP bwd B=100000", "kernel": "tp_bwd_uvw", "dtype": "f32", "units": B3,
                  "ms": round(med, 4), "gflops": round(fl / med / 1e6, 1), "alg_gbs": round(by / med / 1e6, 1),
                  "frac_hbm": round(by / med / 1e6 / HBM_PEAK_GBS, 4), "frac_mfma": round(fl / med / 1e9 / MFMA_F32_PEAK_TFLOPS, 4),
                  "binding": "mfma", "frac_binding": round(fl / med / 1e9 / MFMA_F32_PEAK_TFLOPS, 4)})
        P3.close()
        return r

    head, rows, roofline, graph_ms = run_step(a.dtype if a.step_only else "f32", "step", not a.no_graph)
    ms_per_step, value, step_flops = head["ms_per_step"], head["value"], head["flops_per_step"]
    step_f64 = roofline_f64 = None
    if not a.step_only:
        step_f64, rows64, roofline_f64, _ = run_step("f64", "step_f64", False)
        rows += rows64
        for prec in ("f32", "f64"):
            rows += conv_rows(prec, g4, "cfg4")
        rows += uvw_rows()

    # ---------------------------------------------------------------- per-configuration table
    if a.extra:
        only = set(t for t in a.only.split(",") if t)

        def want(tag):
            return not only or tag in only

        if want("uvw_ps_f32") or want("uvw_ps_f64"):
            # fully connected TP with per-sample weights, DiffDock-shaped irreps (48 scalars and 10 vectors of each
            # parity): every sample streams its own 7128 weights once, HBM-bound
            XD = "48x0e+10x1o+10x1e+48x0o"
            for prec in ("f32", "f64"):
                if not want("uvw_ps_" + prec):
                    continue
                Pd = b.Plan(XD, synth.NEQUIP_Y, XD, mode=b.CGTP_UVW, shared_weights=False,
                            dtype=b.CGTP_F32 if prec == "f32" else b.CGTP_F64, device=0)
                Bd, el = 50000, (4 if prec == "f32" else 8)
                xd = gauss(6000, (Bd, Pd.dim_x), prec)
                yd = torch.from_numpy(synth.sh_edge_attr(synth.unit_vectors(6001, Bd), 2)).to(dev, tdt(prec))
                Wd = gauss(6002, (Bd, Pd.n_w), prec) / (48.0 ** 0.5)
                zd = torch.empty((Bd, Pd.dim_z), device=dev, dtype=tdt(prec))
                med, _ = timed(lambda: b.tp_forward(Pd, xd, yd, Wd, zd), 3, 10)
                fl = Bd * Pd.flops(0)
                by = Bd * (Pd.dim_x + Pd.dim_y + Pd.n_w + Pd.dim_z) * el
                rows.append({"name": "DiffDock-shaped uvw TP, per-sample weights, fwd B=50000", "kernel": "tp_fwd_uvw_ps", "dtype": prec,
                             "units": Bd, "ms": round(med, 4), "gflops": round(fl / med / 1e6, 1), "alg_gbs": round(by / med / 1e6, 1),
                             "frac_hbm": round(by / med / 1e6 / HBM_PEAK_GBS, 4), "binding": "hbm",
                             "frac_binding": round(by / med / 1e6 / HBM_PEAK_GBS, 4)})
                gzd = gauss(6003, (Bd, Pd.dim_z), prec)
                gxd = torch.empty_like(xd); gyd = torch.empty_like(yd); gWd = torch.empty_like(Wd)
                med, _ = timed(lambda: b.tp_backward(Pd, xd, yd, Wd, gzd, gxd, gyd, gWd), 3, 10)
                fl = Bd * Pd.flops(1)
                by = Bd * (2 * Pd.dim_x + 2 * Pd.dim_y + 2 * Pd.n_w + Pd.dim_z) * el
                rows.append({"name": "DiffDock-shaped uvw TP, per-sample weights, bwd B=50000", "kernel": "tp_bwd_uvw_ps", "dtype": prec,
                             "units": Bd, "ms": round(med, 4), "gflops": round(fl / med / 1e6, 1), "alg_gbs": round(by / med / 1e6, 1),
                             "frac_hbm": round(by / med / 1e6 / HBM_PEAK_GBS, 4), "binding": "hbm",
                             "frac_binding": round(by / med / 1e6 / HBM_PEAK_GBS, 4)})
                # second-order pass: one kernel (dL/dx, dL/dy, dL/dW and dL/dgz from the same pass over the W and LC tiles)
                ms_fwd, ms_bwd = rows[-2]["ms"], rows[-1]["ms"]
                Lad = gauss(6004, (Bd, Pd.dim_x), prec); Lbd = gauss(6005, (Bd, Pd.dim_y), prec); LCd = gauss(6006, (Bd, Pd.n_w), prec)
                Lxd = torch.empty_like(xd); Lyd = torch.empty_like(yd); LWd = torch.empty_like(Wd); Lgzd = torch.empty_like(zd)
                med, _ = timed(lambda: b.tp_double_backward(Pd, xd, yd, Wd, gzd, Lad, Lbd, LCd, Lxd, Lyd, LWd, Lgzd), 2, 8)
                fl = Bd * Pd.flops(2)
                by = Bd * (2 * (Pd.dim_x + Pd.dim_y + Pd.n_w + Pd.dim_z) + Pd.dim_x + Pd.dim_y + Pd.n_w) * el
                rows.append({"name": "DiffDock-shaped uvw TP, per-sample weights, double bwd (one fused kernel) B=50000", "kernel": "tp_dbl_uvw_ps",
                             "dtype": prec, "units": Bd, "ms": round(med, 4), "gflops": round(fl / med / 1e6, 1), "alg_gbs": round(by / med / 1e6, 1),
                             "frac_hbm": round(by / med / 1e6 / HBM_PEAK_GBS, 4), "binding": "hbm",
                             "frac_binding": round(by / med / 1e6 / HBM_PEAK_GBS, 4),
                             "note": f"seven separate dispatches = 3 forward + 4 backward launches: {round(3 * ms_fwd + 4 * ms_bwd, 3)} ms"})
                del xd, yd, Wd, zd, gzd, gxd, gyd, gWd, Lad, Lbd, LCd, Lxd, Lyd, LWd, Lgzd
                Pd.close()
        if want("csr"):
            # graph preparation (integer work): COO -> CSR by receiver + transpose permutation
            for tag_, seed_, V_, deg_ in (("cfg4", 4001, 5000, 32.0), ("cfg5", 5001, 20000, 40.0)):
                recv_, send_, _ = synth.periodic_graph(seed_, V_, deg_)
                r_ = torch.from_numpy(recv_).to(dev); s_ = torch.from_numpy(send_).to(dev)
                E_ = recv_.shape[0]
                ws_ = torch.empty(b.cgtp_csr_workspace_bytes(E_, V_), dtype=torch.uint8, device=dev)
                out_ = tuple(torch.empty(n_, dtype=torch.int64, device=dev) for n_ in (V_ + 1, E_, E_, V_ + 1, E_))
                by = E_ * 8 * (2 + 3) + (V_ + 1) * 8 * 2          # two index arrays in, three out, two offset arrays
                for what_, fn_ in (("synchronous call, library scratch", lambda: b.cgtp_csr_from_coo(r_, s_, V_)),
                                   ("asynchronous, caller workspace", lambda: b.cgtp_csr_from_coo_async(r_, s_, V_, out_, ws_, None)),
                                   ("asynchronous, without the transpose", lambda: b.cgtp_csr_from_coo_async(r_, s_, V_, out_, ws_, None, transpose=False))):
                    med, _ = timed(fn_, 2, 8)
                    rows.append({"name": f"{tag_} graph preparation (COO -> CSR + transpose; {what_}) V={V_} E={E_}", "kernel": "csr_from_coo",
                                 "dtype": "int64", "units": E_, "ms": round(med, 4), "gflops": 0.0, "alg_gbs": round(by / med / 1e6, 1),
                                 "frac_hbm": round(by / med / 1e6 / HBM_PEAK_GBS, 4), "binding": "hbm",
                                 "frac_binding": round(by / med / 1e6 / HBM_PEAK_GBS, 4), "edges_per_s": round(E_ / med * 1e3, 1)})
        if want("many_f32"):
            # a Nequip-like layout with both parities (68 paths, multiplicity 64): the plan only fits the register
            # file with the schedules the planner searches for (per-path y products and accumulator updates)
            irr_m = "+".join(f"64x{l}{p}" for l in range(4) for p in "eo")
            PM = b.Plan(irr_m, synth.MANY_Y, irr_m, dtype=b.CGTP_F32, device=0)
            mx, my, mz, mw = PM.dim_x, PM.dim_y, PM.dim_z, PM.n_w
            x = gauss(6000, (B, mx), "f32"); W = gauss(6002, (B, mw), "f32"); gz = gauss(6003, (B, mz), "f32")
            y = sh_of_units(6001, B, "f32")
            z = torch.empty((B, mz), device=dev, dtype=torch.float32)
            gx = torch.empty_like(x); gy = torch.empty_like(y); gW = torch.empty_like(W)
            for kind, fn, by, fl in (
                    ("tp_fwd", lambda: b.tp_forward(PM, x, y, W, z), B * (mx + my + mw + mz) * 4, B * PM.flops(0)),
                    ("tp_bwd", lambda: b.tp_backward(PM, x, y, W, gz, gx, gy, gW), B * (2 * mx + 2 * my + 2 * mw + mz) * 4, B * PM.flops(1))):
                med, _ = timed(fn, 3, 10)
                t_hbm, t_alu = by / (HBM_PEAK_GBS * 1e9) * 1e3, fl / (VALU_PEAK_TFLOPS["f32"] * 1e12) * 1e3
                rows.append({"name": f"68-path both-parity plan (64 channels) {kind} B=50000", "kernel": kind, "dtype": "f32", "units": B,
                             "ms": round(med, 4), "gflops": round(fl / med / 1e6, 1), "alg_gbs": round(by / med / 1e6, 1),
                             "frac_hbm": round(by / med / 1e6 / HBM_PEAK_GBS, 4),
                             "frac_valu": round(fl / med / 1e9 / VALU_PEAK_TFLOPS["f32"], 4),
                             "binding": "hbm" if t_hbm >= t_alu else "alu", "frac_binding": round(max(t_hbm, t_alu) / med, 4),
                             "vgprs": PM.kernel_info(0 if kind == "tp_fwd" else 1)["vgprs"]})
            del x, W, gz, y, z, gx, gy, gW
            PM.close()
        for prec in ("f32", "f64"):
            P = plan(prec)
            if want("cfg2_" + prec):
                x = gauss(2000, (B, DX), prec); W = gauss(2002, (B, NW), prec); gz = gauss(2003, (B, DZ), prec)
                y = sh_of_units(2001, B, prec)
                z = torch.empty((B, DZ), device=dev, dtype=tdt(prec))
                gx = torch.empty_like(x); gy = torch.empty_like(y); gW = torch.empty_like(W)
                med, _ = timed(lambda: b.tp_forward(P, x, y, W, z), 3, 10)
                rows.append(row("cfg2 MACE TP fwd B=50000", "tp_fwd", prec, med, B))
                med, _ = timed(lambda: b.tp_backward(P, x, y, W, gz, gx, gy, gW), 3, 10)
                rows.append(row("cfg2 MACE TP bwd B=50000", "tp_bwd", prec, med, B))
                # double backward (second derivatives): fused kernel vs the seven-dispatch composition
                La = gauss(2004, (B, DX), prec); LC = gauss(2006, (B, NW), prec); Lb = sh_of_units(2005, B, prec)
                Lgz = torch.empty_like(gz)
                med, _ = timed(lambda: b.tp_double_backward(P, x, y, W, gz, La, Lb, LC, gx, gy, gW, Lgz), 3, 10)
                by = B * (2 * (DX + DY + NW + DZ) + DX + DY + NW) * esz(prec)

                def seven():
                    b.tp_backward(P, La, Lb, W, gz, gx, gy, gW); b.tp_backward(P, x, y, LC, gz, gx, gy, gW)
                    b.tp_forward(P, La, y, W, z); b.tp_backward(P, La, y, W, gz, gx, gy, gW)
                    b.tp_backward(P, x, Lb, W, gz, gx, gy, gW); b.tp_forward(P, x, Lb, W, z); b.tp_forward(P, x, y, LC, z)
                med7, _ = timed(seven, 2, 6)
                fl = B * P.flops(2)
                fh, fa = by / med / 1e6 / HBM_PEAK_GBS, fl / med / 1e9 / VALU_PEAK_TFLOPS[prec]
                rows.append({"name": "cfg2-shaped MACE TP double bwd (fused) B=50000", "kernel": "tp_dbl_bwd", "dtype": prec,
                             "units": B, "ms": round(med, 4), "alg_gbs": round(by / med / 1e6, 1),
                             "frac_hbm": round(fh, 4), "frac_valu": round(fa, 4), "binding": "hbm" if fh >= fa else "alu",
                             "frac_binding": round(max(fh, fa), 4),
                             "gflops": round(fl / med / 1e6, 1), "flops_model": "fused pass: 8x contraction + 3x weight part",
                             "seven_dispatch_ms": round(med7, 4), "speedup_vs_seven_dispatches": round(med7 / med, 2)})
                del x, W, gz, y, z, gx, gy, gW, La, Lb, LC, Lgz
            for tag, g in (("cfg4", g4), ("cfg5", g5), ("cfg4cells", None), ("cfg5cells", None)):
                if not want(f"{tag}_{prec}"):
                    continue
                if tag == "cfg4cells":      # same graphs with nodes numbered cell by cell (gathers find their rows in L2)
                    g = Graph(4001, 5000, 32.0, "cells")
                elif tag == "cfg5cells":
                    g = Graph(5001, 20000, 40.0, "cells")
                xn = gauss(4000, (g.V, DX), prec); We = gauss(4002, (g.E, NW), prec); gzn = gauss(4003, (g.V, DZ), prec)
                ye = g.y64.to(tdt(prec))
                zn = torch.empty((g.V, DZ), device=dev, dtype=tdt(prec))
                gxn = torch.empty_like(xn); gye = torch.empty_like(ye); gWe = torch.empty_like(We)
                med, _ = timed(lambda: b.conv_forward(P, xn, ye, We, zn, g.row_ptr, g.col), 3, 10)
                rows.append(row(f"{tag} conv fwd V={g.V} E={g.E}", "conv_fwd", prec, med, g.E, g.V))
                med, _ = timed(lambda: b.conv_backward(P, xn, ye, We, gzn, gxn, gye, gWe, g.row_ptr, g.col, g.t_row_ptr, g.t_perm), 3, 10)
                rows.append(row(f"{tag} conv bwd V={g.V} E={g.E}", "conv_bwd", prec, med, g.E, g.V))
                if tag == "cfg4":
                    # second-order pass of the convolution: two fused kernels vs seven first-order dispatches
                    Lan = gauss(4004, (g.V, DX), prec); LCe = gauss(4006, (g.E, NW), prec); Lbe = ye.clone()
                    Lgzn = torch.empty_like(gzn)
                    med, _ = timed(lambda: b.conv_double_backward(P, xn, ye, We, gzn, Lan, Lbe, LCe, gxn, gye, gWe, Lgzn,
                                                                  g.row_ptr, g.col, g.t_row_ptr, g.t_perm), 2, 8)

                    def seven_conv():
                        cb = lambda a1, a2, a3: b.conv_backward(P, a1, a2, a3, gzn, gxn, gye, gWe, g.row_ptr, g.col, g.t_row_ptr, g.t_perm)
                        cf = lambda a1, a2, a3: b.conv_forward(P, a1, a2, a3, zn, g.row_ptr, g.col)
                        cb(Lan, Lbe, We); cb(xn, ye, LCe); cf(Lan, ye, We); cb(Lan, ye, We); cb(xn, Lbe, We); cf(xn, Lbe, We); cf(xn, ye, LCe)
                    med7, _ = timed(seven_conv, 1, 5)
                    by = (g.E * 3 * (DY + NW) + g.V * (3 * DX + 2 * DZ)) * esz(prec)
                    fl = g.E * P.flops(2)
                    fh, fa = by / med / 1e6 / HBM_PEAK_GBS, fl / med / 1e9 / VALU_PEAK_TFLOPS[prec]
                    rows.append({"name": f"{tag}-shaped conv double bwd (two fused kernels) V={g.V} E={g.E}", "kernel": "conv_dbl_bwd",
                                 "dtype": prec, "units": g.E, "ms": round(med, 4), "alg_gbs": round(by / med / 1e6, 1),
                                 "frac_hbm": round(fh, 4), "frac_valu": round(fa, 4), "binding": "hbm" if fh >= fa else "alu",
                                 "frac_binding": round(max(fh, fa), 4), "gflops": round(fl / med / 1e6, 1),
                                 "flops_model": "fused pass: 8x contraction + 3x weight part", "seven_dispatch_ms": round(med7, 4),
                                 "speedup_vs_seven_dispatches": round(med7 / med, 2), "edges_per_s": round(g.E / med * 1e3, 1)})
                    del Lan, LCe, Lbe, Lgzn
                    # the same launches from a plan with compensated (Kahan) row sums
                    PK = b.Plan(*irr, dtype=b.CGTP_F32 if prec == "f32" else b.CGTP_F64, device=0, kahan_conv=True)
                    med, _ = timed(lambda: b.conv_forward(PK, xn, ye, We, zn, g.row_ptr, g.col), 3, 10)
                    rows.append(row(f"{tag} conv fwd, compensated row sums", "conv_fwd", prec, med, g.E, g.V))
                    med, _ = timed(lambda: b.conv_backward(PK, xn, ye, We, gzn, gxn, gye, gWe, g.row_ptr, g.col, g.t_row_ptr, g.t_perm), 3, 10)
                    rows.append(row(f"{tag} conv bwd, compensated row sums", "conv_bwd", prec, med, g.E, g.V))
                    PK.close()
                if tag.endswith("cells"):
                    del xn, We, gzn, ye, zn, gxn, gye, gWe, g
                    torch.cuda.empty_cache()
                    continue
                # unsorted edge data served deterministically: CSR built on the stream in every call (caller-owned
                # workspace, nothing allocated, nothing awaited), edge rows reached through perm
                csr_ws = torch.empty(b.cgtp_csr_workspace_bytes(g.E, g.V), dtype=torch.uint8, device=dev)
                csr_out = (torch.empty_like(g.row_ptr), torch.empty_like(g.col), torch.empty_like(g.perm),
                           torch.empty_like(g.t_row_ptr), torch.empty_like(g.t_perm))

                def fwd_perm():
                    rp_, cl_, pm_, _, _ = b.cgtp_csr_from_coo_async(g.recv, g.send, g.V, csr_out, csr_ws, None, transpose=False)
                    b.conv_forward_perm(P, xn, ye, We, zn, rp_, cl_, pm_)

                def bwd_perm():
                    rp_, cl_, pm_, trp_, tpm_ = b.cgtp_csr_from_coo_async(g.recv, g.send, g.V, csr_out, csr_ws, None)
                    b.conv_backward_perm(P, xn, ye, We, gzn, gxn, gye, gWe, rp_, cl_, trp_, tpm_, pm_)
                med, _ = timed(fwd_perm, 3, 10)
                rows.append(row(f"{tag} conv fwd, unsorted edges: CSR per call + edge permutation", "conv_fwd", prec, med, g.E, g.V))
                med, _ = timed(bwd_perm, 3, 10)
                rows.append(row(f"{tag} conv bwd, unsorted edges: CSR per call + edge permutation", "conv_bwd", prec, med, g.E, g.V))
                # nondeterministic variant on the unsorted edge list (same algorithmic bytes and flops)
                med, _ = timed(lambda: b.conv_forward_atomic(P, xn, ye, We, zn, g.recv, g.send), 3, 10)
                rows.append(row(f"{tag} conv fwd atomic, unsorted edges", "conv_fwd_atomic", prec, med, g.E, g.V))
                med, _ = timed(lambda: b.conv_backward_atomic(P, xn, ye, We, gzn, gxn, gye, gWe, g.recv, g.send), 3, 10)
                rows.append(row(f"{tag} conv bwd atomic, unsorted edges", "conv_bwd_atomic", prec, med, g.E, g.V))
                del xn, We, gzn, ye, zn, gxn, gye, gWe, csr_ws, csr_out
                torch.cuda.empty_cache()

    if a.calib_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev)   # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    # ---------------------------------------------------------------- CPU oracle on a bounded sample
    cpu = None
    if not a.no_cpu:
        from oracle import conv as oconv, tp as otp
        from oracle.irreps import TPSpec
        spec = TPSpec(*irr)
        # the same four operations as the step, on a sample sized for 10-30 s of CPU work: 1/8 of the batch and a
        # 250-node box of the same density as the 20 000-node graph (mean degree 40)
        Bs, Vs = 6250, 250
        xs = synth.normal(1, (Bs, DX)); Ws = synth.normal(2, (Bs, NW)); gzs = synth.normal(3, (Bs, DZ))
        ys = synth.sh_edge_attr(synth.unit_vectors(4, Bs), 3)
        recv, send, unit = synth.periodic_graph(5, Vs, 40.0, cutoff=1.0)
        row_ptr, col, perm, _, _ = oconv.csr_from_coo(recv, send, Vs)
        Es = col.shape[0]
        xg = synth.normal(6, (Vs, DX)); Wg = synth.normal(7, (Es, NW)); gg = synth.normal(8, (Vs, DZ))
        yg = synth.sh_edge_attr(unit[perm], 3)
        c0, t0 = time.process_time(), time.perf_counter()
        otp.forward(spec, xs, ys, Ws)
        otp.backward(spec, xs, ys, Ws, gzs)
        oconv.forward(spec, xg, yg, Wg, row_ptr, col)
        oconv.backward(spec, xg, yg, Wg, gg, row_ptr, col)
        dt, cpu_s = time.perf_counter() - t0, time.process_time() - c0
        fl = (Bs + Es) * (F_FWD + F_BWD)
        # threads the oracle actually kept busy: CPU time of the process over wall time (numpy's einsum runs the
        # contraction on one thread; a BLAS-backed step would show up here), next to what the box offers
        try:
            from threadpoolctl import threadpool_info
            pools = [f"{t_['internal_api']}:{t_['num_threads']}" for t_ in threadpool_info()]
        except Exception:
            pools = []
        cpu = {"value": round(fl / dt / 1e9, 3), "unit": "GFLOP/s", "cores": max(1, round(cpu_s / dt)), "kind": "oracle",
               "sample": f"numpy fp64 oracle, the step's four operations on {Bs} of {B} samples and a {Vs}-node / {Es}-edge graph "
                         f"of the same mean degree instead of {g5.V} nodes / {g5.E} edges: {dt:.1f} s wall, {cpu_s:.1f} s CPU; "
                         f"the full step at this rate would take {step_flops / (fl / dt):.0f} s (extrapolated, not run)",
               "sample_units": {"samples": Bs, "nodes": Vs, "edges": Es}, "wall_s": round(dt, 2), "cpu_s": round(cpu_s, 2),
               "host_cpus": os.cpu_count(), "thread_pools": pools,
               "extrapolated_full_step_s": round(step_flops / (fl / dt), 1)}

    out = {
        "metric": "CG TP nonzero GFLOP/s (MACE uvu: batched fwd+bwd B=50000 and fused conv fwd+bwd on 20000 nodes / ~800k edges)",
        "value": round(value, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": a.dtype if a.step_only else "f32", "data": "synthetic",
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
