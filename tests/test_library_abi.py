"""CPU-side checks of the C-ABI library: it loads, exports every symbol declared in
include/cgtp.h, plans and generates source without a GPU, and rejects bad problems."""
import os
import re

import numpy as np
import pytest

from oracle import cg
from oracle.irreps import TPSpec
from paper_2501_13986_amd import binding as b, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "cgtp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(\w+)\s*\([^;{]*\)\s*;", text)))


def test_every_declared_symbol_is_exported():
    L = b.lib()
    names = declared_functions()
    assert set(names) == set(b.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_plan_without_gpu_matches_oracle_tables():
    p = b.Plan(synth.MACE_X, synth.MACE_Y, synth.MACE_Z, dtype=b.CGTP_F32, device=-1)
    spec = TPSpec(synth.MACE_X, synth.MACE_Y, synth.MACE_Z)
    assert (p.dim_x, p.dim_y, p.dim_z, p.n_w, p.num_paths) == (1152, 16, 2048, 2176, 17)
    assert p.flops(0) == 73216 and p.flops(1) == 192384
    for t, q in enumerate(spec.paths):
        info = p.path(t)
        assert (info["ix"], info["iy"], info["iz"]) == (q.ix, q.iy, q.iz)
        assert info["l"] == spec.ls(q) and info["w_offset"] == spec.w_off[t]
        ref = cg.cg_nonzeros(*spec.ls(q))
        got = p.path_nonzeros(t)
        assert info["nnz"] == len(ref) == len(got)
        for (i, j, k, v), (i2, j2, k2, v2) in zip(got, ref):
            assert (i, j, k) == (i2, j2, k2) and abs(v - v2) < 1e-14
    for k in range(4):
        src = p.source(k)
        assert src and "__global__" in src and "v_pk_" not in src


@pytest.mark.parametrize("l1,l2,l3", [(a, c, d) for a in range(5) for c in range(5) for d in range(5)
                                       if abs(a - c) <= d <= a + c])
def test_planner_cg_equals_oracle_cg(l1, l2, l3):
    par = lambda l, odd: "eo"[(l % 2) ^ odd]
    odd = (l1 + l2 + l3) % 2
    p = b.Plan(f"1x{l1}{par(l1, 0)}", f"1x{l2}{par(l2, 0)}", f"1x{l3}{par(l3, odd)}", device=-1)
    got, ref = p.path_nonzeros(0), cg.cg_nonzeros(l1, l2, l3)
    assert len(got) == len(ref)
    for (i, j, k, v), (i2, j2, k2, v2) in zip(got, ref):
        assert (i, j, k) == (i2, j2, k2) and abs(v - v2) < 1e-14


def test_bad_problems_are_rejected():
    def status(*a, **k):
        with pytest.raises(b.CgtpError) as e:
            b.Plan(*a, device=-1, **k)
        return e.value.status
    assert status("2x1q", "1x0e", "2x1o") == 1
    assert status("", "1x0e", "2x1o") == 1
    assert status("2x1o", "1x1o", "2x1o", paths=[(0, 0, 0)]) == 1          # parity
    assert status("2x1o", "1x0e", "2x3o", paths=[(0, 0, 0)]) == 1          # triangle
    assert status("2x1o", "1x0e", "3x1o", paths=[(0, 0, 0)]) == 1          # uvu mul mismatch
    assert status("2x1o", "2x0e", "2x1o") == 2                              # mul_y != 1
    assert status("2x9e", "1x0e", "2x9e") == 2                              # l > 8
    assert status("2x1o", "1x0e", "2x1o", paths=[(0, 0, 0), (0, 0, 0)]) == 1
    assert status("2x1o", "1x0e", "2x1o", paths=[(0, 0, 5)]) == 1
    assert status("2x1o", "1x1o", "2x0o") == 1                              # no allowed path
    assert "no path" in b.lib().cgtp_last_error().decode()


def test_uvw_plan_with_per_sample_weights_compiles_without_gpu():
    from oracle.irreps import UVW
    ix = iz = "48x0e+10x1o+10x1e+48x0o"
    spec = TPSpec(ix, synth.NEQUIP_Y, iz, mode=UVW, shared_weights=False)
    for dt in (b.CGTP_F32, b.CGTP_F64):
        p = b.Plan(ix, synth.NEQUIP_Y, iz, mode=b.CGTP_UVW, shared_weights=False, dtype=dt, device=-2)
        assert (p.dim_x, p.dim_y, p.dim_z, p.n_w, p.num_paths) == (spec.dim_x, spec.dim_y, spec.dim_z, spec.n_w, len(spec.paths))
        for t, q in enumerate(spec.paths):
            assert p.path(t)["w_offset"] == spec.w_off[t]
        for k in (b.K_TP_FWD, b.K_TP_BWD):
            info = p.kernel_info(k)
            assert info["vgprs"] > 0 and info["scratch"] == 0
            assert "v_pk_" not in p.source(k)
        # backward counts both dense products of every path
        cg = sum(2 * len(p.path_nonzeros(t)) * spec.irx[q.ix].mul for t, q in enumerate(spec.paths))
        w = sum(2 * (2 * spec.ls(q)[2] + 1) * spec.irx[q.ix].mul * spec.irz[q.iz].mul for q in spec.paths)
        assert p.flops(0) == cg + w and p.flops(1) == 3 * cg + 2 * w and p.flops(2) == 7 * cg + 5 * w
        # the second-order kernel (dL/dx, dL/dy, dL/dW and dL/dgz in one) may trade a few spilled words for two waves per SIMD
        assert p.source(b.K_CONV_DBL_FWD) is None and 0 < p.kernel_info(b.K_TP_DBL_BWD)["vgprs"] and p.kernel_info(b.K_TP_DBL_BWD)["scratch"] <= 64
        p.close()


def test_shared_weight_uvw_kernels_stay_out_of_private_memory():
    """Config 3 (paper Sec. 4, Nequip benchmark shape): the matrix-core forward must not spill at all; the backward
    may keep the three words its prologue parks (they are read back once, outside the tile loop)."""
    p = b.Plan(synth.NEQUIP_X, synth.NEQUIP_Y, synth.NEQUIP_Z, mode=b.CGTP_UVW, shared_weights=True, dtype=b.CGTP_F32, device=-2)
    fwd, bwd = p.kernel_info(b.K_TP_FWD), p.kernel_info(b.K_TP_BWD)
    assert fwd["scratch"] == 0 and 0 < fwd["vgprs"] <= 256, fwd
    assert bwd["scratch"] <= 16 and 0 < bwd["vgprs"] <= 256, bwd
    p.close()


def test_launch_without_device_fails_loudly():
    p = b.Plan("2x1o", "1x0e", "2x1o", device=-1)
    st = b.lib().tp_forward(p._h, 16, 16, 16, 16, 4, None)
    assert st == 2


def test_schedule_search_keeps_a_many_path_plan_out_of_private_memory():
    """68 paths: with the default schedule the backward kernels spill (or need the whole register file);
    the planner's compile-and-check loop has to end on schedules without private memory, and on at most
    256 registers where one of its candidates achieves that."""
    p = b.Plan(synth.MANY_X, synth.MANY_Y, synth.MANY_X, dtype=b.CGTP_F32, device=-2)
    assert p.num_paths == 68
    for k in range(7):
        info = p.kernel_info(k)
        # the double backward may trade a light spill for two waves per SIMD (measured faster); nothing else spills
        assert info["scratch"] <= (256 if k == b.K_TP_DBL_BWD else 0), (k, info)
        assert info["vgprs"] <= 256 or info["scratch"] == 0, (k, info)
    for k in (b.K_TP_FWD, b.K_TP_BWD, b.K_CONV_FWD, b.K_CONV_BWD):
        assert 0 < p.kernel_info(k)["vgprs"] <= 256, (k, p.kernel_info(k))


def test_plan_options():
    """cgtp_plan_create_ex: a NULL options pointer means defaults, struct_size must be set, and kahan_conv
    switches the convolution kernels to compensated row sums (visible in the generated source)."""
    import ctypes as C
    L = b.lib()
    h = C.c_void_p()
    args = (synth.TINY_X.encode(), synth.TINY_Y.encode(), synth.TINY_Z_MERGED.encode(), None, 0, b.CGTP_UVU, 0, b.CGTP_F32, -1, b.CGTP_MUL_IR)
    assert L.cgtp_plan_create_ex(*args, None, C.byref(h)) == 0
    L.cgtp_plan_destroy(h)
    bad = b.cgtp_options(0, 1)
    assert L.cgtp_plan_create_ex(*args, C.byref(bad), C.byref(h)) == 1       # CGTP_EINVAL
    plain = b.Plan(synth.TINY_X, synth.TINY_Y, synth.TINY_Z_MERGED, device=-1)
    comp = b.Plan(synth.TINY_X, synth.TINY_Y, synth.TINY_Z_MERGED, device=-1, kahan_conv=True)
    for k in (b.K_CONV_FWD, b.K_CONV_BWD, b.K_CONV_FWD_ATOMIC):
        assert "(t_ - a" in comp.source(k) and "(t_ - a" not in plain.source(k)
    for k in (b.K_TP_FWD, b.K_TP_BWD, b.K_TP_DBL_BWD):
        assert comp.source(k) == plain.source(k)


@pytest.mark.parametrize("compiler,std,ext", [("gcc", "-std=c99", "c"), ("g++", "-std=c++17", "cpp")])
def test_header_compiles_on_its_own(tmp_path, compiler, std, ext):
    """include/cgtp.h is a complete C and C++ header: a translation unit that includes nothing else compiles."""
    import subprocess
    src = tmp_path / f"only_header.{ext}"
    src.write_text('#include "cgtp.h"\nint only_header_probe(void) { return (int)sizeof(cgtp_path) + (int)CGTP_IR_MUL; }\n')
    r = subprocess.run([compiler, std, "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), "-c", str(src),
                        "-o", str(tmp_path / "only_header.o")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_plan_flags():
    """The layout flag of cgtp_plan_create (paper Sec. 4, data layout): IR_MUL changes the generated accesses of a uvu
    plan, is refused for uvw plans (CGTP_EUNSUPPORTED), and unknown bits are an error (CGTP_EINVAL)."""
    import ctypes as C
    L = b.lib()
    h = C.c_void_p()
    irr = (synth.TINY_X.encode(), synth.TINY_Y.encode(), synth.TINY_Z_MERGED.encode())
    assert L.cgtp_plan_create(*irr, None, 0, b.CGTP_UVU, 0, b.CGTP_F32, -1, 2, C.byref(h)) == 1           # unknown bit
    assert L.cgtp_plan_create(*irr, None, 0, b.CGTP_UVU, 0, b.CGTP_F32, -1, 0x80000001, C.byref(h)) == 1
    assert L.cgtp_plan_create(*irr, None, 0, b.CGTP_UVU, 0, b.CGTP_F32, -1, b.CGTP_IR_MUL, C.byref(h)) == 0
    L.cgtp_plan_destroy(h)
    uvw = (synth.NEQUIP_X.encode(), synth.NEQUIP_Y.encode(), synth.NEQUIP_Z.encode())
    for shared in (0, 1):
        assert L.cgtp_plan_create(*uvw, None, 0, b.CGTP_UVW, shared, b.CGTP_F32, -1, b.CGTP_IR_MUL, C.byref(h)) == 2
        assert b"IR_MUL" in L.cgtp_last_error()
    a = b.Plan(synth.TINY_X, synth.TINY_Y, synth.TINY_Z_MERGED, device=-1)
    t = b.Plan(synth.TINY_X, synth.TINY_Y, synth.TINY_Z_MERGED, device=-1, flags=b.CGTP_IR_MUL)
    assert (a.dim_x, a.dim_z, a.n_w) == (t.dim_x, t.dim_z, t.n_w)
    for k in range(9):
        assert a.source(k) != t.source(k), k
    # 4x1o in the transposed layout: component i of the lane's channel sits at offset 4 (after 4x0e) + i*4 + u0
    assert "+ 8 + u0" in t.source(b.K_TP_FWD) and "u0 * 3" not in t.source(b.K_TP_FWD)
