"""Checks on compiled code objects of the per-sample uvw kernels (tests/_gcn_emu.py): every address the compiled
code forms stays in bounds when registers start with junk, no stored value and no address derives from a register,
lane, LDS word or private-memory word that nothing defined, and no vector instruction sits where the execution mask is
empty.  The source-level bounds check (tests/test_uvw_ps_bounds.py) cannot see any of this.  Two mistakes of exactly
these kinds were found on the GPU first: a lane index kept in an accumulation register through a copy the compiler
had placed behind the exit of a lane-strided loop, where no lane is active (a memory fault), and z' read across lanes
from lanes a store condition had switched off (wrong dL/dW rows); the emulator reproduces both on the old sources.
"""
import glob
import os
import subprocess

import pytest

from paper_2501_13986_amd import binding as b
from tests import _gcn_emu

HIPCC = "/opt/rocm/bin/hipcc"

PLANS = {
    # 64-wide tiles, a single-channel segment, multiplicities that do not divide 64; fp64 kernels of 330-450 registers
    "wide_and_single": ("33x0o+2x1e+1x2o+64x2e", "1x2o", "64x3e+21x2e+13x3o+5x1o", b.CGTP_F64),
    "odd_muls": ("3x0e+5x1o+7x2e", "1x0e+1x1o+1x2e", "9x0e+2x1o+33x2e", b.CGTP_F32),
    "rows_beyond_the_tile_width": ("64x2o+3x2o+13x0e", "1x2o+1x0o", "48x3e", b.CGTP_F64),     # mul_x > mul_z > 32
    "diffdock_shaped": ("48x0e+10x1o+10x1e+48x0o", "1x0e+1x1o+1x2e", "48x0e+10x1o+10x1e+48x0o", b.CGTP_F32),
}


def _kernels(p):
    """kernel id -> (name, words per row of each pointer argument, which of them are outputs).  By default the
    backward-like second-order kernel also writes dL/dgz and there is no forward-like one."""
    x, y, w, z = p.dim_x, p.dim_y, p.n_w, p.dim_z
    ks = {b.K_TP_FWD: ("cgtp_tp_fwd_uvw_ps", [x, y, w, z], (3,)), b.K_TP_BWD: ("cgtp_tp_bwd_uvw_ps", [x, y, w, z, x, y, w], (4, 5, 6))}
    if p.source(b.K_CONV_DBL_FWD):
        ks[b.K_CONV_DBL_FWD] = ("cgtp_tp_dbl_fwd_uvw_ps", [x, y, w, x, y, w, z], (6,))
        ks[b.K_TP_DBL_BWD] = ("cgtp_tp_dbl_bwd_uvw_ps", [x, y, w, z, x, y, w, x, y, w], (7, 8, 9))
    else:
        ks[b.K_TP_DBL_BWD] = ("cgtp_tp_dbl_bwd_uvw_ps", [x, y, w, z, x, y, w, x, y, w, z], (7, 8, 9, 10))
    return ks


@pytest.fixture(scope="module")
def compiled(tmp_path_factory):
    """name -> (plan, {kernel id: code object path}): each plan compiled into a cache directory of its own."""
    out = {}
    old = os.environ.get("CGTP_CACHE_DIR")
    try:
        for name, (ix, iy, iz, dt) in PLANS.items():
            d = str(tmp_path_factory.mktemp(name))
            os.environ["CGTP_CACHE_DIR"] = d
            p = b.Plan(ix, iy, iz, mode=b.CGTP_UVW, shared_weights=False, dtype=dt, device=-2)
            files = {}
            for k, (kname, _, _) in _kernels(p).items():
                # the plan may have compiled two variants of a kernel (an occupancy request it then dropped): the one
                # it kept has the register count the plan reports
                match = [f for f in glob.glob(os.path.join(d, kname + "_*.hsaco"))]
                assert match, kname
                files[k] = match
            out[name] = (p, files, dt)
    finally:
        if old is None: os.environ.pop("CGTP_CACHE_DIR", None)
        else: os.environ["CGTP_CACHE_DIR"] = old
    return out


@pytest.mark.parametrize("name", list(PLANS))
def test_no_vector_instruction_under_an_empty_mask(compiled, name):
    p, files, dt = compiled[name]
    for k, paths in files.items():
        for f in paths:
            assert _gcn_emu.exec_zero_windows(f) == [], (name, os.path.basename(f))


@pytest.mark.parametrize("kernel", [b.K_TP_FWD, b.K_TP_BWD, b.K_TP_DBL_BWD])
@pytest.mark.parametrize("name", list(PLANS))
def test_compiled_kernels_form_valid_addresses_and_store_defined_values(compiled, name, kernel):
    """Two workgroups over five rows: the persistent loop runs two or three times per wave.  Every byte of every
    output has to be written."""
    p, files, dt = compiled[name]
    info = p.kernel_info(kernel)
    for f in files[kernel]:
        problems = _gcn_emu.check(f, info["lds"], B=5, grid=2, row_words=_kernels(p)[kernel][1],
                                  elt=8 if dt == b.CGTP_F64 else 4, waves=info["wg"] // 64, outputs=_kernels(p)[kernel][2])
        assert problems == [], (name, os.path.basename(f), problems[:3])


KERNEL_TEXT = """
#include <hip/hip_runtime.h>
extern "C" __global__ void __launch_bounds__(64) probe(const double* __restrict__ x, double* __restrict__ y, long long B) {
  __shared__ double t[64];
  const int lane = threadIdx.x;
  for (long long b = blockIdx.x; b < B; b += gridDim.x) {
    t[lane] = x[b * 64 + lane];
    y[b * 64 + lane] = t[lane + SHIFT] + x[b * 64 + lane + SHIFT];
  }
}
"""


@pytest.mark.parametrize("shift,clean", [(0, True), (1, False)])
def test_emulator_sees_a_planted_mistake(tmp_path, shift, clean):
    """A small kernel compiled here and only ever emulated: with SHIFT = 1 lane 63 reads one word past the LDS array
    and one word past its row (in the last row: past the buffer)."""
    src = tmp_path / "probe.hip"
    src.write_text(KERNEL_TEXT.replace("SHIFT", str(shift)))
    obj = tmp_path / "probe.hsaco"
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-O3", "--cuda-device-only", "--no-gpu-bundle-output", "-Xclang", "-target-feature",
                    "-Xclang", "-packed-fp32-ops", "-o", str(obj), str(src)], check=True, capture_output=True)
    problems = _gcn_emu.check(str(obj), 512, B=3, grid=2, row_words=[64, 64], elt=8)
    assert (problems == []) == clean, problems[:3]


def test_no_cached_code_object_has_a_vector_instruction_under_an_empty_mask():
    """Every code object in the library's kernel cache (whatever this machine has compiled: the plans of the tests,
    smoke() and bench.py once they have run or been built), all kernel families, through the library's own check
    (objects compiled before the library had it were never checked at compile time)."""
    cache = os.path.join(os.path.dirname(os.path.abspath(b.__file__)), "_jit_cache")
    bad = {os.path.basename(f): h for f in sorted(glob.glob(os.path.join(cache, "*.hsaco"))) for h in [b.check_code_object(f)] if h}
    assert bad == {}


UVU_PLANS = {
    "mace": ("128x0e+128x1o+128x2e", "1x0e+1x1o+1x2e+1x3o", "128x0e+128x1o+128x2e+128x3o", None, b.CGTP_F32),     # the benchmark's irreps
    "mixed_mul": ("8x0e+4x1o+2x2e", "1x0e+1x1o+1x2e", "8x0e+4x1o+2x2e+4x1e+4x2e",
                  [(0, 0, 0), (1, 0, 1), (1, 1, 3), (1, 1, 4), (1, 2, 1), (2, 0, 2), (2, 2, 2)], b.CGTP_F64),     # several samples per wave
}


@pytest.mark.parametrize("name", list(UVU_PLANS))
def test_compiled_uvu_batched_kernels(tmp_path, name, monkeypatch):
    """The same emulation for the batched uvu kernels (forward, backward, second-order pass): 40 rows, two workgroups."""
    ix, iy, iz, paths, dt = UVU_PLANS[name]
    monkeypatch.setenv("CGTP_CACHE_DIR", str(tmp_path))
    p = b.Plan(ix, iy, iz, paths=paths, dtype=dt, device=-2)
    x, y, w, z = p.dim_x, p.dim_y, p.n_w, p.dim_z
    kernels = {b.K_TP_FWD: ("cgtp_tp_fwd", [x, y, w, z], (3,)), b.K_TP_BWD: ("cgtp_tp_bwd", [x, y, w, z, x, y, w], (4, 5, 6)),
               b.K_TP_DBL_BWD: ("cgtp_tp_dbl_bwd", [x, y, w, z, x, y, w, x, y, w, z], (7, 8, 9, 10))}
    for k, (kname, rows, outs) in kernels.items():
        info = p.kernel_info(k)
        files = [f for f in glob.glob(os.path.join(str(tmp_path), kname + "_*.hsaco")) if len(os.path.basename(f)) == len(kname) + 23]
        assert files, kname
        for f in files:
            assert _gcn_emu.exec_zero_windows(f) == [], (name, os.path.basename(f))
            problems = _gcn_emu.check(f, info["lds"], B=40, grid=2, row_words=rows, elt=8 if dt == b.CGTP_F64 else 4, waves=info["wg"] // 64,
                                      outputs=outs)
            assert problems == [], (name, os.path.basename(f), problems[:3])


@pytest.mark.parametrize("kernel", ["forward", "backward", "backward_pipelined", "backward_pipelined_yw"])
def test_compiled_convolution_kernels(tmp_path, kernel, monkeypatch):
    """The fused convolution kernels of the benchmark plan (MACE irreps, fp32) on a small graph with an empty row, eight
    edge ranges (of odd and even length: the software-pipelined walks start odd ranges with a phantom edge): the
    emulator reads the graph arrays, so gathered rows, CSR positions and the side buffer of split rows are all checked.
    With one sender index out of range the gather must be reported."""
    import numpy as np
    from oracle import conv as oconv
    from paper_2501_13986_amd import synth
    monkeypatch.setenv("CGTP_CACHE_DIR", str(tmp_path))
    if kernel.startswith("backward_pipelined"):      # 1: y, W and gz of the next edge in flight, 2: y and W only
        monkeypatch.setenv("CGTP_PREFETCH_CONV_BWD", "2" if kernel.endswith("yw") else "1")
        kernel = "backward"
    p = b.Plan(synth.MACE_X, synth.MACE_Y, synth.MACE_Z, dtype=b.CGTP_F32, device=-2)
    V, E, el = 7, 45, 4
    rng = np.random.default_rng(5)
    recv, send = rng.integers(0, V, E), rng.integers(0, V, E)
    recv[recv == 3] = 4
    row_ptr, col, perm, t_row_ptr, t_perm = oconv.csr_from_coo(recv.astype(np.int64), send.astype(np.int64), V)
    t_recv = oconv.rows_of_edges(row_ptr)[t_perm].astype(np.int64)
    x, y, w, z = p.dim_x, p.dim_y, p.n_w, p.dim_z
    kid, kname = (b.K_CONV_FWD, "cgtp_conv_fwd") if kernel == "forward" else (b.K_CONV_BWD, "cgtp_conv_bwd")
    info = p.kernel_info(kid); waves = info["wg"] // 64
    grid = 2; nchunk = grid * waves

    def args(col_, t_recv_):
        if kernel == "forward":
            return [("buf", V * x * el), ("buf", E * y * el), ("buf", E * w * el), ("buf", V * z * el), ("buf", (V + 1) * 8, row_ptr),
                    ("buf", E * 8, col_), ("i64", V), ("i64", E), ("buf", nchunk * 2 * z * el), ("i64", nchunk), ("null",)]
        return [("buf", V * x * el), ("buf", E * y * el), ("buf", E * w * el), ("buf", V * z * el), ("buf", V * x * el), ("buf", E * y * el),
                ("buf", E * w * el), ("buf", (V + 1) * 8, t_row_ptr), ("buf", E * 8, t_perm), ("buf", E * 8, t_recv_), ("i64", V), ("i64", E),
                ("buf", nchunk * 2 * x * el), ("i64", nchunk), ("null",), ("buf", (64 + w) * el)]
    files = [f for f in glob.glob(os.path.join(str(tmp_path), kname + "_*.hsaco")) if len(os.path.basename(f)) == len(kname) + 23]
    assert files
    for f in files:
        assert _gcn_emu.check_args(f, info["lds"], args(col, t_recv), grid, waves) == []
        bad_col, bad_recv = col.copy(), t_recv.copy()
        bad_col[E // 2] = V; bad_recv[E // 2] = V          # one node index past the last row
        problems = _gcn_emu.check_args(f, info["lds"], args(bad_col, bad_recv), grid, waves)
        assert problems and "outside every buffer" in problems[0], problems[:2]


HAZARD_ASM = """
	.text
	.globl	probe
	.p2align	8
	.type	probe,@function
probe:
	v_mov_b32_e32 v1, 0
	s_mov_b64 s[2:3], 0
	s_and_saveexec_b64 s[4:5], vcc
.Lloop:
	v_add_u32_e32 v1, 64, v1
	v_cmp_lt_i32_e32 vcc, 100, v1
	s_or_b64 s[2:3], vcc, s[2:3]
	s_andn2_b64 exec, exec, s[2:3]
	s_cbranch_execnz .Lloop
	WINDOW
	s_or_b64 exec, exec, s[4:5]
	s_endpgm
"""


@pytest.mark.parametrize("window,found", [("v_accvgpr_write_b32 a0, v0", "v_accvgpr_write_b32 a0, v0"), ("s_mov_b32 s7, 0", ""),
                                          ("v_readlane_b32 s7, v0, 3", "")])
def test_library_refuses_vector_instructions_under_an_empty_mask(tmp_path, window, found):
    """The check the library applies to every freshly compiled kernel (cgtp_check_code_object), on a hand-assembled
    code object that is never run: a lane-divergent loop followed by one instruction before the mask is restored."""
    src = tmp_path / "t.s"; src.write_text(HAZARD_ASM.replace("WINDOW", window))
    obj = tmp_path / "t.o"
    subprocess.run(["/opt/rocm/llvm/bin/clang", "-x", "assembler", "-target", "amdgcn-amd-amdhsa", "-mcpu=gfx950", "-c", str(src), "-o", str(obj)],
                   check=True, capture_output=True)
    assert b.check_code_object(str(obj)).strip() == found
    assert (_gcn_emu.exec_zero_windows(str(obj)) != []) == (found != "")          # the test-side scan agrees


def test_library_check_agrees_with_the_scan_on_compiled_kernels(compiled):
    for name, (p, files, dt) in compiled.items():
        for paths in files.values():
            for f in paths:
                assert b.check_code_object(f) == "", (name, os.path.basename(f))
