// Internal types of the planner: irreps, paths with their CG nonzeros, launch geometry,
// compiled kernels.  Nothing here is visible across the C ABI.
#pragma once

#include <hip/hip_runtime_api.h>

#include <cstdint>
#include <stdexcept>
#include <string>
#include <vector>

#include "../../include/cgtp.h"

namespace cgtp {

struct Irrep {
  int mul = 0;
  int l = 0;
  int p = 1;  // +1 even, -1 odd
  int dim() const { return mul * (2 * l + 1); }
};

// "32x0e + 32x1o" -> list of irreps (paper Sec. 2.1).  Throws std::invalid_argument.
std::vector<Irrep> parse_irreps(const std::string& s);

struct Nz {
  int i, j, k;
  double v;
};

// Nonzeros of the real-basis block P^(l1,l2,l3) (paper Sec. 2.2), lexicographic in (i,j,k),
// normalised to sum_{ij} C[ijk]C[ijk'] = delta_kk', first nonzero positive.
std::vector<Nz> cg_nonzeros(int l1, int l2, int l3);

constexpr int kMaxL = 8;

struct PathInfo {
  int ix, iy, iz;
  int mode;
  double coeff;
  int l1, l2, l3;
  int mul_x, mul_z;
  int64_t w_off;  // first weight word of this path's tile
  std::vector<Nz> nz;
};

// How channels are laid over the 64 lanes of a wavefront.
//   G     lanes that share one sample (power of two, <= 64)
//   spw   samples per wavefront = 64 / G (batched kernels only; conv kernels use one edge per wave)
//   cpl   adjacent channels per lane
//   npass passes over channel blocks of G*cpl
// Channel handled by lane t in pass c, slot e:  u = (c*G + t%G)*cpl + e.
struct LaneMap {
  int G = 64, spw = 1, cpl = 1, npass = 1;
  int occ = 0;  // register budget: ask the compiler for at least this many waves per SIMD (0 = no request)
};

// Code-generation choices the planner varies per kernel until the compiled code fits the register
// file (paper Sec. 3.1: the schedule is fixed by static analysis when the plan is made).  -1 = the
// emitter's own default for that kernel.  Every field can be forced from the environment (tuning).
struct Schedule {
  int w_upfront = -1;  // forward: issue all weight loads of a row before the first path (1) or per path (0)
  int upfront = -1;    // backward: 0 loads per output segment, 1 all weights first, 2 weights and gz first
  int prefetch = -1;   // conv: software-pipelined edge loop with two operand register sets
  int pin = -1;        // backward: accumulators brought up to date 0 = per output segment only, 2 = after every path
  int fresh_y = -1;    // 1: the products v*y[j] are formed anew in every path (never shared between paths)
  int occ = -1;        // waves per SIMD asked of the compiler (overrides the lane map's request)
  int one_kernel = 0;  // per-sample uvw second-order pass: the backward-like kernel also computes dL/dgz (no forward-like kernel)
  int phases = 1;      // backward: x segments, forward convolution: output segments, split into this many phases
                       // (only a phase's own rows and accumulators are live)
};

struct Kernel {
  std::string source;
  std::string name;
  hipModule_t module = nullptr;
  hipFunction_t fn = nullptr;
  int vgprs = 0, agprs = 0, sgprs = 0, lds = 0, scratch = 0;  // vgprs counts both register kinds
  Schedule sched;
  // uvu kernels: refuse compiled code that both changes the execution mask (a lane-conditional region or loop) and
  // relocates registers (accumulation registers or private memory in use); see jit_compile
  bool screen_divergence = false;
  int wg = 256;         // threads per workgroup
  int blocks_per_cu = 0;
};

struct Plan {
  std::vector<Irrep> irx, iry, irz;
  std::vector<int64_t> offx, offy, offz;  // segment starts; last entry = dim
  std::vector<PathInfo> paths;
  int64_t n_w = 0;
  int mode = CGTP_UVU;  // all paths share one mode
  bool shared_w = false;
  int dtype = CGTP_F32;
  bool ir_mul = false;      // segment layout (m+l)*mul + u instead of u*(2l+1) + (m+l) (paper Sec. 4, data layout)
  bool kahan_conv = false;  // compensated accumulation over the edges of a row in the convolution kernels
  int device = -1;
  int num_cu = 256;
  LaneMap map[9];  // indexed by cgtp_kernel
  Kernel k[9];  // indexed by cgtp_kernel
  Kernel k_fix;  // merges split rows after the conv kernels (uvu) / adds per-wave gW partial sums (uvw)
  // workspace for split-row partial sums and per-edge receiver ids (conv)
  void* ws = nullptr;
  size_t ws_bytes = 0;

  int64_t dim_x() const { return offx.back(); }
  int64_t dim_y() const { return offy.back(); }
  int64_t dim_z() const { return offz.back(); }
  size_t elt() const { return dtype == CGTP_F64 ? 8 : 4; }
};

// Source emitters (emit_uvu.cpp, emit_uvw.cpp).  Each fills Kernel::source/name/wg.
// The uvu emitters follow out.sched.
void emit_uvu_forward(const Plan& P, bool conv, Kernel& out);
void emit_uvu_backward(const Plan& P, bool conv, Kernel& out);
void emit_uvu_double_backward(const Plan& P, Kernel& K);
void emit_uvu_atomic(const Plan& P, bool backward, Kernel& out);
void emit_uvu_conv_double(const Plan& P, bool backward_like, Kernel& out);
void emit_uvw_forward(const Plan& P, Kernel& out);
void emit_uvw_backward(const Plan& P, Kernel& out, Kernel& reduce);
int64_t uvw_tile_samples(const Plan& P);  // samples handled by one workgroup of the uvw kernel
void emit_fixup(const Plan& P, Kernel& out);
// uvw with per-sample weights (emit_uvw_ps.cpp): one wave per sample, VALU, fp32 and fp64
void emit_uvw_ps_forward(const Plan& P, Kernel& out);
void emit_uvw_ps_backward(const Plan& P, Kernel& out);
void emit_uvw_ps_double_forward(const Plan& P, Kernel& out);    // second-order pass: dL/dgz
void emit_uvw_ps_double_backward(const Plan& P, Kernel& out);   // second-order pass: dL/dx, dL/dy, dL/dW

// thrown by an emitter for a valid problem whose shape its kernel does not cover
struct ShapeNotCovered : std::runtime_error {
  using std::runtime_error::runtime_error;
};

// Run-time compilation (jit.cpp).  Throws std::runtime_error with the compiler log.
// device >= 0: compile (or fetch from the cache) and load; -2: compile into the cache only; -1: nothing.
// Whenever code is produced, the register / private-memory figures of the Kernel are filled in from the
// code object's metadata, so schedules can be compared without a GPU.
// thrown by jit_compile for a kernel whose compiled code fails the check described at jit_check_code_object
struct RefusedCode : std::runtime_error {
  using std::runtime_error::runtime_error;
};
void jit_compile(Kernel& k, int device);
void jit_unload(Kernel& k);
// first vector instruction found under an empty execution mask behind a lane-divergent loop ("" if none)
std::string jit_check_code_object(const std::string& path);

// Tunables read from the environment (integers; unset or empty -> fallback).
int env_int(const char* name, int fallback);

}  // namespace cgtp
