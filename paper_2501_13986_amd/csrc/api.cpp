// The C ABI of include/cgtp.h: planning (static analysis of the irreps, paper Sec. 3.1),
// kernel generation and the launches.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <stdexcept>
#include <string>
#include <tuple>

#include "csr.hpp"
#include "plan.hpp"

struct cgtp_plan {
  cgtp::Plan P;
};

namespace {

thread_local std::string g_err;

cgtp_status fail(cgtp_status s, const std::string& msg) {
  g_err = msg;
  return s;
}

#define HIP_TRY(expr)                                                                                   \
  do {                                                                                                  \
    hipError_t e_ = (expr);                                                                             \
    if (e_ != hipSuccess) return fail(CGTP_ERUNTIME, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)

using cgtp::Irrep;
using cgtp::Kernel;
using cgtp::LaneMap;
using cgtp::PathInfo;
using cgtp::Plan;

bool allowed(const Irrep& a, const Irrep& b, const Irrep& c) {
  return std::abs(a.l - b.l) <= c.l && c.l <= a.l + b.l && c.p == a.p * b.p;
}

std::vector<int64_t> prefix(const std::vector<Irrep>& v) {
  std::vector<int64_t> o{0};
  for (auto& ir : v) o.push_back(o.back() + ir.dim());
  return o;
}

int pow2ceil(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

// Channel -> lane assignment.  Adjacent channels share a lane (`cpl` of them) so that a lane's
// words are contiguous; a wave is filled with several samples when the multiplicity is small.
LaneMap pick_map(const Plan& P, int kind) {
  static const char* const kTag[9] = {"TP_FWD",          "TP_BWD",     "CONV_FWD",     "CONV_BWD",    "CONV_FWD_ATOMIC",
                                      "CONV_BWD_ATOMIC", "TP_DBL_BWD", "CONV_DBL_FWD", "CONV_DBL_BWD"};
  const bool conv = kind == CGTP_K_CONV_FWD || kind == CGTP_K_CONV_BWD || kind == CGTP_K_CONV_FWD_ATOMIC ||
                    kind == CGTP_K_CONV_DBL_FWD || kind == CGTP_K_CONV_DBL_BWD;
  const bool atomic = kind == CGTP_K_CONV_FWD_ATOMIC || kind == CGTP_K_CONV_BWD_ATOMIC;
  int M = 1;
  bool even = true;
  for (auto& q : P.paths) {
    M = std::max(M, q.mul_x);
    even = even && (q.mul_x % 2 == 0);
  }
  LaneMap m;
  // tuning overrides: CGTP_CPL / CGTP_OCC for all kernels, CGTP_CPL_<KIND> / CGTP_OCC_<KIND> for one
  int cpl = cgtp::env_int((std::string("CGTP_CPL_") + kTag[kind]).c_str(), cgtp::env_int("CGTP_CPL", 0));
  if (cpl <= 0) {
    cpl = (even && M >= 128) ? 2 : 1;
    // measured on the 128-channel MACE shape: the fp32 batched backward is faster with one channel per
    // lane and two passes (more waves in flight), everything else with two adjacent channels per lane
    if (kind == CGTP_K_TP_BWD && P.dtype == CGTP_F32) cpl = 1;
    // float atomics are carried out at the memory side in 32-byte requests: one channel per lane makes the
    // 64 lanes of an atomic instruction cover contiguous words (8 requests in fp32 instead of 16 with pairs)
    if (atomic) cpl = 1;
    // twice the operands of the first-order kernels per channel
    // (measured: the sender walk of the convolution's second-order pass is faster with two, 1.49 -> 1.05 ms)
    if (kind == CGTP_K_TP_DBL_BWD || kind == CGTP_K_CONV_DBL_FWD) cpl = 1;
  }
  for (auto& q : P.paths)
    if (q.mul_x % cpl) cpl = 1;
  m.cpl = cpl;
  m.occ = cgtp::env_int((std::string("CGTP_OCC_") + kTag[kind]).c_str(), cgtp::env_int("CGTP_OCC", 0));
  if (m.occ == 0 && kind == CGTP_K_TP_FWD && P.dtype == CGTP_F64 && cpl == 2) m.occ = 2;  // measured: 0.45 vs 0.49 ms
  int lanes = (M + cpl - 1) / cpl;
  // a multiplicity that fills only part of a wave: several samples (batched kernels) or several independent
  // edge-range workers (convolution kernels) share the wave
  m.G = (conv && cgtp::env_int("CGTP_CONV_SPLIT_WAVE", 1) == 0) ? 64 : std::min(64, pow2ceil(lanes));
  m.spw = 64 / m.G;
  m.npass = (M + m.G * cpl - 1) / (m.G * cpl);
  return m;
}

// Schedules to try for a kernel, most aggressive first (all loads of a row in flight, software pipelining)
// down to the most economical in registers (products v*y[j] local to each path, accumulators brought up to
// date after every path, loads where they are used, x segments in phases).
std::vector<cgtp::Schedule> schedule_candidates(int kind, bool small) {
  using S = cgtp::Schedule;
  auto mk = [](int w_upfront, int upfront, int prefetch, int pin, int fresh_y, int phases) {
    S s;
    s.w_upfront = w_upfront;
    s.upfront = upfront;
    s.prefetch = prefetch;
    s.pin = pin;
    s.fresh_y = fresh_y;
    s.phases = phases;
    return s;
  };
  switch (kind) {
    case CGTP_K_TP_FWD:
      // many paths: per-path y products first (measured 0.32 vs 0.40 ms on a 68-path plan, fewer registers)
      if (!small) return {mk(-1, -1, -1, -1, 1, 1), mk(0, -1, -1, -1, 1, 1), S()};
      return {S(), mk(-1, -1, -1, -1, 1, 1), mk(0, -1, -1, -1, 1, 1)};
    case CGTP_K_CONV_FWD:
    case CGTP_K_CONV_FWD_ATOMIC:
      return {S(), mk(-1, -1, 0, -1, -1, 1), mk(-1, -1, 0, -1, 1, 1), mk(0, -1, 0, -1, 1, 1),
              mk(0, -1, 0, -1, 1, 2), mk(0, -1, 0, -1, 1, 3)};   // last: phases over output segments
    case CGTP_K_TP_BWD:
      return {S(), mk(-1, -1, -1, 2, 1, 1), mk(-1, 0, -1, 2, 1, 1), mk(-1, 0, -1, 2, 1, 3)};
    case CGTP_K_CONV_BWD:
      return {S(), mk(-1, -1, -1, 2, 1, 1), mk(-1, 0, -1, 2, 1, 1), mk(-1, 0, -1, 2, 1, 2), mk(-1, 0, -1, 2, 1, 3)};  // last: x phases
    case CGTP_K_CONV_BWD_ATOMIC:
      return {S(), mk(-1, -1, -1, 2, 1, 1), mk(-1, 0, -1, 2, 1, 1)};
    case CGTP_K_CONV_DBL_FWD:
      return {mk(-1, -1, -1, 1, 1, 1), mk(0, -1, -1, 1, 1, 1)};
    case CGTP_K_CONV_DBL_BWD:
      return {mk(-1, -1, -1, 2, 1, 1), mk(-1, 0, -1, 2, 1, 1)};
    case CGTP_K_TP_DBL_BWD: {
      // last: the economical schedule held to two waves per SIMD; a light spill at that occupancy measured
      // faster than no spill at one wave per SIMD (0.83 vs 1.05 ms on a 68-path plan)
      S two = mk(-1, -1, -1, 2, 1, 1);
      two.occ = 2;
      return {mk(-1, -1, -1, 1, 1, 1), mk(-1, -1, -1, 2, 1, 1), two, mk(-1, -1, -1, 2, 1, 2), mk(-1, -1, -1, 2, 1, 3),
              mk(-1, -1, -1, 2, 1, 5)};
    }
  }
  return {S()};
}

// Emits and compiles the candidates of one kernel in turn and keeps the first that is free of private-memory
// spills and (for plans with many paths) fits 256 registers, i.e. two waves per SIMD.  If none does, candidates
// are ranked: within 256 registers with a light spill (<= 256 B), then spill-free with more registers, then by
// the amount of spill.  Small plans keep their first spill-free schedule: those defaults were tuned by
// measurement and some of them are fastest with more than 256 registers.  Without compilation (device == -1)
// the first candidate is taken.
struct CompileError {
  std::string msg;
};

template <class Emit>
void build_kernel(cgtp::Plan& P, int kind, Emit emit, int device) {
  Kernel& K = P.k[kind];
  const bool small = P.paths.size() <= 24;
  std::vector<cgtp::Schedule> cands = schedule_candidates(kind, small);
  if (cgtp::env_int("CGTP_NO_SCHEDULE_SEARCH", 0)) cands.resize(1);
  Kernel best;
  long best_key = -1;
  std::string refused;
  for (size_t c = 0; c < cands.size(); ++c) {
    // phases cost re-reads (measured slower than a single phase at one wave per SIMD): they are tried only while
    // every schedule so far needs more than a light spill
    if (cands[c].phases > 1 && best_key >= 0 && best_key < 1000000L) continue;
    Kernel cur;
    cur.sched = cands[c];
    emit(cur);
    if (device == -1) {
      K = std::move(cur);
      return;
    }
    bool dup = false;   // environment overrides can make candidates identical
    if (best_key >= 0 && cur.source == best.source) dup = true;
    if (dup) continue;
    try {
      cgtp::jit_compile(cur, -2);
    } catch (const cgtp::RefusedCode& e) {   // this schedule's code failed the mask check: next candidate
      refused = e.what();
      continue;
    } catch (const std::exception& e) {
      throw CompileError{e.what()};
    }
    const bool fits = cur.scratch == 0 && (small || cur.vgprs <= 256);
    // ranking of the candidates that do not fit (many-path plans): within 256 registers with at most 256 B of
    // private memory, then spill-free with more registers (one wave per SIMD), then by the amount of spill
    long key;
    if (cur.scratch == 0) key = cur.vgprs <= 256 ? cur.vgprs : 20000L + cur.vgprs;
    else if (!small && cur.scratch <= 256 && cur.vgprs <= 256) key = 10000L + cur.scratch;
    else key = 1000000L + cur.scratch;
    if (best_key < 0 || key < best_key) {
      best = cur;
      best_key = key;
    }
    if (fits) {
      best = std::move(cur);
      break;
    }
  }
  if (best_key < 0 && !refused.empty()) throw CompileError{refused};
  K = std::move(best);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

cgtp_status launch(const Kernel& k, unsigned grid, void** args, hipStream_t st) {
  if (!k.fn) return fail(CGTP_EUNSUPPORTED, "kernel " + k.name + " is not loaded (plan created without a device?)");
  HIP_TRY(hipModuleLaunchKernel(k.fn, grid, 1, 1, (unsigned)k.wg, 1, 1, 0, st, args, nullptr));
  return CGTP_OK;
}

cgtp_status ensure_ws(Plan& P, size_t bytes) {
  if (bytes <= P.ws_bytes) return CGTP_OK;
  if (P.ws) {
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipFree(P.ws));
    P.ws = nullptr;
    P.ws_bytes = 0;
  }
  hipError_t e = hipMalloc(&P.ws, bytes);
  if (e != hipSuccess) return fail(CGTP_ENOMEM, "workspace allocation of " + std::to_string(bytes) + " bytes failed");
  P.ws_bytes = bytes;
  return CGTP_OK;
}

int64_t resident_waves(const Plan& P, const Kernel& k) { return (int64_t)k.blocks_per_cu * P.num_cu * (k.wg / 64); }

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

extern "C" {

const char* cgtp_last_error(void) { return g_err.c_str(); }

cgtp_status cgtp_check_code_object(const char* path, char* found, size_t capacity) {
  if (!path || !found || capacity == 0) return fail(CGTP_EINVAL, "NULL argument");
  try {
    const std::string t = cgtp::jit_check_code_object(path);
    std::snprintf(found, capacity, "%s", t.c_str());
  } catch (const std::exception& e) {
    return fail(CGTP_EINVAL, e.what());
  }
  return CGTP_OK;
}

cgtp_status cgtp_plan_create(const char* irreps_x, const char* irreps_y, const char* irreps_z, const cgtp_path* paths,
                             int32_t n_paths, int32_t default_mode, int32_t shared_weights, int32_t dtype,
                             int32_t device, uint32_t flags, cgtp_plan** out) {
  return cgtp_plan_create_ex(irreps_x, irreps_y, irreps_z, paths, n_paths, default_mode, shared_weights, dtype, device,
                             flags, nullptr, out);
}

cgtp_status cgtp_plan_create_ex(const char* irreps_x, const char* irreps_y, const char* irreps_z, const cgtp_path* paths,
                                int32_t n_paths, int32_t default_mode, int32_t shared_weights, int32_t dtype,
                                int32_t device, uint32_t flags, const cgtp_options* options, cgtp_plan** out) {
  if (!out) return fail(CGTP_EINVAL, "out is NULL");
  *out = nullptr;
  if (flags & ~(uint32_t)CGTP_IR_MUL) return fail(CGTP_EINVAL, "unknown bit in flags");
  bool kahan = false;
  if (options) {
    if (options->struct_size < (int32_t)sizeof(int32_t)) return fail(CGTP_EINVAL, "cgtp_options.struct_size is not set");
    if (options->struct_size >= (int32_t)(2 * sizeof(int32_t))) kahan = options->kahan_conv != 0;
  }
  if (!irreps_x || !irreps_y || !irreps_z) return fail(CGTP_EINVAL, "irreps string is NULL");
  if (dtype != CGTP_F32 && dtype != CGTP_F64) return fail(CGTP_EINVAL, "dtype must be CGTP_F32 or CGTP_F64");
  if (n_paths < 0 || (n_paths > 0 && !paths)) return fail(CGTP_EINVAL, "bad path list");
  if (default_mode != CGTP_UVU && default_mode != CGTP_UVW) return fail(CGTP_EINVAL, "bad default_mode");
  std::unique_ptr<cgtp_plan> H(new (std::nothrow) cgtp_plan());
  if (!H) return fail(CGTP_ENOMEM, "out of host memory");
  Plan& P = H->P;
  P.kahan_conv = kahan;
  try {
    P.irx = cgtp::parse_irreps(irreps_x);
    P.iry = cgtp::parse_irreps(irreps_y);
    P.irz = cgtp::parse_irreps(irreps_z);
  } catch (const std::invalid_argument& e) {
    return fail(CGTP_EINVAL, e.what());
  }
  for (auto* v : {&P.irx, &P.iry, &P.irz})
    for (auto& ir : *v)
      if (ir.l > cgtp::kMaxL) return fail(CGTP_EUNSUPPORTED, "degree l > 8 is not supported");
  P.offx = prefix(P.irx);
  P.offy = prefix(P.iry);
  P.offz = prefix(P.irz);
  P.dtype = dtype;
  P.shared_w = shared_weights != 0;
  P.device = device;
  P.ir_mul = (flags & CGTP_IR_MUL) != 0;

  std::vector<cgtp_path> list;
  if (n_paths == 0) {
    for (int a = 0; a < (int)P.irx.size(); ++a)
      for (int b = 0; b < (int)P.iry.size(); ++b)
        for (int c = 0; c < (int)P.irz.size(); ++c)
          if (allowed(P.irx[a], P.iry[b], P.irz[c])) list.push_back(cgtp_path{a, b, c, default_mode, 1.0});
  } else {
    list.assign(paths, paths + n_paths);
  }
  if (list.empty()) return fail(CGTP_EINVAL, "no path: nothing to compute");
  std::stable_sort(list.begin(), list.end(), [](const cgtp_path& a, const cgtp_path& b) {
    return std::tie(a.ix, a.iy, a.iz) < std::tie(b.ix, b.iy, b.iz);
  });
  P.mode = list[0].mode;
  int64_t woff = 0;
  for (auto& q : list) {
    if (q.ix < 0 || q.ix >= (int)P.irx.size() || q.iy < 0 || q.iy >= (int)P.iry.size() || q.iz < 0 ||
        q.iz >= (int)P.irz.size())
      return fail(CGTP_EINVAL, "path segment index out of range");
    if (q.mode != CGTP_UVU && q.mode != CGTP_UVW) return fail(CGTP_EINVAL, "bad path mode");
    const Irrep &a = P.irx[q.ix], &b = P.iry[q.iy], &c = P.irz[q.iz];
    if (!allowed(a, b, c)) return fail(CGTP_EINVAL, "path violates the triangle or parity rule");
    if (!std::isfinite(q.coeff)) return fail(CGTP_EINVAL, "path coefficient is not finite");
    if (b.mul != 1) return fail(CGTP_EUNSUPPORTED, "y multiplicity must be 1");
    if (q.mode != P.mode) return fail(CGTP_EUNSUPPORTED, "mixing uvu and uvw paths in one plan is not supported");
    if (q.mode == CGTP_UVU && a.mul != c.mul) return fail(CGTP_EINVAL, "uvu path needs mul_x == mul_z");
    PathInfo pi;
    pi.ix = q.ix; pi.iy = q.iy; pi.iz = q.iz; pi.mode = q.mode; pi.coeff = q.coeff;
    pi.l1 = a.l; pi.l2 = b.l; pi.l3 = c.l;
    pi.mul_x = a.mul; pi.mul_z = c.mul;
    pi.w_off = woff;
    try {
      pi.nz = cgtp::cg_nonzeros(a.l, b.l, c.l);
    } catch (const std::exception& e) {
      return fail(CGTP_ERUNTIME, e.what());
    }
    woff += (int64_t)a.mul * (q.mode == CGTP_UVU ? 1 : c.mul);
    P.paths.push_back(std::move(pi));
  }
  for (size_t t = 1; t < P.paths.size(); ++t)
    if (P.paths[t].ix == P.paths[t - 1].ix && P.paths[t].iy == P.paths[t - 1].iy && P.paths[t].iz == P.paths[t - 1].iz)
      return fail(CGTP_EINVAL, "duplicate path");
  P.n_w = woff;
  if (P.shared_w && P.mode == CGTP_UVU) return fail(CGTP_EUNSUPPORTED, "shared weights are supported for uvw plans only");
  if (P.ir_mul && P.mode != CGTP_UVU) return fail(CGTP_EUNSUPPORTED, "the IR_MUL layout is implemented for uvu plans only");

  for (int k = 0; k < 9; ++k) P.map[k] = pick_map(P, k);
  try {
    if (P.mode == CGTP_UVU) {
      // A convolution kernel whose wave holds several edge-range workers is lane-divergent by design.  If every
      // schedule of it is refused (see jit_compile: divergence together with register relocation), the kernel is
      // generated again with one worker per wave, which has no lane-conditional code.
      auto build_conv = [&](int kind, auto emit) {
        try {
          build_kernel(P, kind, emit, device);
        } catch (const CompileError&) {
          if (P.map[kind].spw <= 1) throw;
          LaneMap& m = P.map[kind];
          int M = 1;
          for (auto& q : P.paths) M = std::max(M, q.mul_x);
          m.G = 64;
          m.spw = 1;
          m.npass = (M + m.G * m.cpl - 1) / (m.G * m.cpl);
          build_kernel(P, kind, emit, device);
        }
      };
      build_kernel(P, CGTP_K_TP_FWD, [&](Kernel& k) { cgtp::emit_uvu_forward(P, false, k); }, device);
      build_kernel(P, CGTP_K_TP_BWD, [&](Kernel& k) { cgtp::emit_uvu_backward(P, false, k); }, device);
      build_conv(CGTP_K_CONV_FWD, [&](Kernel& k) { cgtp::emit_uvu_forward(P, true, k); });
      build_conv(CGTP_K_CONV_BWD, [&](Kernel& k) { cgtp::emit_uvu_backward(P, true, k); });
      build_conv(CGTP_K_CONV_FWD_ATOMIC, [&](Kernel& k) { cgtp::emit_uvu_atomic(P, false, k); });
      build_kernel(P, CGTP_K_CONV_BWD_ATOMIC, [&](Kernel& k) { cgtp::emit_uvu_atomic(P, true, k); }, device);
      build_kernel(P, CGTP_K_TP_DBL_BWD, [&](Kernel& k) { cgtp::emit_uvu_double_backward(P, k); }, device);
      build_conv(CGTP_K_CONV_DBL_FWD, [&](Kernel& k) { cgtp::emit_uvu_conv_double(P, false, k); });
      build_conv(CGTP_K_CONV_DBL_BWD, [&](Kernel& k) { cgtp::emit_uvu_conv_double(P, true, k); });
      cgtp::emit_fixup(P, P.k_fix);
    } else if (!P.shared_w) {
      cgtp::emit_uvw_ps_forward(P, P.k[CGTP_K_TP_FWD]);
      cgtp::emit_uvw_ps_backward(P, P.k[CGTP_K_TP_BWD]);
      // second-order pass: a forward-like kernel (dL/dgz; kept in the slot of the convolution's forward-like kernel,
      // which a uvw plan does not use) and a backward-like kernel (dL/dx, dL/dy, dL/dW)
      // CGTP_UVWPS_DBL_ONE=1 (default): the backward-like kernel computes dL/dgz as well, from the weight tiles it
      // holds in registers anyway (W and LC are then read once per call instead of twice); 0: two kernels
      const int one = cgtp::env_int("CGTP_UVWPS_DBL_ONE", 1) ? 1 : 0;
      if (!one) cgtp::emit_uvw_ps_double_forward(P, P.k[CGTP_K_CONV_DBL_FWD]);
      {
        // the backward-like kernel lands just above 256 registers for some plans (258 in fp64 on the DiffDock-shaped
        // benchmark): two waves per SIMD are asked of the compiler, and kept only if that costs at most 64 bytes of private memory
        Kernel& kd = P.k[CGTP_K_TP_DBL_BWD];
        kd.sched.occ = device == -1 ? 0 : 2;
        kd.sched.one_kernel = one;
        cgtp::emit_uvw_ps_double_backward(P, kd);
        if (device != -1) {
          cgtp::jit_compile(kd, -2);
          if (kd.scratch > 64) {   // a few spilled words are cheaper than one wave per SIMD
            kd = Kernel();
            kd.sched.occ = 0;
            kd.sched.one_kernel = one;
            cgtp::emit_uvw_ps_double_backward(P, kd);
          }
        }
      }
    } else {
      cgtp::emit_uvw_forward(P, P.k[CGTP_K_TP_FWD]);
      try {
        cgtp::emit_uvw_backward(P, P.k[CGTP_K_TP_BWD], P.k_fix);
      } catch (const cgtp::ShapeNotCovered&) {  // multiplicities the backward does not cover: forward-only plan
        P.k[CGTP_K_TP_BWD] = Kernel();          // (any other error of the emitter is a bug and is reported)
        P.k_fix = Kernel();
      }
    }
  } catch (const CompileError& e) {
    return fail(CGTP_ECOMPILE, e.msg);
  } catch (const std::exception& e) {
    return fail(CGTP_EUNSUPPORTED, e.what());
  }
  if (device >= 0) {
    HIP_TRY(hipSetDevice(device));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, device));
    P.num_cu = prop.multiProcessorCount;
    if (std::string(prop.gcnArchName).rfind("gfx950", 0) != 0)
      return fail(CGTP_EUNSUPPORTED, std::string("this library targets gfx950, device is ") + prop.gcnArchName);
  }
  try {
    for (auto& k : P.k) cgtp::jit_compile(k, device);
    cgtp::jit_compile(P.k_fix, device);
  } catch (const std::exception& e) {
    for (auto& k : P.k) cgtp::jit_unload(k);
    cgtp::jit_unload(P.k_fix);
    return fail(CGTP_ECOMPILE, e.what());
  }
  *out = H.release();
  return CGTP_OK;
}

cgtp_status cgtp_plan_destroy(cgtp_plan* plan) {
  if (!plan) return CGTP_OK;
  for (auto& k : plan->P.k) cgtp::jit_unload(k);
  cgtp::jit_unload(plan->P.k_fix);
  if (plan->P.ws) (void)hipFree(plan->P.ws);
  delete plan;
  return CGTP_OK;
}

int64_t cgtp_plan_dim(const cgtp_plan* plan, int32_t which) {
  if (!plan) return -1;
  switch (which) {
    case 0: return plan->P.dim_x();
    case 1: return plan->P.dim_y();
    case 2: return plan->P.dim_z();
    case 3: return plan->P.n_w;
    default: return -1;
  }
}

int32_t cgtp_plan_num_paths(const cgtp_plan* plan) { return plan ? (int32_t)plan->P.paths.size() : -1; }

cgtp_status cgtp_plan_get_path(const cgtp_plan* plan, int32_t p, cgtp_path* path, int32_t* l1l2l3, int32_t* nnz,
                               int64_t* w_offset) {
  if (!plan || p < 0 || p >= (int32_t)plan->P.paths.size()) return fail(CGTP_EINVAL, "bad plan or path index");
  const PathInfo& q = plan->P.paths[p];
  if (path) *path = cgtp_path{q.ix, q.iy, q.iz, q.mode, q.coeff};
  if (l1l2l3) {
    l1l2l3[0] = q.l1; l1l2l3[1] = q.l2; l1l2l3[2] = q.l3;
  }
  if (nnz) *nnz = (int32_t)q.nz.size();
  if (w_offset) *w_offset = q.w_off;
  return CGTP_OK;
}

int32_t cgtp_plan_path_nonzeros(const cgtp_plan* plan, int32_t p, int32_t cap, int32_t* i, int32_t* j, int32_t* k,
                                double* v) {
  if (!plan || p < 0 || p >= (int32_t)plan->P.paths.size()) return -1;
  const auto& nz = plan->P.paths[p].nz;
  for (int32_t t = 0; t < (int32_t)nz.size() && t < cap; ++t) {
    if (i) i[t] = nz[t].i;
    if (j) j[t] = nz[t].j;
    if (k) k[t] = nz[t].k;
    if (v) v[t] = nz[t].v;
  }
  return (int32_t)nz.size();
}

int64_t cgtp_plan_flops(const cgtp_plan* plan, int32_t which) {
  if (!plan) return -1;
  int64_t cg = 0, w = 0;
  for (auto& q : plan->P.paths) {
    cg += 2LL * (int64_t)q.nz.size() * q.mul_x;
    w += 2LL * (2 * q.l3 + 1) * (q.mode == CGTP_UVU ? (int64_t)q.mul_x : (int64_t)q.mul_x * q.mul_z);
  }
  if (which == 0) return cg + w;
  // backward: 3x the contraction; the weight part is 1.5x for uvu (g' = w*gz, gW += z'*gz) and 2x for uvw (two GEMMs)
  if (which == 1) return 3 * cg + (plan->P.mode == CGTP_UVU ? (3 * w) / 2 : 2 * w);
  // fused second-order pass.  uvu: 8 FMAs per nonzero and channel.  uvw (per-sample weights), one kernel: z' three times
  // (S = z'(La, y) + z'(x, Lb) and Z = z'(x, y)), dL/dx and dL/dy with two terms each -> 7x the contraction; five dense
  // products (W S, LC Z, S (x) gz, W gz, LC gz) -> 5x the weight part.  The two-kernel variant forms S twice more: 9x.
  if (which == 2) return plan->P.mode == CGTP_UVU ? 8 * cg + 3 * w : (plan->P.k[CGTP_K_TP_DBL_BWD].sched.one_kernel > 0 ? 7 : 9) * cg + 5 * w;
  return -1;
}

const char* cgtp_plan_source(const cgtp_plan* plan, int32_t kernel) {
  if (!plan || kernel < 0 || kernel > 8) return nullptr;
  const std::string& s = plan->P.k[kernel].source;
  return s.empty() ? nullptr : s.c_str();
}

cgtp_status cgtp_plan_kernel_info(const cgtp_plan* plan, int32_t kernel, int32_t info[6]) {
  if (!plan || kernel < 0 || kernel > 8 || !info) return fail(CGTP_EINVAL, "bad argument");
  const Kernel& k = plan->P.k[kernel];
  if (!k.fn && k.vgprs == 0) return fail(CGTP_EUNSUPPORTED, "kernel is neither compiled nor loaded");
  info[0] = k.vgprs; info[1] = k.sgprs; info[2] = k.lds; info[3] = k.scratch; info[4] = k.wg; info[5] = k.blocks_per_cu;
  return CGTP_OK;
}

cgtp_status tp_forward(cgtp_plan* plan, const void* x, const void* y, const void* W, void* z, int64_t B,
                       void* hip_stream) {
  if (!plan) return fail(CGTP_EINVAL, "plan is NULL");
  if (B < 0) return fail(CGTP_EINVAL, "negative batch size");
  if (B == 0) return CGTP_OK;
  if (!x || !y || !W || !z) return fail(CGTP_EINVAL, "NULL data pointer");
  if (!aligned16(x) || !aligned16(y) || !aligned16(W) || !aligned16(z)) return fail(CGTP_EINVAL, "data pointers must be 16-byte aligned");
  Plan& P = plan->P;
  const Kernel& k = P.k[CGTP_K_TP_FWD];
  hipStream_t st = (hipStream_t)hip_stream;
  if (P.mode == CGTP_UVU) {
    const int wpw = k.wg / 64;
    int64_t need = (B + (int64_t)P.map[CGTP_K_TP_FWD].spw * wpw - 1) / ((int64_t)P.map[CGTP_K_TP_FWD].spw * wpw);
    int64_t cap = std::max<int64_t>(1, (int64_t)k.blocks_per_cu * P.num_cu * cgtp::env_int("CGTP_GRID_MULT", 8));
    unsigned grid = (unsigned)std::min(need, cap);
    void* args[] = {(void*)&x, (void*)&y, (void*)&W, (void*)&z, (void*)&B};
    return launch(k, grid, args, st);
  }
  if (!P.shared_w) {   // per-sample weights: one wave per sample, grid-stride
    const int wpw = k.wg / 64;
    int64_t need = (B + wpw - 1) / wpw;
    int64_t cap = std::max<int64_t>(1, (int64_t)k.blocks_per_cu * P.num_cu * cgtp::env_int("CGTP_GRID_MULT", 8));
    unsigned grid = (unsigned)std::min(need, cap);
    void* args[] = {(void*)&x, (void*)&y, (void*)&W, (void*)&z, (void*)&B};
    return launch(k, grid, args, st);
  }
  // uvw: one workgroup per tile of samples (geometry fixed by the emitter: k.wg threads, tile in k.lds slot)
  // persistent workgroups: the weights are copied to LDS once per workgroup
  // at most one workgroup per 16-sample tile: the tiles of the last, incomplete round of the waves are worked on by
  // a whole workgroup each (for a small batch that is every tile)
  int64_t need = (B + 15) / 16;
  int64_t cap = std::max<int64_t>(1, (int64_t)k.blocks_per_cu * P.num_cu);
  unsigned grid = (unsigned)std::min(need, cap);
  void* args[] = {(void*)&x, (void*)&y, (void*)&W, (void*)&z, (void*)&B};
  return launch(k, grid, args, st);
}

cgtp_status tp_backward(cgtp_plan* plan, const void* x, const void* y, const void* W, const void* gz, void* gx,
                        void* gy, void* gW, int64_t B, void* hip_stream) {
  if (!plan) return fail(CGTP_EINVAL, "plan is NULL");
  if (B < 0) return fail(CGTP_EINVAL, "negative batch size");
  Plan& P = plan->P;
  if (P.mode != CGTP_UVU && P.k[CGTP_K_TP_BWD].source.empty())
    return fail(CGTP_EUNSUPPORTED, "backward of this uvw plan is not supported (needs mul_x, mul_z multiples of 16)");
  if (B == 0 && (P.mode == CGTP_UVU || !P.shared_w)) return CGTP_OK;
  if (B == 0) {   // shared weights: gW is the empty sum; no other buffer is touched
    if (!gW || !aligned16(gW)) return fail(CGTP_EINVAL, "gW must be a 16-byte aligned device pointer");
    HIP_TRY(cgtp::launch_fill_zero(gW, (size_t)P.n_w * P.elt(), (hipStream_t)hip_stream));
    return CGTP_OK;
  }
  if (!x || !y || !W || !gz || !gx || !gy || !gW) return fail(CGTP_EINVAL, "NULL data pointer");
  for (const void* p : {x, y, W, gz, (const void*)gx, (const void*)gy, (const void*)gW})
    if (!aligned16(p)) return fail(CGTP_EINVAL, "data pointers must be 16-byte aligned");
  const Kernel& k = P.k[CGTP_K_TP_BWD];
  const int wpw = k.wg / 64;
  if (P.mode == CGTP_UVW && !P.shared_w) {   // per-sample weights: gW [B, n_w], one wave per sample
    int64_t need = (B + wpw - 1) / wpw;
    int64_t cap = std::max<int64_t>(1, (int64_t)k.blocks_per_cu * P.num_cu * cgtp::env_int("CGTP_GRID_MULT", 8));
    unsigned grid = (unsigned)std::min(need, cap);
    void* args[] = {(void*)&x, (void*)&y, (void*)&W, (void*)&gz, (void*)&gx, (void*)&gy, (void*)&gW, (void*)&B};
    return launch(k, grid, args, (hipStream_t)hip_stream);
  }
  if (P.mode == CGTP_UVW) {
    // shared weights: gW [n_w] is the sum over the batch; per-wave partial sums go through the workspace
    hipStream_t st = (hipStream_t)hip_stream;
    int64_t tile = cgtp::uvw_tile_samples(P);
    unsigned grid = (unsigned)std::min<int64_t>((B + tile - 1) / tile, std::max<int64_t>(1, (int64_t)k.blocks_per_cu * P.num_cu));
    int64_t nparts = grid;   // one partial gW per workgroup
    cgtp_status s = ensure_ws(P, (size_t)nparts * P.n_w * P.elt());
    if (s != CGTP_OK) return s;
    void* part = P.ws;
    void* args[] = {(void*)&x, (void*)&y, (void*)&W, (void*)&gz, (void*)&gx, (void*)&gy, (void*)&part, (void*)&B};
    s = launch(k, grid, args, st);
    if (s != CGTP_OK) return s;
    int64_t n = P.n_w;
    void* rargs[] = {(void*)&part, (void*)&gW, (void*)&nparts, (void*)&n};
    return launch(P.k_fix, (unsigned)((n + 63) / 64), rargs, st);
  }
  int64_t need = (B + (int64_t)P.map[CGTP_K_TP_BWD].spw * wpw - 1) / ((int64_t)P.map[CGTP_K_TP_BWD].spw * wpw);
  int64_t cap = std::max<int64_t>(1, (int64_t)k.blocks_per_cu * P.num_cu * cgtp::env_int("CGTP_GRID_MULT", 8));
  unsigned grid = (unsigned)std::min(need, cap);
  void* args[] = {(void*)&x, (void*)&y, (void*)&W, (void*)&gz, (void*)&gx, (void*)&gy, (void*)&gW, (void*)&B};
  return launch(k, grid, args, (hipStream_t)hip_stream);
}

cgtp_status tp_double_backward(cgtp_plan* plan, const void* x, const void* y, const void* W, const void* gz,
                               const void* La, const void* Lb, const void* LC, void* Lx, void* Ly, void* LW,
                               void* Lgz, int64_t B, void* hip_stream) {
  if (!plan) return fail(CGTP_EINVAL, "plan is NULL");
  if (B < 0) return fail(CGTP_EINVAL, "negative batch size");
  Plan& P = plan->P;
  if (P.mode != CGTP_UVU && P.shared_w) return fail(CGTP_EUNSUPPORTED, "double backward is not implemented for uvw plans with shared weights");
  if (B == 0) return CGTP_OK;
  if (P.mode != CGTP_UVU) {
    // uvw with per-sample weights: one kernel for all four results (W and LC streamed once), or, for plans created
    // with CGTP_UVWPS_DBL_ONE=0, the split of paper Sec. 3.4 into a forward-like and a backward-like kernel (each
    // streams W and LC); one wave per sample, no workspace
    for (const void* p : {x, y, W, gz, La, Lb, LC, (const void*)Lx, (const void*)Ly, (const void*)LW, (const void*)Lgz}) {
      if (!p) return fail(CGTP_EINVAL, "NULL data pointer");
      if (!aligned16(p)) return fail(CGTP_EINVAL, "data pointers must be 16-byte aligned");
    }
    hipStream_t st = (hipStream_t)hip_stream;
    // CGTP_UVWPS_DBL_FUSED=0 (environment) selects the unfused route instead of the fused kernel(s): a second
    // way to the same result, kept for verification
    if (cgtp::env_int("CGTP_UVWPS_DBL_FUSED", 1) == 0) {
      // the seven dispatches of paper Sec. 3.4 as they stand (three forward, four backward calls on
      // permuted operands), sums formed in place; temporaries [B, dim_x + dim_y + dim_z + n_w] in the plan's
      // workspace (the per-sample kernels themselves use none)
      const size_t el = P.elt();
      const size_t nx = round_up((size_t)B * P.dim_x() * el, 256), ny = round_up((size_t)B * P.dim_y() * el, 256),
                   nz = round_up((size_t)B * P.dim_z() * el, 256), nw = round_up((size_t)B * P.n_w * el, 256);
      cgtp_status s = ensure_ws(P, nx + ny + nz + nw);
      if (s != CGTP_OK) return s;
      char* base = (char*)P.ws;
      void *tx = base, *ty = base + nx, *tz = base + nx + ny, *tw = base + nx + ny + nz;
      const bool f64 = P.dtype == CGTP_F64;
      auto add = [&](void* a, const void* b_, int64_t n) -> cgtp_status {
        HIP_TRY(cgtp::launch_add_inplace(a, b_, n, f64, st));
        return CGTP_OK;
      };
#define DBL_TRY(e) do { cgtp_status s_ = (e); if (s_ != CGTP_OK) return s_; } while (0)
      DBL_TRY(tp_backward(plan, La, Lb, W, gz, Lx, Ly, tw, B, hip_stream));     // op1 -> dL/dx, dL/dy
      DBL_TRY(tp_backward(plan, x, y, LC, gz, tx, ty, tw, B, hip_stream));      // op2
      DBL_TRY(add(Lx, tx, B * P.dim_x()));
      DBL_TRY(add(Ly, ty, B * P.dim_y()));
      DBL_TRY(tp_forward(plan, La, y, W, Lgz, B, hip_stream));                  // op3 -> dL/dgz
      DBL_TRY(tp_forward(plan, x, Lb, W, tz, B, hip_stream));                   // op6
      DBL_TRY(add(Lgz, tz, B * P.dim_z()));
      DBL_TRY(tp_forward(plan, x, y, LC, tz, B, hip_stream));                   // op7
      DBL_TRY(add(Lgz, tz, B * P.dim_z()));
      DBL_TRY(tp_backward(plan, La, y, W, gz, tx, ty, LW, B, hip_stream));      // op4 -> dL/dW
      DBL_TRY(tp_backward(plan, x, Lb, W, gz, tx, ty, tw, B, hip_stream));      // op5
      DBL_TRY(add(LW, tw, B * P.n_w));
#undef DBL_TRY
      return CGTP_OK;
    }
    const bool one = P.k[CGTP_K_TP_DBL_BWD].sched.one_kernel > 0;
    for (int which = one ? 1 : 0; which < 2; ++which) {
      const Kernel& kk = P.k[which == 0 ? CGTP_K_CONV_DBL_FWD : CGTP_K_TP_DBL_BWD];
      const int wpw_ = kk.wg / 64;
      int64_t need = (B + wpw_ - 1) / wpw_;
      int64_t cap = std::max<int64_t>(1, (int64_t)kk.blocks_per_cu * P.num_cu * cgtp::env_int("CGTP_GRID_MULT", 8));
      unsigned grid = (unsigned)std::min(need, cap);
      cgtp_status s_;
      if (which == 0) {
        void* args[] = {(void*)&x, (void*)&y, (void*)&W, (void*)&La, (void*)&Lb, (void*)&LC, (void*)&Lgz, (void*)&B};
        s_ = launch(kk, grid, args, st);
      } else {
        void* args[] = {(void*)&x, (void*)&y, (void*)&W, (void*)&gz, (void*)&La, (void*)&Lb, (void*)&LC, (void*)&Lx, (void*)&Ly, (void*)&LW, (void*)&B};
        void* args1[] = {(void*)&x, (void*)&y, (void*)&W, (void*)&gz, (void*)&La, (void*)&Lb, (void*)&LC, (void*)&Lx, (void*)&Ly, (void*)&LW, (void*)&Lgz, (void*)&B};
        s_ = launch(kk, grid, one ? args1 : args, st);
      }
      if (s_ != CGTP_OK) return s_;
    }
    return CGTP_OK;
  }
  for (const void* p : {x, y, W, gz, La, Lb, LC, (const void*)Lx, (const void*)Ly, (const void*)LW, (const void*)Lgz}) {
    if (!p) return fail(CGTP_EINVAL, "NULL data pointer");
    if (!aligned16(p)) return fail(CGTP_EINVAL, "data pointers must be 16-byte aligned");
  }
  const Kernel& k = P.k[CGTP_K_TP_DBL_BWD];
  const int wpw = k.wg / 64;
  const int64_t per_wg = (int64_t)P.map[CGTP_K_TP_DBL_BWD].spw * wpw;
  int64_t need = (B + per_wg - 1) / per_wg;
  int64_t cap = std::max<int64_t>(1, (int64_t)k.blocks_per_cu * P.num_cu * cgtp::env_int("CGTP_GRID_MULT_DBL", 2));
  unsigned grid = (unsigned)std::min(need, cap);
  void* args[] = {(void*)&x,  (void*)&y,  (void*)&W,  (void*)&gz,  (void*)&La,  (void*)&Lb,
                  (void*)&LC, (void*)&Lx, (void*)&Ly, (void*)&LW, (void*)&Lgz, (void*)&B};
  return launch(k, grid, args, (hipStream_t)hip_stream);
}

cgtp_status conv_forward(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges, void* z_nodes,
                         int64_t V, int64_t E, const int64_t* row_ptr, const int64_t* col, void* hip_stream) {
  return conv_forward_perm(plan, x_nodes, y_edges, W_edges, z_nodes, V, E, row_ptr, col, nullptr, hip_stream);
}

}  // extern "C"

namespace {
// conv_forward / conv_forward_perm / conv_forward_static.  use_static: the side buffer of split rows is the library's
// static device array instead of the plan's workspace (nothing is allocated).
cgtp_status conv_forward_impl(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                              void* z_nodes, int64_t V, int64_t E, const int64_t* row_ptr, const int64_t* col,
                              const int64_t* edge_perm, void* hip_stream, bool use_static) {
  if (!plan) return fail(CGTP_EINVAL, "plan is NULL");
  if (V < 0 || E < 0) return fail(CGTP_EINVAL, "negative size");
  Plan& P = plan->P;
  if (P.mode != CGTP_UVU) return fail(CGTP_EUNSUPPORTED, "convolution is implemented for uvu plans only");
  if (V == 0) return E == 0 ? CGTP_OK : fail(CGTP_EINVAL, "edges without nodes");
  if (!z_nodes || !row_ptr) return fail(CGTP_EINVAL, "NULL data pointer");
  hipStream_t st = (hipStream_t)hip_stream;
  if (!aligned16(z_nodes)) return fail(CGTP_EINVAL, "data pointers must be 16-byte aligned");
  if (E == 0) {
    HIP_TRY(cgtp::launch_fill_zero(z_nodes, (size_t)V * P.dim_z() * P.elt(), st));
    return CGTP_OK;
  }
  if (!x_nodes || !y_edges || !W_edges || !col) return fail(CGTP_EINVAL, "NULL data pointer");
  if (!aligned16(x_nodes) || !aligned16(y_edges) || !aligned16(W_edges)) return fail(CGTP_EINVAL, "data pointers must be 16-byte aligned");
  const Kernel& k = P.k[CGTP_K_CONV_FWD];
  if (!k.fn) return fail(CGTP_EUNSUPPORTED, "kernel is not loaded (plan created without a device?)");
  const int spw = P.map[CGTP_K_CONV_FWD].spw;   // edge-range workers per wave
  int64_t nchunk = std::min<int64_t>(E, resident_waves(P, k) * spw * cgtp::env_int("CGTP_CONV_CHUNK_MULT", 1));
  size_t part_bytes = (size_t)nchunk * 2 * P.dim_z() * P.elt();
  void* part = nullptr;
  cgtp_status s = CGTP_OK;
  if (use_static) {
    int cur = -1;
    HIP_TRY(hipGetDevice(&cur));
    if (cur != P.device) return fail(CGTP_EINVAL, "the plan's device is not the current device");
    size_t cap = 0;
    hipError_t e = cgtp::static_scratch(&part, &cap);
    if (e != hipSuccess) return fail(CGTP_ERUNTIME, std::string("static scratch: ") + hipGetErrorString(e));
    if (part_bytes > cap)
      return fail(CGTP_EINVAL, "conv_forward_static: this problem needs " + std::to_string(part_bytes) + " bytes of scratch for " +
                                   std::to_string(nchunk) + " edge ranges, the static buffer holds " + std::to_string(cap) +
                                   "; use conv_forward");
  } else {
    s = ensure_ws(P, part_bytes);
    if (s != CGTP_OK) return s;
    part = P.ws;
  }
  const int wpw = k.wg / 64;
  unsigned grid = (unsigned)((nchunk + (int64_t)wpw * spw - 1) / ((int64_t)wpw * spw));
  void* args[] = {(void*)&x_nodes, (void*)&y_edges, (void*)&W_edges, (void*)&z_nodes, (void*)&row_ptr,  (void*)&col,
                  (void*)&V,       (void*)&E,       (void*)&part,    (void*)&nchunk,  (void*)&edge_perm};
  s = launch(k, grid, args, st);
  if (s != CGTP_OK) return s;
  int dim = (int)P.dim_z();
  void* fargs[] = {(void*)&z_nodes, (void*)&part, (void*)&row_ptr, (void*)&V, (void*)&E, (void*)&nchunk, (void*)&dim};
  return launch(P.k_fix, (unsigned)nchunk, fargs, st);
}
}  // namespace

extern "C" {

cgtp_status conv_forward_perm(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                              void* z_nodes, int64_t V, int64_t E, const int64_t* row_ptr, const int64_t* col,
                              const int64_t* edge_perm, void* hip_stream) {
  return conv_forward_impl(plan, x_nodes, y_edges, W_edges, z_nodes, V, E, row_ptr, col, edge_perm, hip_stream, false);
}

cgtp_status conv_forward_static(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                                void* z_nodes, int64_t V, int64_t E, const int64_t* row_ptr, const int64_t* col,
                                void* hip_stream) {
  return conv_forward_impl(plan, x_nodes, y_edges, W_edges, z_nodes, V, E, row_ptr, col, nullptr, hip_stream, true);
}

cgtp_status conv_backward(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                          const void* gz_nodes, void* gx_nodes, void* gy_edges, void* gW_edges, int64_t V, int64_t E,
                          const int64_t* row_ptr, const int64_t* col, const int64_t* t_row_ptr, const int64_t* t_perm,
                          void* hip_stream) {
  return conv_backward_perm(plan, x_nodes, y_edges, W_edges, gz_nodes, gx_nodes, gy_edges, gW_edges, V, E, row_ptr, col,
                            t_row_ptr, t_perm, nullptr, hip_stream);
}

cgtp_status conv_backward_perm(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                               const void* gz_nodes, void* gx_nodes, void* gy_edges, void* gW_edges, int64_t V,
                               int64_t E, const int64_t* row_ptr, const int64_t* col, const int64_t* t_row_ptr,
                               const int64_t* t_perm, const int64_t* edge_perm, void* hip_stream) {
  (void)col;
  if (!plan) return fail(CGTP_EINVAL, "plan is NULL");
  if (V < 0 || E < 0) return fail(CGTP_EINVAL, "negative size");
  Plan& P = plan->P;
  if (P.mode != CGTP_UVU) return fail(CGTP_EUNSUPPORTED, "convolution is implemented for uvu plans only");
  if (V == 0) return E == 0 ? CGTP_OK : fail(CGTP_EINVAL, "edges without nodes");
  if (!gx_nodes) return fail(CGTP_EINVAL, "NULL data pointer");
  hipStream_t st = (hipStream_t)hip_stream;
  if (E == 0) {
    HIP_TRY(cgtp::launch_fill_zero(gx_nodes, (size_t)V * P.dim_x() * P.elt(), st));
    return CGTP_OK;
  }
  if (!x_nodes || !y_edges || !W_edges || !gz_nodes || !gy_edges || !gW_edges || !row_ptr || !t_row_ptr || !t_perm)
    return fail(CGTP_EINVAL, "NULL data pointer");
  for (const void* p : {x_nodes, y_edges, W_edges, gz_nodes, (const void*)gx_nodes, (const void*)gy_edges, (const void*)gW_edges})
    if (!aligned16(p)) return fail(CGTP_EINVAL, "data pointers must be 16-byte aligned");
  const Kernel& k = P.k[CGTP_K_CONV_BWD];
  if (!k.fn) return fail(CGTP_EUNSUPPORTED, "kernel is not loaded (plan created without a device?)");
  const int spw = P.map[CGTP_K_CONV_BWD].spw;   // edge-range workers per wave
  int64_t nchunk = std::min<int64_t>(E, resident_waves(P, k) * spw * cgtp::env_int("CGTP_CONV_CHUNK_MULT", 1));
  size_t part_bytes = round_up((size_t)nchunk * 2 * P.dim_x() * P.elt(), 256);
  const size_t recv_bytes = round_up((size_t)E * 8, 256);
  // one scratch row for the gy / gW words of the pipelined kernel's phantom edge (odd edge ranges)
  const size_t dummy_bytes = (round_up((size_t)P.dim_y(), 64) + (size_t)P.n_w) * P.elt();
  cgtp_status s = ensure_ws(P, part_bytes + recv_bytes + dummy_bytes);
  if (s != CGTP_OK) return s;
  void* part = P.ws;
  int64_t* t_recv = (int64_t*)((char*)P.ws + part_bytes);
  void* dummy = (char*)P.ws + part_bytes + recv_bytes;
  HIP_TRY(cgtp::launch_recv_of_tperm(row_ptr, t_perm, V, E, t_recv, st));
  const int wpw = k.wg / 64;
  unsigned grid = (unsigned)((nchunk + (int64_t)wpw * spw - 1) / ((int64_t)wpw * spw));
  void* args[] = {(void*)&x_nodes,  (void*)&y_edges,  (void*)&W_edges, (void*)&gz_nodes, (void*)&gx_nodes,
                  (void*)&gy_edges, (void*)&gW_edges, (void*)&t_row_ptr, (void*)&t_perm, (void*)&t_recv,
                  (void*)&V,        (void*)&E,        (void*)&part,    (void*)&nchunk,   (void*)&edge_perm,
                  (void*)&dummy};
  s = launch(k, grid, args, st);
  if (s != CGTP_OK) return s;
  int dim = (int)P.dim_x();
  void* fargs[] = {(void*)&gx_nodes, (void*)&part, (void*)&t_row_ptr, (void*)&V, (void*)&E, (void*)&nchunk, (void*)&dim};
  return launch(P.k_fix, (unsigned)nchunk, fargs, st);
}

cgtp_status conv_double_backward(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                                 const void* gz_nodes, const void* La_nodes, const void* Lb_edges,
                                 const void* LC_edges, void* Lx_nodes, void* Ly_edges, void* LW_edges,
                                 void* Lgz_nodes, int64_t V, int64_t E, const int64_t* row_ptr, const int64_t* col,
                                 const int64_t* t_row_ptr, const int64_t* t_perm, void* hip_stream) {
  if (!plan) return fail(CGTP_EINVAL, "plan is NULL");
  if (V < 0 || E < 0) return fail(CGTP_EINVAL, "negative size");
  Plan& P = plan->P;
  if (P.mode != CGTP_UVU) return fail(CGTP_EUNSUPPORTED, "convolution is implemented for uvu plans only");
  if (V == 0) return E == 0 ? CGTP_OK : fail(CGTP_EINVAL, "edges without nodes");
  if (!Lx_nodes || !Lgz_nodes) return fail(CGTP_EINVAL, "NULL data pointer");
  hipStream_t st = (hipStream_t)hip_stream;
  if (E == 0) {
    HIP_TRY(cgtp::launch_fill_zero(Lx_nodes, (size_t)V * P.dim_x() * P.elt(), st));
    HIP_TRY(cgtp::launch_fill_zero(Lgz_nodes, (size_t)V * P.dim_z() * P.elt(), st));
    return CGTP_OK;
  }
  for (const void* p : {x_nodes, y_edges, W_edges, gz_nodes, La_nodes, Lb_edges, LC_edges, (const void*)Lx_nodes,
                        (const void*)Ly_edges, (const void*)LW_edges, (const void*)Lgz_nodes}) {
    if (!p) return fail(CGTP_EINVAL, "NULL data pointer");
    if (!aligned16(p)) return fail(CGTP_EINVAL, "data pointers must be 16-byte aligned");
  }
  if (!row_ptr || !col || !t_row_ptr || !t_perm) return fail(CGTP_EINVAL, "NULL graph pointer");
  const Kernel& kf = P.k[CGTP_K_CONV_DBL_FWD];
  const Kernel& kb = P.k[CGTP_K_CONV_DBL_BWD];
  if (!kf.fn || !kb.fn) return fail(CGTP_EUNSUPPORTED, "kernel is not loaded (plan created without a device?)");
  const int spwf = P.map[CGTP_K_CONV_DBL_FWD].spw, spwb = P.map[CGTP_K_CONV_DBL_BWD].spw;
  const int mult = cgtp::env_int("CGTP_CONV_CHUNK_MULT", 1);
  int64_t nf = std::min<int64_t>(E, resident_waves(P, kf) * spwf * mult);
  int64_t nb = std::min<int64_t>(E, resident_waves(P, kb) * spwb * mult);
  // the two walks run one after the other on the stream and share the side buffer
  size_t part_f = (size_t)nf * 2 * P.dim_z() * P.elt();
  size_t part_b = round_up((size_t)nb * 2 * P.dim_x() * P.elt(), 256);
  cgtp_status s = ensure_ws(P, std::max(part_f, part_b + (size_t)E * 8));
  if (s != CGTP_OK) return s;
  void* part = P.ws;
  {
    const int wpw = kf.wg / 64;
    unsigned grid = (unsigned)((nf + (int64_t)wpw * spwf - 1) / ((int64_t)wpw * spwf));
    void* args[] = {(void*)&x_nodes,   (void*)&y_edges, (void*)&W_edges, (void*)&La_nodes, (void*)&Lb_edges, (void*)&LC_edges,
                    (void*)&Lgz_nodes, (void*)&row_ptr, (void*)&col,     (void*)&V,        (void*)&E,        (void*)&part,
                    (void*)&nf};
    s = launch(kf, grid, args, st);
    if (s != CGTP_OK) return s;
    int dim = (int)P.dim_z();
    void* fargs[] = {(void*)&Lgz_nodes, (void*)&part, (void*)&row_ptr, (void*)&V, (void*)&E, (void*)&nf, (void*)&dim};
    s = launch(P.k_fix, (unsigned)nf, fargs, st);
    if (s != CGTP_OK) return s;
  }
  int64_t* t_recv = (int64_t*)((char*)P.ws + part_b);
  HIP_TRY(cgtp::launch_recv_of_tperm(row_ptr, t_perm, V, E, t_recv, st));
  {
    const int wpw = kb.wg / 64;
    unsigned grid = (unsigned)((nb + (int64_t)wpw * spwb - 1) / ((int64_t)wpw * spwb));
    void* args[] = {(void*)&x_nodes,  (void*)&y_edges,  (void*)&W_edges,  (void*)&gz_nodes, (void*)&La_nodes, (void*)&Lb_edges,
                    (void*)&LC_edges, (void*)&Lx_nodes, (void*)&Ly_edges, (void*)&LW_edges, (void*)&t_row_ptr, (void*)&t_perm,
                    (void*)&t_recv,   (void*)&V,        (void*)&E,        (void*)&part,     (void*)&nb};
    s = launch(kb, grid, args, st);
    if (s != CGTP_OK) return s;
    int dim = (int)P.dim_x();
    void* fargs[] = {(void*)&Lx_nodes, (void*)&part, (void*)&t_row_ptr, (void*)&V, (void*)&E, (void*)&nb, (void*)&dim};
    return launch(P.k_fix, (unsigned)nb, fargs, st);
  }
}

cgtp_status conv_forward_atomic(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                                void* z_nodes, int64_t V, int64_t E, const int64_t* recv, const int64_t* send,
                                void* hip_stream) {
  if (!plan) return fail(CGTP_EINVAL, "plan is NULL");
  if (V < 0 || E < 0) return fail(CGTP_EINVAL, "negative size");
  Plan& P = plan->P;
  if (P.mode != CGTP_UVU) return fail(CGTP_EUNSUPPORTED, "convolution is implemented for uvu plans only");
  if (V == 0) return E == 0 ? CGTP_OK : fail(CGTP_EINVAL, "edges without nodes");
  if (!z_nodes || !aligned16(z_nodes)) return fail(CGTP_EINVAL, "z_nodes must be a 16-byte aligned device pointer");
  hipStream_t st = (hipStream_t)hip_stream;
  HIP_TRY(cgtp::launch_fill_zero(z_nodes, (size_t)V * P.dim_z() * P.elt(), st));
  if (E == 0) return CGTP_OK;
  if (!x_nodes || !y_edges || !W_edges || !recv || !send) return fail(CGTP_EINVAL, "NULL data pointer");
  if (!aligned16(x_nodes) || !aligned16(y_edges) || !aligned16(W_edges)) return fail(CGTP_EINVAL, "data pointers must be 16-byte aligned");
  const Kernel& k = P.k[CGTP_K_CONV_FWD_ATOMIC];
  const int wpw = k.wg / 64;
  const int spw = P.map[CGTP_K_CONV_FWD_ATOMIC].spw;   // edge-range workers per wave
  int64_t nchunk = std::min<int64_t>(E, resident_waves(P, k) * spw * cgtp::env_int("CGTP_CONV_CHUNK_MULT", 1));
  unsigned grid = (unsigned)((nchunk + (int64_t)wpw * spw - 1) / ((int64_t)wpw * spw));
  const int64_t* no_perm = nullptr;
  void* args[] = {(void*)&x_nodes, (void*)&y_edges, (void*)&W_edges, (void*)&z_nodes, (void*)&recv,
                  (void*)&send,    (void*)&E,       (void*)&nchunk,  (void*)&no_perm};
  return launch(k, grid, args, st);
}

cgtp_status conv_backward_atomic(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                                 const void* gz_nodes, void* gx_nodes, void* gy_edges, void* gW_edges, int64_t V,
                                 int64_t E, const int64_t* recv, const int64_t* send, void* hip_stream) {
  if (!plan) return fail(CGTP_EINVAL, "plan is NULL");
  if (V < 0 || E < 0) return fail(CGTP_EINVAL, "negative size");
  Plan& P = plan->P;
  if (P.mode != CGTP_UVU) return fail(CGTP_EUNSUPPORTED, "convolution is implemented for uvu plans only");
  if (V == 0) return E == 0 ? CGTP_OK : fail(CGTP_EINVAL, "edges without nodes");
  if (!gx_nodes || !aligned16(gx_nodes)) return fail(CGTP_EINVAL, "gx_nodes must be a 16-byte aligned device pointer");
  hipStream_t st = (hipStream_t)hip_stream;
  HIP_TRY(cgtp::launch_fill_zero(gx_nodes, (size_t)V * P.dim_x() * P.elt(), st));
  if (E == 0) return CGTP_OK;
  if (!x_nodes || !y_edges || !W_edges || !gz_nodes || !gy_edges || !gW_edges || !recv || !send)
    return fail(CGTP_EINVAL, "NULL data pointer");
  for (const void* p : {x_nodes, y_edges, W_edges, gz_nodes, (const void*)gy_edges, (const void*)gW_edges})
    if (!aligned16(p)) return fail(CGTP_EINVAL, "data pointers must be 16-byte aligned");
  const Kernel& k = P.k[CGTP_K_CONV_BWD_ATOMIC];
  const int wpw = k.wg / 64;
  const int spw = P.map[CGTP_K_CONV_BWD_ATOMIC].spw;
  int64_t need = (E + (int64_t)spw * wpw - 1) / ((int64_t)spw * wpw);
  int64_t cap = std::max<int64_t>(1, (int64_t)k.blocks_per_cu * P.num_cu * cgtp::env_int("CGTP_GRID_MULT", 8));
  void* args[] = {(void*)&x_nodes,  (void*)&y_edges,  (void*)&W_edges, (void*)&gz_nodes, (void*)&gx_nodes,
                  (void*)&gy_edges, (void*)&gW_edges, (void*)&recv,    (void*)&send,     (void*)&E};
  return launch(k, (unsigned)std::min(need, cap), args, st);
}

size_t cgtp_csr_workspace_bytes(int64_t E, int64_t V) {
  size_t bytes = 0;
  if (E < 0 || V < 0 || cgtp::csr_workspace_bytes(E, V, &bytes) != hipSuccess) return 0;
  return bytes;
}

cgtp_status cgtp_csr_from_coo_async(const int64_t* recv, const int64_t* send, int64_t E, int64_t V, int64_t* row_ptr,
                                    int64_t* col, int64_t* perm, int64_t* t_row_ptr, int64_t* t_perm, void* workspace,
                                    size_t workspace_bytes, int32_t* bad_flag, void* hip_stream) {
  if (E < 0 || V < 0) return fail(CGTP_EINVAL, "negative size");
  if (!row_ptr) return fail(CGTP_EINVAL, "NULL output pointer");
  if ((t_row_ptr == nullptr) != (t_perm == nullptr) && E > 0) return fail(CGTP_EINVAL, "t_row_ptr and t_perm must both be given or both be NULL");
  if (E > 0 && (!recv || !send || !col || !perm)) return fail(CGTP_EINVAL, "NULL pointer");
  if (E > 0 && V == 0) return fail(CGTP_EINVAL, "edges without nodes");
  if (E > 0) {
    const size_t need = cgtp_csr_workspace_bytes(E, V);
    if (!workspace || workspace_bytes < need)
      return fail(CGTP_EINVAL, "workspace too small: " + std::to_string(need) + " bytes needed (cgtp_csr_workspace_bytes)");
  }
  hipError_t e = cgtp::csr_from_coo_async(recv, send, E, V, row_ptr, col, perm, t_row_ptr, t_perm, workspace, workspace_bytes,
                                          (int*)bad_flag, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(CGTP_ERUNTIME, std::string("csr_from_coo: ") + hipGetErrorString(e));
  return CGTP_OK;
}

cgtp_status cgtp_csr_from_coo(const int64_t* recv, const int64_t* send, int64_t E, int64_t V, int64_t* row_ptr,
                              int64_t* col, int64_t* perm, int64_t* t_row_ptr, int64_t* t_perm, void* hip_stream) {
  if (E < 0 || V < 0) return fail(CGTP_EINVAL, "negative size");
  if (!row_ptr || !t_row_ptr) return fail(CGTP_EINVAL, "NULL output pointer");
  if (E > 0 && (!recv || !send || !col || !perm || !t_perm)) return fail(CGTP_EINVAL, "NULL pointer");
  if (E > 0 && V == 0) return fail(CGTP_EINVAL, "edges without nodes");
  // scratch owned by the library, one buffer per (device, stream), grown on demand and kept until the process ends:
  // a call allocates only when a larger graph than any before arrives on that stream
  struct Scratch {
    void* p = nullptr;
    size_t bytes = 0;
  };
  static std::mutex mu;
  static std::map<std::pair<int, void*>, Scratch> pool;
  int device = 0;
  HIP_TRY(hipGetDevice(&device));
  const size_t need = cgtp_csr_workspace_bytes(E, V) + 256;   // + the range-check flag
  void* ws = nullptr;
  {
    std::lock_guard<std::mutex> lock(mu);
    Scratch& sc = pool[{device, hip_stream}];
    if (sc.bytes < need) {
      if (sc.p) {
        HIP_TRY(hipStreamSynchronize((hipStream_t)hip_stream));
        HIP_TRY(hipFree(sc.p));
        sc = Scratch();
      }
      if (hipMalloc(&sc.p, need) != hipSuccess) {
        sc = Scratch();
        return fail(CGTP_ENOMEM, "scratch allocation of " + std::to_string(need) + " bytes failed");
      }
      sc.bytes = need;
    }
    ws = sc.p;
  }
  int32_t* flag = (int32_t*)ws;
  cgtp_status s = cgtp_csr_from_coo_async(recv, send, E, V, row_ptr, col, perm, t_row_ptr, t_perm, (char*)ws + 256, need - 256,
                                          flag, hip_stream);
  if (s != CGTP_OK) return s;
  // the one synchronisation of this call: the range check is part of its return value
  int bad = 0;
  HIP_TRY(hipMemcpyAsync(&bad, flag, sizeof(int), hipMemcpyDeviceToHost, (hipStream_t)hip_stream));
  HIP_TRY(hipStreamSynchronize((hipStream_t)hip_stream));
  if (bad) return fail(CGTP_EINVAL, "edge index outside [0, V)");
  return CGTP_OK;
}

}  // extern "C"
