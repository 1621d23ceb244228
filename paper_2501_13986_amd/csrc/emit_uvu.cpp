// HIP source generation for "uvu" problems (the paper's sub-kernel B: every x channel u is
// contracted with the shared y segment through one CG block and scaled by its own weight).
//
// What is kept from the paper (Sec. 3, Alg. 1-4): one wavefront owns one sample / edge and
// reads it with contiguous accesses; the CG nonzeros are literals and the contraction is a
// straight unrolled stream; operands persist in registers across the paths that reuse them;
// the backward pass produces all three gradients in one sweep; the convolution walks
// row-sorted edges with a running accumulator that is written once per row, and rows split
// between wavefronts are merged from a side buffer by a second small kernel.
//
// What is different on gfx950: 512 VGPRs per lane hold x, W, z of a whole sample, so there
// is no shared-memory staging and no multi-phase schedule; a lane owns `cpl` adjacent channels
// so that its words are contiguous in memory (wide loads, no transpose); the products
// v * y[j] are formed once per sample and shared by all channels of the lane, and the weight
// is folded into the shorter of x / z', so the inner stream is one FMA per nonzero per channel.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <map>
#include <regex>
#include <set>
#include <sstream>

#include "plan.hpp"

namespace cgtp {
namespace {

using i64 = long long;

std::string lit(double v) {
  char b[48];
  std::snprintf(b, sizeof b, "(T)(%.17e)", v);
  return b;
}

struct Em {
  std::ostringstream o;
  const Plan& P;
  LaneMap M;
  bool f64;
  int tcount = 0;
  Schedule S;
  Em(const Plan& p, const LaneMap& m, const Schedule& sc = Schedule()) : P(p), M(m), f64(p.dtype == CGTP_F64), S(sc) {}
  // a code-generation choice: the environment (tuning) wins over the plan's schedule, which wins over the default
  static int knob(const char* env, int sched, int dflt) {
    int v = env_int(env, -1);
    return v >= 0 ? v : (sched >= 0 ? sched : dflt);
  }
  // phase selection (backward): when not empty, only these x segments and the paths reading them are emitted
  std::set<int> xsel, zsel;  // zsel: the same for phases over output segments (forward convolution)
  bool store_unused = true;  // zero-fill the segments no path touches (first phase only)
  bool sel(const PathInfo& q) const {
    return (xsel.empty() || xsel.count(q.ix) > 0) && (zsel.empty() || zsel.count(q.iz) > 0);
  }

  void preamble() {
    o << "typedef " << (f64 ? "double" : "float") << " T;\n";
    o << "typedef T V2 __attribute__((ext_vector_type(2), aligned(" << (f64 ? 8 : 4) << ")));\n";
    if (!f64) o << "typedef T V4 __attribute__((ext_vector_type(4), aligned(4)));\n";
    o << "#define FMA(a, b, c) " << (f64 ? "__builtin_fma" : "__builtin_fmaf") << "((a), (b), (c))\n";
    o << "typedef long long i64;\n";
  }

  // Device function: the row that holds CSR position e, i.e. the largest r in [0, V) with ptr[r] <= e.  A 64-way search:
  // the lanes of the wave probe 64 evenly spaced entries per round (three dependent loads for 20 000 rows where a
  // binary search needs fifteen); every value that steers the loop comes from a ballot, so the loop is wave-uniform.
  // All 64 lanes must be active at the call.
  void emit_row_of() {
    o << "static __device__ __forceinline__ i64 row_of(const i64* __restrict__ ptr, i64 V, i64 e) {\n"
         "  const int l_ = threadIdx.x & 63;\n"
         "  i64 lo = 0, hi = V;\n"
         "  while (hi - lo > 1) {\n"
         "    const i64 step = (hi - lo + 63) >> 6;\n"
         "    const i64 p = lo + step * l_;\n"
         "    const bool in = p < hi;\n"
         "    const i64 v = ptr[in ? p : lo];\n"
         "    const int c = __builtin_popcountll(__builtin_amdgcn_ballot_w64(in && v <= e));\n"
         "    const i64 nhi = lo + step * c;\n"
         "    lo += step * (c - 1);\n"
         "    hi = nhi < hi ? nhi : hi;\n"
         "  }\n"
         "  return lo;\n"
         "}\n";
  }

  // names[0..n) <- n contiguous words at `ptr` (an expression of type const T*)
  void load_chunk(const std::string& ptr, const std::vector<std::string>& names, const char* ind) {
    size_t n = names.size(), at = 0;
    static const char* comp[4] = {"x", "y", "z", "w"};
    while (at < n) {
      size_t w = (!f64 && n - at >= 4) ? 4 : (n - at >= 2 ? 2 : 1);
      if (w == 1) {
        if (nt_loads || (nt_all & 1))
          o << ind << names[at] << " = __builtin_nontemporal_load(" << ptr << " + " << at << ");\n";
        else
          o << ind << names[at] << " = " << ptr << "[" << at << "];\n";
      } else {
        if (nt_loads || (nt_all & 1))
          o << ind << "{ const V" << w << " q_ = __builtin_nontemporal_load((const V" << w << "*)(" << ptr << " + " << at << "));";
        else
        o << ind << "{ const V" << w << " q_ = *(const V" << w << "*)(" << ptr << " + " << at << ");";
        for (size_t c = 0; c < w; ++c) o << " " << names[at + c] << " = q_." << comp[c] << ";";
        o << " }\n";
      }
      at += w;
    }
  }
  // use-once streams (per-edge weights, y, gW, gy) marked non-temporal so that they do not push the gathered
  // node rows out of the L2
  bool nt_loads = false, nt_stores = false;
  int nt_all = 0;             // batched kernels (every operand is used once): 1 = non-temporal loads, 2 = stores, 3 = both
  bool stream_nt = false;     // the kernel wants its per-edge streams non-temporal (conv kernels)
  bool emit_lz = true;            // double backward: also form dL/dgz (the convolution's sender walk leaves it out)
  bool accumulate_store = false;  // add to what memory holds (plain read-modify-write by the owning lane)
  std::set<int> written_z;        // double backward with phases: dL/dgz segments an earlier phase has stored
  bool atomic_store = false;  // accumulate with hardware float atomics instead of storing (unsorted-edge convolution)
  std::string atomic_mask;    // branch-free mode: condition under which the lane's own value (not zero) is added
  std::string atomic_live;    // ... its part that does not depend on the segment (the lane has a sample of its own)
  void store_chunk(const std::string& ptr, const std::vector<std::string>& names, const char* ind) {
    if (atomic_store) {
      for (size_t t = 0; t < names.size(); ++t) {
        const std::string v = atomic_mask.empty() ? names[t] : "(" + atomic_mask + " ? " + names[t] + " : (T)0)";
        o << ind << "__hip_atomic_fetch_add(" << ptr << " + " << t << ", " << v << ", __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);\n";
      }
      return;
    }
    size_t n = names.size(), at = 0;
    static const char* comp[4] = {"x", "y", "z", "w"};
    if (accumulate_store) {   // read-modify-write of the lane's own words
      while (at < n) {
        size_t w = (!f64 && n - at >= 4) ? 4 : (n - at >= 2 ? 2 : 1);
        if (w == 1) {
          o << ind << ptr << "[" << at << "] += " << names[at] << ";\n";
        } else {
          o << ind << "{ V" << w << " q_ = *(const V" << w << "*)(" << ptr << " + " << at << ");";
          for (size_t c = 0; c < w; ++c) o << " q_." << comp[c] << " += " << names[at + c] << ";";
          o << " *(V" << w << "*)(" << ptr << " + " << at << ") = q_; }\n";
        }
        at += w;
      }
      return;
    }
    while (at < n) {
      size_t w = (!f64 && n - at >= 4) ? 4 : (n - at >= 2 ? 2 : 1);
      if (w == 1) {
        if (nt_stores || (nt_all & 2))
          o << ind << "__builtin_nontemporal_store(" << names[at] << ", " << ptr << " + " << at << ");\n";
        else
          o << ind << ptr << "[" << at << "] = " << names[at] << ";\n";
      } else {
        o << ind << "{ V" << w << " q_;";
        for (size_t c = 0; c < w; ++c) o << " q_." << comp[c] << " = " << names[at + c] << ";";
        if (nt_stores || (nt_all & 2))
          o << " __builtin_nontemporal_store(q_, (V" << w << "*)(" << ptr << " + " << at << ")); }\n";
        else
          o << " *(V" << w << "*)(" << ptr << " + " << at << ") = q_; }\n";
      }
      at += w;
    }
  }

  // One irreps segment of a row (multiplicity mul, degree l, first word `off`) <-> the lane's registers names[e*(2l+1)+i]
  // (e: the lane's channel slot, i: component).  MUL_IR layout: the lane's cpl*(2l+1) words are contiguous.  IR_MUL
  // layout ((m+l)*mul + u, paper Sec. 4 "data layout"): for every component the lane's cpl words are contiguous and the
  // wave's words of that component are one contiguous run.
  void load_seg(const std::string& base, int64_t off, int mul, int l, const std::vector<std::string>& names, const char* ind) {
    const int n = 2 * l + 1;
    const std::string u0 = uch(mul);
    if (!P.ir_mul) {
      o << ind << "const T* p_ = " << base << " + " << off << " + " << u0 << " * " << n << ";\n";
      load_chunk("p_", names, ind);
      return;
    }
    for (int i = 0; i < n; ++i) {
      std::vector<std::string> part;
      for (int e = 0; e < M.cpl; ++e) part.push_back(names[(size_t)e * n + i]);
      o << ind << "{ const T* p_ = " << base << " + " << (off + (int64_t)i * mul) << " + " << u0 << ";\n";
      load_chunk("p_", part, (std::string(ind) + "  ").c_str());
      o << ind << "}\n";
    }
  }
  void store_seg(const std::string& base, int64_t off, int mul, int l, const std::vector<std::string>& names, const char* ind) {
    const int n = 2 * l + 1;
    const std::string u0 = uch(mul);
    if (!P.ir_mul) {
      o << ind << "{ T* p_ = " << base << " + " << off << " + " << u0 << " * " << n << ";\n";
      store_chunk("p_", names, (std::string(ind) + "  ").c_str());
      o << ind << "}\n";
      return;
    }
    for (int i = 0; i < n; ++i) {
      std::vector<std::string> part;
      for (int e = 0; e < M.cpl; ++e) part.push_back(names[(size_t)e * n + i]);
      o << ind << "{ T* p_ = " << base << " + " << (off + (int64_t)i * mul) << " + " << u0 << ";\n";
      store_chunk("p_", part, (std::string(ind) + "  ").c_str());
      o << ind << "}\n";
    }
  }

  // ---- naming -------------------------------------------------------------------------
  static std::string X(int s, int e, int i) { return "x" + std::to_string(s) + "_" + std::to_string(e) + "_" + std::to_string(i); }
  static std::string GX(int s, int e, int i) { return "gx" + std::to_string(s) + "_" + std::to_string(e) + "_" + std::to_string(i); }
  static std::string Z(int s, int e, int k) { return "z" + std::to_string(s) + "_" + std::to_string(e) + "_" + std::to_string(k); }
  static std::string Wn(int p, int e) { return "w" + std::to_string(p) + "_" + std::to_string(e); }
  static std::string Y(int j) { return "y" + std::to_string(j); }
  static std::string GY(int j) { return "gy" + std::to_string(j); }
  static std::string ZA(int s, int e, int k) { return "a" + Z(s, e, k); }    // compensated row sums: running sum ...
  static std::string ZC(int s, int e, int k) { return "c" + Z(s, e, k); }    // ... and its compensation term
  static std::string GA(int s, int e, int i) { return "a" + GX(s, e, i); }
  static std::string GC(int s, int e, int i) { return "c" + GX(s, e, i); }
  static std::string AX(int s, int e, int i) { return "a" + X(s, e, i); }    // dL/da row (double backward)
  static std::string LZ(int s, int e, int k) { return "l" + Z(s, e, k); }    // dL/dgz accumulators

  std::set<int> used_x() const {
    std::set<int> s;
    for (auto& q : P.paths)
      if (sel(q)) s.insert(q.ix);
    return s;
  }
  std::set<int> all_used_x() const {
    std::set<int> s;
    for (auto& q : P.paths) s.insert(q.ix);
    return s;
  }
  std::set<int> used_z() const {
    std::set<int> s;
    for (auto& q : P.paths)
      if (sel(q)) s.insert(q.iz);
    return s;
  }
  std::set<int> all_used_z() const {
    std::set<int> s;
    for (auto& q : P.paths) s.insert(q.iz);
    return s;
  }
  std::set<int> used_y_words() const {
    std::set<int> s;
    for (auto& q : P.paths)
      for (auto& n : q.nz) s.insert((int)P.offy[q.iy] + n.j);
    return s;
  }
  int full() const { return M.G * M.cpl * M.npass; }
  // loads/stores need a channel guard when the lane map covers more channels than the segment
  // has, or when a wave holds several samples (lanes of a missing last sample are parked)
  bool force_guard = false;
  int sched_barrier = env_int("CGTP_SCHED_BARRIER", 1);  // 0 none, 1 per output segment, 2 per path (backward)
  bool guarded(int mul) const { return force_guard || mul != full(); }
  // Branch-free mode (every kernel except the atomic variants and the convolution kernels whose wave holds several
  // edge-range workers).  A lane whose channel index lies beyond a segment's multiplicity is not switched off: it
  // works as a duplicate of the segment's last channel slot - it reads that slot's words, computes the same values and
  // stores them to the same addresses - and only its contribution to the sums over channels (gy) is replaced by
  // zero.  Lanes of a wave that have no sample of their own (several samples per wave, ragged end of the batch)
  // duplicate the last sample in the same way.  The generated code then has no lane-divergent region at all, only
  // wave-uniform branches: the compiler has been seen to place register-allocation copies of values that are live
  // in all lanes inside lane-conditional regions (where only the active lanes execute them), which ended in a wild
  // address on the GPU.
  bool dup = false;
  std::string uch(int mul) const {   // the lane's (clamped) first channel in a segment of multiplicity `mul`
    if (!dup || !guarded(mul)) return "u0";
    return "(u0 < " + std::to_string(mul) + " ? u0 : " + std::to_string(mul - M.cpl) + ")";
  }
  // opens the block around an access to a segment of multiplicity `mul`; closed with "}"
  std::string open_guard(int mul) const {
    if (!guarded(mul)) return "{\n";
    if (!dup) return "if (u0 < " + std::to_string(mul) + ") {\n";
    // passes that lie entirely beyond the multiplicity are skipped by a wave-uniform branch
    if (M.npass > 1) return "if (pass * " + std::to_string(M.G * M.cpl) + " < " + std::to_string(mul) + ") {\n";
    return "{\n";
  }
  std::string lane_ok(int mul) const { return "(u0 < " + std::to_string(mul) + ")"; }

  std::vector<std::string> seg_names(std::string (*f)(int, int, int), int s, int l) const {
    std::vector<std::string> v;
    for (int e = 0; e < M.cpl; ++e)
      for (int i = 0; i < 2 * l + 1; ++i) v.push_back(f(s, e, i));
    return v;
  }

  void declare(const std::vector<std::string>& v, const char* ind, bool zero) {
    o << ind << "T";
    for (size_t t = 0; t < v.size(); ++t) o << (t ? ", " : " ") << v[t] << (zero ? " = (T)0" : "");
    o << ";\n";
  }

  // x rows: declares (unless `decl` is false) and loads every used x segment from row pointer `xb`
  // which half of "declare + load" the operand loaders emit (the pipelined kernels declare the
  // operand sets once and load them in several places)
  bool do_decl = true, do_load = true;
  bool gz_in_path_code = false;  // the gz segments are declared and loaded by the path code even if W and y are not
  void load_x(const char* xb, const char* ind, bool decl = true, bool load = true, std::string (*nm)(int, int, int) = &Em::X) {
    decl = decl && do_decl;
    load = load && do_load;
    for (int s : used_x()) {
      const Irrep& ir = P.irx[s];
      auto names = seg_names(nm, s, ir.l);
      bool g = guarded(ir.mul);
      if (decl) declare(names, ind, g || !load);
      if (!load) continue;
      o << ind << open_guard(ir.mul);
      load_seg(xb, P.offx[s], ir.mul, ir.l, names, (std::string(ind) + "  ").c_str());
      o << ind << "}\n";
    }
  }
  // weights of path p (cpl adjacent words), loaded where the path starts so that few are live at once
  void load_w_path(const char* wb, size_t p, const char* ind, const char* pre = "") {
    const PathInfo& q = P.paths[p];
    std::vector<std::string> names;
    for (int e = 0; e < M.cpl; ++e) names.push_back(pre + Wn((int)p, e));
    bool g = guarded(q.mul_x);
    if (do_decl) declare(names, ind, g || !do_load);
    if (!do_load) return;
    std::string ptr = std::string(wb) + " + " + std::to_string(q.w_off) + " + " + uch(q.mul_x);
    o << ind << open_guard(q.mul_x);
    o << ind << "  const T* p_ = " << ptr << ";\n";
    nt_loads = stream_nt;
    load_chunk("p_", names, (std::string(ind) + "  ").c_str());
    nt_loads = false;
    o << ind << "}\n";
  }
  // y is the same for all lanes of a sample.  It is nevertheless loaded with vector loads (through
  // `vz`, a per-lane zero the compiler cannot see through) so that it lives in VGPRs: with y in
  // SGPRs every product y[j] * literal needs its literal in a VGPR (one constant-bus operand per
  // VALU instruction on this ISA), and those loop-invariant literals then occupy dozens of VGPRs.
  void load_y(const char* yb, const char* ind, const char* pre = "") {
    std::set<int> used = used_y_words();
    if (used.empty()) return;
    int lo = *used.begin(), hi = *used.rbegin();
    std::vector<std::string> names;
    for (int j = lo; j <= hi; ++j) names.push_back(pre + Y(j));
    if (do_decl) declare(names, ind, !do_load);
    if (!do_load) return;
    o << ind << "{ const T* p_ = " << yb << " + vz + " << lo << ";\n";
    nt_loads = stream_nt;
    load_chunk("p_", names, (std::string(ind) + "  ").c_str());
    nt_loads = false;
    o << ind << "}\n";
  }

  // The products v * y[j] of different paths often coincide; the compiler then merges them and keeps the
  // merged value alive from its first to its last use, which for a plan with many paths is hundreds of
  // registers.  Claiming (with an empty asm) that the y words of a path change where the path starts
  // keeps every product local to its path.
  void fresh_y(const PathInfo& q, const char* ind, const char* pre = "") {
    std::set<int> js;
    for (auto& n : q.nz) js.insert((int)P.offy[q.iy] + n.j);
    std::vector<std::string> v;
    for (int j : js) v.push_back(pre + Y(j));
    pin(v, ind);
  }
  // t-products of one path: distinct (|alpha*v|, j) -> variable.  Returns map nz index -> (name, negative?)
  struct TRef {
    std::string name;
    bool neg;
  };
  std::vector<TRef> emit_tprods(const PathInfo& q, const char* ind, const char* pre = "") {
    std::map<std::pair<long long, int>, std::string> seen;
    std::vector<TRef> refs;
    for (auto& n : q.nz) {
      double c = n.v * q.coeff;
      double a = std::fabs(c);
      long long key = std::llround(a * 1e13);
      auto it = seen.find({key, n.j});
      if (it == seen.end()) {
        std::string name;
        if (std::fabs(a - 1.0) < 1e-15) {
          name = pre + Y((int)P.offy[q.iy] + n.j);  // coefficient 1: the y word itself
        } else {
          name = "t" + std::to_string(tcount++);
          o << ind << "const T " << name << " = " << pre << Y((int)P.offy[q.iy] + n.j) << " * " << lit(a) << ";\n";
        }
        it = seen.insert({{key, n.j}, name}).first;
      }
      refs.push_back({it->second, c < 0});
    }
    return refs;
  }

  // z accumulators += TP contribution of every path, for the sample whose x/w/y are loaded
  void forward_paths(const char* wb, const char* ind) {
    // All weight loads of the sample are issued before the first path: a wave then has its whole
    // row in flight at once, which measured faster than loading per path at higher occupancy.
    // wb == nullptr: the weights are already in registers (pipelined kernels).
    const bool upfront = wb == nullptr || knob("CGTP_W_UPFRONT_FWD", S.w_upfront, 1) != 0;
    if (upfront && wb)
      for (size_t p = 0; p < P.paths.size(); ++p)
        if (sel(P.paths[p])) load_w_path(wb, p, ind);
    for (size_t p = 0; p < P.paths.size(); ++p) {
      const PathInfo& q = P.paths[p];
      if (!sel(q)) continue;
      o << ind << "{ // path " << p << ": l=(" << q.l1 << "," << q.l2 << "," << q.l3 << ") nnz=" << q.nz.size() << "\n";
      std::string in2 = std::string(ind) + "  ";
      if (!upfront) load_w_path(wb, p, in2.c_str());
      if (knob("CGTP_FRESH_Y", S.fresh_y, 0)) fresh_y(q, in2.c_str());
      auto tr = emit_tprods(q, in2.c_str());
      const int n1 = 2 * q.l1 + 1, n3 = 2 * q.l3 + 1;
      if (n1 <= n3) {
        // fold the weight into x: a[i] = w * x[i]; z[k] += (+-t) * a[i]
        for (int e = 0; e < M.cpl; ++e)
          for (int i = 0; i < n1; ++i)
            o << in2 << "const T a" << e << "_" << i << " = " << X(q.ix, e, i) << " * " << Wn((int)p, e) << ";\n";
        for (size_t n = 0; n < q.nz.size(); ++n)
          for (int e = 0; e < M.cpl; ++e) {
            std::string zz = Z(q.iz, e, q.nz[n].k);
            o << in2 << zz << " = FMA(" << (tr[n].neg ? "-" : "") << tr[n].name << ", a" << e << "_" << q.nz[n].i << ", " << zz << ");\n";
          }
      } else {
        // contract first, then scale: q[k] = sum (+-t) x[i]; z[k] += w * q[k]
        std::vector<bool> started((size_t)M.cpl * n3, false);
        for (size_t n = 0; n < q.nz.size(); ++n)
          for (int e = 0; e < M.cpl; ++e) {
            int k = q.nz[n].k;
            std::string qq = "q" + std::to_string(e) + "_" + std::to_string(k);
            std::string tt = std::string(tr[n].neg ? "-" : "") + tr[n].name;
            if (!started[(size_t)e * n3 + k]) {
              o << in2 << "T " << qq << " = " << tt << " * " << X(q.ix, e, q.nz[n].i) << ";\n";
              started[(size_t)e * n3 + k] = true;
            } else {
              o << in2 << qq << " = FMA(" << tt << ", " << X(q.ix, e, q.nz[n].i) << ", " << qq << ");\n";
            }
          }
        for (int e = 0; e < M.cpl; ++e)
          for (int k = 0; k < n3; ++k)
            if (started[(size_t)e * n3 + k]) {
              std::string zz = Z(q.iz, e, k);
              o << in2 << zz << " = FMA(" << Wn((int)p, e) << ", q" << e << "_" << k << ", " << zz << ");\n";
            }
      }
      o << ind << "}\n";
    }
  }

  void declare_z(const char* ind) {
    for (int s : used_z()) declare(seg_names(&Em::Z, s, P.irz[s].l), ind, true);
  }
  void zero_z(const char* ind) {
    for (int s : used_z())
      for (auto& n : seg_names(&Em::Z, s, P.irz[s].l)) o << ind << n << " = (T)0;\n";
  }
  // Compensated (Kahan) accumulation over the edges of a row (convolution kernels; the paper's Sec. 5
  // names it as the extension that keeps neighbourhood sums stable).  The per-edge result is formed in the
  // ordinary accumulator names, then added to a running sum `a*` with the compensation term `c*`:
  //   y = v - c;  t = a + y;  c = (t - a) - y;  a = t.
  // The kernels are compiled without contraction or reassociation, so the sequence survives as written.
  bool kahan = false;
  void kahan_add(const std::vector<std::string>& val, const std::vector<std::string>& acc, const std::vector<std::string>& cmp, const char* ind) {
    for (size_t t = 0; t < val.size(); ++t) {
      o << ind << "{ const T y_ = " << val[t] << " - " << cmp[t] << "; const T t_ = " << acc[t] << " + y_; " << cmp[t] << " = (t_ - " << acc[t]
        << ") - y_; " << acc[t] << " = t_; }\n";
    }
  }
  void declare_z_sums(const char* ind) {
    for (int s : used_z()) {
      declare(seg_names(&Em::ZA, s, P.irz[s].l), ind, true);
      declare(seg_names(&Em::ZC, s, P.irz[s].l), ind, true);
    }
  }
  void zero_z_sums(const char* ind) {
    for (int s : used_z()) {
      for (auto& n : seg_names(&Em::ZA, s, P.irz[s].l)) o << ind << n << " = (T)0;\n";
      for (auto& n : seg_names(&Em::ZC, s, P.irz[s].l)) o << ind << n << " = (T)0;\n";
    }
  }
  void kahan_add_z(const char* ind) {
    for (int s : used_z())
      kahan_add(seg_names(&Em::Z, s, P.irz[s].l), seg_names(&Em::ZA, s, P.irz[s].l), seg_names(&Em::ZC, s, P.irz[s].l), ind);
  }
  void declare_gx_sums(const char* ind) {
    for (int s : used_x()) {
      declare(seg_names(&Em::GA, s, P.irx[s].l), ind, true);
      declare(seg_names(&Em::GC, s, P.irx[s].l), ind, true);
    }
  }
  void zero_gx_sums(const char* ind) {
    for (int s : used_x()) {
      for (auto& n : seg_names(&Em::GA, s, P.irx[s].l)) o << ind << n << " = (T)0;\n";
      for (auto& n : seg_names(&Em::GC, s, P.irx[s].l)) o << ind << n << " = (T)0;\n";
    }
  }
  void kahan_add_gx(const char* ind) {
    for (int s : used_x())
      kahan_add(seg_names(&Em::GX, s, P.irx[s].l), seg_names(&Em::GA, s, P.irx[s].l), seg_names(&Em::GC, s, P.irx[s].l), ind);
  }
  // store the z accumulators of every used segment to row pointer `zb`; segments of z that no
  // path writes are zero-filled by lanes in the same pattern.
  void store_z(const char* zb, const char* ind) {
    for (size_t s = 0; s < P.irz.size(); ++s) store_z_seg(zb, s, ind, kahan ? &Em::ZA : &Em::Z);
  }
  void store_z_seg(const char* zb, size_t s, const char* ind, std::string (*nm)(int, int, int)) {
    {
      const Irrep& ir = P.irz[s];
      bool used = used_z().count((int)s) > 0;
      if (!used && (atomic_store || !store_unused || all_used_z().count((int)s) > 0)) return;
      std::vector<std::string> names = used ? seg_names(nm, (int)s, ir.l) : std::vector<std::string>((size_t)M.cpl * (2 * ir.l + 1), "(T)0");
      // unused segments: channels beyond `full()` per pass never occur for used ones (mul_z == mul_x <= full)
      store_row_seg(zb, P.offz[s], ir, used, names, ind);
    }
  }
  // one segment of an output row: the lane's accumulators (used) or zeros (a segment no path touches)
  void store_row_seg(const char* base, int64_t off, const Irrep& ir, bool used, const std::vector<std::string>& names, const char* ind) {
    const int mul = ir.mul;
    const std::string in2 = std::string(ind) + "  ";
    if (!used && dup) {
      // zero fill by all lanes of the sample's group, the same trip count in every lane; lanes past the end write
      // the segment's last word again
      o << ind << "if (pass == 0) for (int c_ = 0; c_ < " << ir.dim() << "; c_ += " << M.G << ") { int i_ = c_ + g_; i_ = i_ < " << ir.dim()
        << " ? i_ : " << ir.dim() - 1 << "; " << base << "[" << off << " + i_] = (T)0; }\n";
      return;
    }
    if (!used && mul > full()) {
      // more channels than the lane map covers: plain strided zero fill
      o << ind << "for (int c_ = g_; c_ < " << ir.dim() << "; c_ += " << M.G << ") if (pass == 0) " << base << "[" << off << " + c_] = (T)0;\n";
      return;
    }
    o << ind << open_guard(mul);
    if (atomic_store && dup) {
      atomic_mask = guarded(mul) ? lane_ok(mul) : std::string();
      if (!atomic_live.empty()) atomic_mask = atomic_mask.empty() ? atomic_live : atomic_mask + " && " + atomic_live;
    }
    store_seg(base, off, mul, ir.l, names, in2.c_str());
    atomic_mask.clear();
    o << ind << "}\n";
  }

  // ---- backward -----------------------------------------------------------------------
  void declare_gx(const char* ind) {
    for (int s : used_x()) declare(seg_names(&Em::GX, s, P.irx[s].l), ind, true);
  }
  void zero_gx(const char* ind) {
    for (int s : used_x())
      for (auto& n : seg_names(&Em::GX, s, P.irx[s].l)) o << ind << n << " = (T)0;\n";
  }
  void store_gx(const char* gb, const char* ind) {
    for (size_t s = 0; s < P.irx.size(); ++s) {
      const Irrep& ir = P.irx[s];
      bool used = used_x().count((int)s) > 0;
      if (!used && (atomic_store || !store_unused || all_used_x().count((int)s) > 0)) continue;
      std::vector<std::string> names = used ? seg_names(kahan ? &Em::GA : &Em::GX, (int)s, ir.l) : std::vector<std::string>((size_t)M.cpl * (2 * ir.l + 1), "(T)0");
      store_row_seg(gb, P.offx[s], ir, used, names, ind);
    }
  }
  // one segment of the gz row, named z*_*_* (the z accumulators are not needed in backward)
  void load_gz_seg(const char* gzb, int s, const char* ind) {
    const Irrep& ir = P.irz[s];
    auto names = seg_names(&Em::Z, s, ir.l);
    bool g = guarded(ir.mul);
    const bool decl = do_decl || gz_in_path_code, load = do_load || gz_in_path_code;
    if (decl) declare(names, ind, g || !load);
    if (!load) return;
    o << ind << open_guard(ir.mul);
    load_seg(gzb, P.offz[s], ir.mul, ir.l, names, (std::string(ind) + "  ").c_str());
    o << ind << "}\n";
  }

  // Per path (paper Alg. 3 with a diagonal weight tile), in one of two forms.  Two FMAs per nonzero and channel:
  //   r[i] += (+-t) gz[k];  gx[i] += w r[i];  gW = sum_i x[i] r[i]
  //   gy[j] += |alpha v| * sum_{same (j,|v|)} (+-) w x[i] gz[k]     (w folded into x or gz, scaled once per group)
  // or three, with shorter dependent chains:
  //   g'[k] = w * gz[k];  gx[i] += (+-t) g'[k];  q[k] += (+-t) x[i];  gW = sum_k gz[k] q[k]
  //   gy[j] += |alpha v| * sum_{same (j,|v|)} (+-) x[i] g'[k]
  // Paths are visited grouped by output segment so that only one segment of gz is live at a time.
  void backward_paths(const char* wb, const char* gzb, const char* gwb, const char* ind0) {
    std::vector<size_t> order;
    for (size_t t = 0; t < P.paths.size(); ++t)
      if (sel(P.paths[t])) order.push_back(t);
    std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b) { return P.paths[a].iz < P.paths[b].iz; });
    const std::string ind_s = std::string(ind0) + "  ";
    const char* ind = ind_s.c_str();
    // 1: all W at the top, 2: W and gz at the top (the conv kernel keeps its loads per segment)
    // convolution: fp64 issues all weight loads of the edge first (measured 3-4 % faster on the benchmark graphs: one
    // wave per SIMD there, and every load placed at its segment is an exposed round trip); fp32 runs three waves per
    // SIMD and is faster with the loads at their segments
    const int upfront = pin_accumulators ? knob("CGTP_UPFRONT_CONV_BWD", S.upfront, f64 ? 1 : 0) : knob("CGTP_UPFRONT_TP_BWD", S.upfront, upfront_tp_bwd_default);
    const bool pin_per_path = knob("CGTP_PIN_PER_PATH", S.pin, 0) >= 2;
    // two forms of the per-path arithmetic (below); measured: the two-FMA form is 5-10 % faster in the convolution
    // (both precisions) and equal in the fp32 batched kernel, the three-FMA form 10 % faster in the fp64 batched kernel
    const bool r_form = pin_accumulators ? env_int("CGTP_RFORM_CONV_BWD", 1) != 0 : env_int("CGTP_RFORM_TP_BWD", f64 ? 0 : 1) != 0;
    if (upfront >= 1)
      for (size_t p : order) load_w_path(wb, p, ind0);
    if (upfront >= 2)
      for (int s : used_z()) load_gz_seg(gzb, s, ind0);
    int open_iz = -1;
    for (size_t oi = 0; oi < order.size(); ++oi) {
      const size_t p = order[oi];
      const PathInfo& q = P.paths[p];
      if (q.iz != open_iz) {
        if (open_iz >= 0) {
          o << ind0 << "}\n";
          pin_gx(ind0);
        }
        // keep the instruction scheduler from hoisting every load of the edge to the top (which
        // would hold all of W and gz in registers at once): nothing moves across a group boundary
        if (open_iz >= 0 && sched_barrier) o << ind0 << "__builtin_amdgcn_sched_barrier(0);\n";
        o << ind0 << "{ // output segment " << q.iz << "\n";
        if (upfront < 2) load_gz_seg(gzb, q.iz, ind);
        if (upfront < 1)
          for (size_t oj = oi; oj < order.size() && P.paths[order[oj]].iz == q.iz; ++oj) load_w_path(wb, order[oj], ind);
        open_iz = q.iz;
      }
      o << ind << "{ // path " << p << ": l=(" << q.l1 << "," << q.l2 << "," << q.l3 << ") nnz=" << q.nz.size() << "\n";
      std::string in2 = std::string(ind) + "  ";
      if (sched_barrier > 1) o << in2 << "__builtin_amdgcn_sched_barrier(0);\n";
      if (knob("CGTP_FRESH_Y", S.fresh_y, 0)) fresh_y(q, in2.c_str());
      auto tr = emit_tprods(q, in2.c_str());
      const int n1 = 2 * q.l1 + 1, n3 = 2 * q.l3 + 1;
      std::vector<std::string> gw;
      if (r_form) {
        // r[i] = sum over the nonzeros with this i of (+-t) gz[k] serves both dL/dx[i] (times w) and dL/dW (times x[i])
        std::vector<bool> started((size_t)M.cpl * n1, false);
        for (size_t n = 0; n < q.nz.size(); ++n)
          for (int e = 0; e < M.cpl; ++e) {
            const Nz& z = q.nz[n];
            const std::string tt = std::string(tr[n].neg ? "-" : "") + tr[n].name;
            const std::string rr = "r" + std::to_string(e) + "_" + std::to_string(z.i);
            if (!started[(size_t)e * n1 + z.i]) {
              o << in2 << "T " << rr << " = " << tt << " * " << Z(q.iz, e, z.k) << ";\n";
              started[(size_t)e * n1 + z.i] = true;
            } else {
              o << in2 << rr << " = FMA(" << tt << ", " << Z(q.iz, e, z.k) << ", " << rr << ");\n";
            }
          }
        for (int e = 0; e < M.cpl; ++e) {
          const std::string name = "gw" + std::to_string(e);
          gw.push_back(name);
          bool first = true;
          for (int i = 0; i < n1; ++i) {
            if (!started[(size_t)e * n1 + i]) continue;
            const std::string rr = "r" + std::to_string(e) + "_" + std::to_string(i), gx = GX(q.ix, e, i);
            o << in2 << gx << " = FMA(" << Wn((int)p, e) << ", " << rr << ", " << gx << ");\n";
            if (first) {
              o << in2 << "T " << name << " = " << X(q.ix, e, i) << " * " << rr << ";\n";
              first = false;
            } else {
              o << in2 << name << " = FMA(" << X(q.ix, e, i) << ", " << rr << ", " << name << ");\n";
            }
          }
          if (first) o << in2 << "T " << name << " = (T)0;\n";
        }
        // gy groups: the weight goes onto whichever of x[i], gz[k] has fewer components
        const bool weight_on_x = n1 < n3;
        for (int e = 0; e < M.cpl; ++e) {
          if (weight_on_x) {
            for (int i = 0; i < n1; ++i)
              if (started[(size_t)e * n1 + i]) o << in2 << "const T xw" << e << "_" << i << " = " << X(q.ix, e, i) << " * " << Wn((int)p, e) << ";\n";
          } else {
            for (int k = 0; k < n3; ++k) o << in2 << "const T g" << e << "_" << k << " = " << Z(q.iz, e, k) << " * " << Wn((int)p, e) << ";\n";
          }
        }
        std::map<std::pair<int, long long>, std::vector<size_t>> groups;
        for (size_t n = 0; n < q.nz.size(); ++n)
          groups[{q.nz[n].j, std::llround(std::fabs(q.nz[n].v * q.coeff) * 1e13)}].push_back(n);
        int gi = 0;
        for (auto& kv : groups) {
          std::string s = "s" + std::to_string(gi++);
          bool first = true;
          for (size_t n : kv.second)
            for (int e = 0; e < M.cpl; ++e) {
              const Nz& z = q.nz[n];
              bool neg = z.v * q.coeff < 0;
              const std::string es = std::to_string(e);
              std::string xx = std::string(neg ? "-" : "") + (weight_on_x ? "xw" + es + "_" + std::to_string(z.i) : X(q.ix, e, z.i));
              std::string gg = weight_on_x ? Z(q.iz, e, z.k) : "g" + es + "_" + std::to_string(z.k);
              if (first) {
                o << in2 << "T " << s << " = " << xx << " * " << gg << ";\n";
                first = false;
              } else {
                o << in2 << s << " = FMA(" << xx << ", " << gg << ", " << s << ");\n";
              }
            }
          std::string gy = GY((int)P.offy[q.iy] + kv.first.first);
          double a = std::fabs(q.nz[kv.second[0]].v * q.coeff);
          // a lane that duplicates another channel must not add that channel to the sum over channels a second time
          const std::string sv = (dup && guarded(q.mul_x)) ? "(" + lane_ok(q.mul_x) + " ? " + s + " : (T)0)" : s;
          o << in2 << gy << " = FMA(" << sv << ", " << lit(a) << ", " << gy << ");\n";
        }
      } else {
        for (int e = 0; e < M.cpl; ++e)
          for (int k = 0; k < n3; ++k)
            o << in2 << "const T g" << e << "_" << k << " = " << Z(q.iz, e, k) << " * " << Wn((int)p, e) << ";\n";
        std::vector<bool> started((size_t)M.cpl * n3, false);
        for (size_t n = 0; n < q.nz.size(); ++n)
          for (int e = 0; e < M.cpl; ++e) {
            const Nz& z = q.nz[n];
            std::string tt = std::string(tr[n].neg ? "-" : "") + tr[n].name;
            std::string gx = GX(q.ix, e, z.i);
            o << in2 << gx << " = FMA(" << tt << ", g" << e << "_" << z.k << ", " << gx << ");\n";
            std::string qq = "q" + std::to_string(e) + "_" + std::to_string(z.k);
            if (!started[(size_t)e * n3 + z.k]) {
              o << in2 << "T " << qq << " = " << tt << " * " << X(q.ix, e, z.i) << ";\n";
              started[(size_t)e * n3 + z.k] = true;
            } else {
              o << in2 << qq << " = FMA(" << tt << ", " << X(q.ix, e, z.i) << ", " << qq << ");\n";
            }
          }
        // gy groups
        std::map<std::pair<int, long long>, std::vector<size_t>> groups;
        for (size_t n = 0; n < q.nz.size(); ++n)
          groups[{q.nz[n].j, std::llround(std::fabs(q.nz[n].v * q.coeff) * 1e13)}].push_back(n);
        int gi = 0;
        for (auto& kv : groups) {
          std::string s = "s" + std::to_string(gi++);
          bool first = true;
          for (size_t n : kv.second)
            for (int e = 0; e < M.cpl; ++e) {
              const Nz& z = q.nz[n];
              bool neg = z.v * q.coeff < 0;
              std::string xx = std::string(neg ? "-" : "") + X(q.ix, e, z.i);
              std::string gg = "g" + std::to_string(e) + "_" + std::to_string(z.k);
              if (first) {
                o << in2 << "T " << s << " = " << xx << " * " << gg << ";\n";
                first = false;
              } else {
                o << in2 << s << " = FMA(" << xx << ", " << gg << ", " << s << ");\n";
              }
            }
          std::string gy = GY((int)P.offy[q.iy] + kv.first.first);
          double a = std::fabs(q.nz[kv.second[0]].v * q.coeff);
          // a lane that duplicates another channel must not add that channel to the sum over channels a second time
          const std::string sv = (dup && guarded(q.mul_x)) ? "(" + lane_ok(q.mul_x) + " ? " + s + " : (T)0)" : s;
          o << in2 << gy << " = FMA(" << sv << ", " << lit(a) << ", " << gy << ");\n";
        }
        // gW
              for (int e = 0; e < M.cpl; ++e) {
          std::string name = "gw" + std::to_string(e);
          gw.push_back(name);
          bool first = true;
          for (int k = 0; k < n3; ++k) {
            if (!started[(size_t)e * n3 + k]) continue;
            if (first) {
              o << in2 << "T " << name << " = " << Z(q.iz, e, k) << " * q" << e << "_" << k << ";\n";
              first = false;
            } else {
              o << in2 << name << " = FMA(" << Z(q.iz, e, k) << ", q" << e << "_" << k << ", " << name << ");\n";
            }
          }
          if (first) o << in2 << "T " << name << " = (T)0;\n";
        }
      }
      o << in2 << open_guard(q.mul_x);
      o << in2 << "  T* p_ = " << gwb << " + " << q.w_off << " + " << uch(q.mul_x) << ";\n";
      nt_stores = stream_nt;
      store_chunk("p_", gw, (in2 + "  ").c_str());
      nt_stores = false;
      o << in2 << "}\n";
      o << ind << "}\n";
      if (pin_per_path) {
        // gx of the path's x segment and the gy words it touched are brought up to date here
        std::vector<std::string> acc = seg_names(&Em::GX, q.ix, q.l1);
        std::set<int> js;
        for (auto& z : q.nz) js.insert((int)P.offy[q.iy] + z.j);
        for (int j : js) acc.push_back(GY(j));
        pin(acc, ind);
      }
    }
    if (open_iz >= 0) {
      o << ind0 << "}\n";
      pin_gx(ind0);
    }
  }
  // Second-order pass (paper Sec. 3.4), all seven dispatches of the paper fused into one sweep.
  // With abar = dL/da, bbar = dL/db (words "by*"), cbar = dL/dC (words "cw*"), per path and nonzero
  // (i, j, k, v), t = |alpha v| y[j], tb = |alpha v| bbar[j], g1 = w gz, g2 = cbar gz,
  // r = w abar + cbar x, s = w x:
  //   dL/dx[i]  += (+-tb) g1[k] + (+-t) g2[k]                      (op1[1] + op2[1])
  //   dL/dgz[k] += (+-t) r[i] + (+-tb) s[i]                         (op3 + op6 + op7)
  //   Q[k]      += (+-t) abar[i] + (+-tb) x[i];  dL/dW = sum_k gz[k] Q[k]   (op4[3] + op5[3])
  //   dL/dy[j]  += |alpha v| sum (+-)(abar[i] g1[k] + x[i] g2[k])   (op1[2] + op2[2])
  // 8 FMAs per nonzero and channel instead of the 15 of the separate calls; every operand is read once.
  // The dL/dx accumulators use the gx names, dL/dy the gy names (shared store / reduction code).
  void double_backward_paths(const char* wb, const char* cwb, const char* gzb, const char* lwb, const char* lgzb, const char* ind0) {
    std::vector<size_t> order;
    for (size_t t = 0; t < P.paths.size(); ++t)
      if (sel(P.paths[t])) order.push_back(t);
    std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b) { return P.paths[a].iz < P.paths[b].iz; });
    const std::string ind_s = std::string(ind0) + "  ";
    const char* ind = ind_s.c_str();
    const int upfront = knob("CGTP_UPFRONT_DBL", S.upfront, 0);   // 1: W and cbar at the top, 2: gz as well (measured: 0 is best)
    if (upfront >= 1)
      for (size_t p : order) {
        load_w_path(wb, p, ind0);
        load_w_path(cwb, p, ind0, "c");
      }
    if (upfront >= 2)
      for (int s : used_z()) load_gz_seg(gzb, s, ind0);
    int open_iz = -1;
    auto close_group = [&]() {
      // with phases over the x segments, a dL/dgz segment receives contributions from several phases: the
      // first one to reach it stores, the later ones add to what is there (same lane, same addresses)
      if (emit_lz) {
        accumulate_store = written_z.count(open_iz) > 0;
        store_z_seg(lgzb, (size_t)open_iz, ind, &Em::LZ);
        accumulate_store = false;
        written_z.insert(open_iz);
      }
      o << ind0 << "}\n";
    };
    for (size_t oi = 0; oi < order.size(); ++oi) {
      const size_t p = order[oi];
      const PathInfo& q = P.paths[p];
      if (q.iz != open_iz) {
        if (open_iz >= 0) close_group();
        if (open_iz >= 0 && sched_barrier) o << ind0 << "__builtin_amdgcn_sched_barrier(0);\n";
        o << ind0 << "{ // output segment " << q.iz << "\n";
        if (upfront < 2) load_gz_seg(gzb, q.iz, ind);
        if (upfront < 1)
          for (size_t oj = oi; oj < order.size() && P.paths[order[oj]].iz == q.iz; ++oj) {
            load_w_path(wb, order[oj], ind);
            load_w_path(cwb, order[oj], ind, "c");
          }
        if (emit_lz) declare(seg_names(&Em::LZ, q.iz, P.irz[q.iz].l), ind, true);
        open_iz = q.iz;
      }
      o << ind << "{ // path " << p << ": l=(" << q.l1 << "," << q.l2 << "," << q.l3 << ") nnz=" << q.nz.size() << "\n";
      std::string in2 = std::string(ind) + "  ";
      if (sched_barrier > 1) o << in2 << "__builtin_amdgcn_sched_barrier(0);\n";
      if (knob("CGTP_FRESH_Y", S.fresh_y, 0)) {
        fresh_y(q, in2.c_str());
        fresh_y(q, in2.c_str(), "b");
      }
      auto tr = emit_tprods(q, in2.c_str());
      auto tb = emit_tprods(q, in2.c_str(), "b");
      const int n1 = 2 * q.l1 + 1, n3 = 2 * q.l3 + 1;
      std::set<int> used_i;
      for (auto& z : q.nz) used_i.insert(z.i);
      for (int e = 0; e < M.cpl; ++e) {
        const std::string w = Wn((int)p, e), c = "c" + Wn((int)p, e), es = std::to_string(e);
        for (int k = 0; k < n3; ++k) {
          o << in2 << "const T g1_" << es << "_" << k << " = " << Z(q.iz, e, k) << " * " << w << ";";
          o << " const T g2_" << es << "_" << k << " = " << Z(q.iz, e, k) << " * " << c << ";\n";
        }
        for (int i = 0; emit_lz && i < n1; ++i) {
          if (!used_i.count(i)) continue;
          o << in2 << "const T sx" << es << "_" << i << " = " << X(q.ix, e, i) << " * " << w << ";";
          o << " const T ra" << es << "_" << i << " = FMA(" << AX(q.ix, e, i) << ", " << w << ", " << X(q.ix, e, i) << " * " << c << ");\n";
        }
      }
      std::vector<bool> started((size_t)M.cpl * n3, false);
      for (size_t n = 0; n < q.nz.size(); ++n)
        for (int e = 0; e < M.cpl; ++e) {
          const Nz& z = q.nz[n];
          const std::string es = std::to_string(e), ks = std::to_string(z.k), is = std::to_string(z.i);
          const std::string t1 = std::string(tr[n].neg ? "-" : "") + tr[n].name, t2 = std::string(tb[n].neg ? "-" : "") + tb[n].name;
          const std::string gx = GX(q.ix, e, z.i), lz = LZ(q.iz, e, z.k), qq = "q" + es + "_" + ks;
          o << in2 << gx << " = FMA(" << t2 << ", g1_" << es << "_" << ks << ", FMA(" << t1 << ", g2_" << es << "_" << ks << ", " << gx << "));\n";
          if (emit_lz)
            o << in2 << lz << " = FMA(" << t1 << ", ra" << es << "_" << is << ", FMA(" << t2 << ", sx" << es << "_" << is << ", " << lz << "));\n";
          if (!started[(size_t)e * n3 + z.k]) {
            o << in2 << "T " << qq << " = FMA(" << t1 << ", " << AX(q.ix, e, z.i) << ", " << t2 << " * " << X(q.ix, e, z.i) << ");\n";
            started[(size_t)e * n3 + z.k] = true;
          } else {
            o << in2 << qq << " = FMA(" << t1 << ", " << AX(q.ix, e, z.i) << ", FMA(" << t2 << ", " << X(q.ix, e, z.i) << ", " << qq << "));\n";
          }
        }
      // dL/dy groups
      std::map<std::pair<int, long long>, std::vector<size_t>> groups;
      for (size_t n = 0; n < q.nz.size(); ++n)
        groups[{q.nz[n].j, std::llround(std::fabs(q.nz[n].v * q.coeff) * 1e13)}].push_back(n);
      int gi = 0;
      for (auto& kv : groups) {
        std::string sn = "sy" + std::to_string(gi++);
        bool first = true;
        for (size_t n : kv.second)
          for (int e = 0; e < M.cpl; ++e) {
            const Nz& z = q.nz[n];
            const std::string sg = z.v * q.coeff < 0 ? "-" : "";
            const std::string es = std::to_string(e), ks = std::to_string(z.k);
            const std::string ga = "g1_" + es + "_" + ks, gb = "g2_" + es + "_" + ks;
            if (first) {
              o << in2 << "T " << sn << " = FMA(" << sg << AX(q.ix, e, z.i) << ", " << ga << ", " << sg << X(q.ix, e, z.i) << " * " << gb << ");\n";
              first = false;
            } else {
              o << in2 << sn << " = FMA(" << sg << AX(q.ix, e, z.i) << ", " << ga << ", FMA(" << sg << X(q.ix, e, z.i) << ", " << gb << ", " << sn << "));\n";
            }
          }
        std::string gy = GY((int)P.offy[q.iy] + kv.first.first);
        double a = std::fabs(q.nz[kv.second[0]].v * q.coeff);
        const std::string sv = (dup && guarded(q.mul_x)) ? "(" + lane_ok(q.mul_x) + " ? " + sn + " : (T)0)" : sn;
        o << in2 << gy << " = FMA(" << sv << ", " << lit(a) << ", " << gy << ");\n";
      }
      // dL/dW
      std::vector<std::string> gw;
      for (int e = 0; e < M.cpl; ++e) {
        std::string name = "lw" + std::to_string(e);
        gw.push_back(name);
        bool first = true;
        for (int k = 0; k < n3; ++k) {
          if (!started[(size_t)e * n3 + k]) continue;
          if (first) {
            o << in2 << "T " << name << " = " << Z(q.iz, e, k) << " * q" << e << "_" << k << ";\n";
            first = false;
          } else {
            o << in2 << name << " = FMA(" << Z(q.iz, e, k) << ", q" << e << "_" << k << ", " << name << ");\n";
          }
        }
        if (first) o << in2 << "T " << name << " = (T)0;\n";
      }
      o << in2 << open_guard(q.mul_x);
      o << in2 << "  T* p_ = " << lwb << " + " << q.w_off << " + " << uch(q.mul_x) << ";\n";
      nt_stores = stream_nt;
      store_chunk("p_", gw, (in2 + "  ").c_str());
      nt_stores = false;
      o << in2 << "}\n";
      o << ind << "}\n";
      // the accumulators this path updated must be up to date here: without this the compiler postpones
      // the updates to the end of the sample and keeps every operand of every path alive until then
      const int pin_mode = knob("CGTP_PIN_DBL", S.pin, 1);
      if (pin_mode >= 1) {
        std::vector<std::string> acc = seg_names(&Em::GX, q.ix, q.l1);
        if (emit_lz)
          for (auto& n : seg_names(&Em::LZ, q.iz, q.l3)) acc.push_back(n);
        if (pin_mode >= 2) {
          std::set<int> js;
          for (auto& z : q.nz) js.insert((int)P.offy[q.iy] + z.j);
          for (int j : js) acc.push_back(GY(j));
        }
        pin(acc, ind);
      }
    }
    if (open_iz >= 0) close_group();
    // segments of dL/dgz that no path touches are zero
    for (size_t s = 0; emit_lz && s < P.irz.size(); ++s)
      if (!used_z().count((int)s)) store_z_seg(lgzb, s, ind0, &Em::LZ);
  }

  // dL/dgz part of the second-order pass in the accumulator names of the forward (z*), for the receiver walk of
  // the convolution: z[k] += (+-t) ra[i] + (+-tb) sx[i] with ra = w abar + cbar x, sx = w x (paper Sec. 3.4:
  // op3 + op6 + op7).
  void double_forward_paths(const char* wb, const char* cwb, const char* ind) {
    const bool upfront = knob("CGTP_W_UPFRONT_FWD", S.w_upfront, 1) != 0;
    if (upfront)
      for (size_t p = 0; p < P.paths.size(); ++p)
        if (sel(P.paths[p])) {
          load_w_path(wb, p, ind);
          load_w_path(cwb, p, ind, "c");
        }
    for (size_t p = 0; p < P.paths.size(); ++p) {
      const PathInfo& q = P.paths[p];
      if (!sel(q)) continue;
      o << ind << "{ // path " << p << ": l=(" << q.l1 << "," << q.l2 << "," << q.l3 << ") nnz=" << q.nz.size() << "\n";
      std::string in2 = std::string(ind) + "  ";
      if (!upfront) {
        load_w_path(wb, p, in2.c_str());
        load_w_path(cwb, p, in2.c_str(), "c");
      }
      if (knob("CGTP_FRESH_Y", S.fresh_y, 0)) {
        fresh_y(q, in2.c_str());
        fresh_y(q, in2.c_str(), "b");
      }
      auto tr = emit_tprods(q, in2.c_str());
      auto tb = emit_tprods(q, in2.c_str(), "b");
      std::set<int> used_i;
      for (auto& z : q.nz) used_i.insert(z.i);
      for (int e = 0; e < M.cpl; ++e) {
        const std::string w = Wn((int)p, e), c = "c" + Wn((int)p, e), es = std::to_string(e);
        for (int i : used_i) {
          o << in2 << "const T sx" << es << "_" << i << " = " << X(q.ix, e, i) << " * " << w << ";";
          o << " const T ra" << es << "_" << i << " = FMA(" << AX(q.ix, e, i) << ", " << w << ", " << X(q.ix, e, i) << " * " << c << ");\n";
        }
      }
      for (size_t n = 0; n < q.nz.size(); ++n)
        for (int e = 0; e < M.cpl; ++e) {
          const Nz& z = q.nz[n];
          const std::string es = std::to_string(e), is = std::to_string(z.i);
          const std::string t1 = std::string(tr[n].neg ? "-" : "") + tr[n].name, t2 = std::string(tb[n].neg ? "-" : "") + tb[n].name;
          const std::string zz = Z(q.iz, e, z.k);
          o << in2 << zz << " = FMA(" << t1 << ", ra" << es << "_" << is << ", FMA(" << t2 << ", sx" << es << "_" << is << ", " << zz << "));\n";
        }
      o << ind << "}\n";
      if (knob("CGTP_PIN_DBL", S.pin, 1) >= 1) pin(seg_names(&Em::Z, q.iz, q.l3), ind);
    }
  }

  // An empty asm that claims to read and write the gx accumulators: the compiler must have them
  // up to date here, so it cannot postpone their updates (and keep every operand alive) until the
  // end of the edge.
  int upfront_tp_bwd_default = 2;  // batched backward: every load of the sample in flight at once (measured best)
  bool pin_accumulators = false;  // set for the conv kernels, whose gx accumulators live across edges
  void pin(const std::vector<std::string>& all, const char* ind) {
    for (size_t at = 0; at < all.size(); at += 12) {
      o << ind << "asm volatile(\"\" :";
      for (size_t t = at; t < all.size() && t < at + 12; ++t) o << (t > at ? ", " : " ") << "\"+v\"(" << all[t] << ")";
      o << ");\n";
    }
  }
  void pin_gx(const char* ind) {
    if (!pin_accumulators) return;
    std::vector<std::string> all;
    for (int s : used_x())
      for (auto& n : seg_names(&Em::GX, s, P.irx[s].l)) all.push_back(n);
    for (size_t at = 0; at < all.size(); at += 12) {
      o << ind << "asm volatile(\"\" :";
      for (size_t t = at; t < all.size() && t < at + 12; ++t) o << (t > at ? ", " : " ") << "\"+v\"(" << all[t] << ")";
      o << ");\n";
    }
  }

  // Sum gy over the G lanes of a sample and store.  Values are halved across lanes at each
  // step while more than one is held (n + log cost instead of n log), then a plain butterfly.
  void reduce_store_gy(const char* gyb, const char* ind, const char* cond = "gy_store") {
    const int n = (int)P.dim_y();
    int N2 = 1;
    while (N2 < n) N2 <<= 1;
    std::vector<std::string> cur;
    std::set<int> used = used_y_words();
    for (int j = 0; j < N2; ++j) cur.push_back(j < n && used.count(j) ? GY(j) : std::string("(T)0"));
    int off = M.G / 2, step = 0;
    while (off >= 1 && cur.size() > 1) {
      size_t h = cur.size() / 2;
      std::vector<std::string> nxt;
      o << ind << "{ const bool hi_ = (lane & " << off << ") != 0;\n";
      for (size_t i = 0; i < h; ++i) {
        std::string nm = "r" + std::to_string(step) + "_" + std::to_string(i);
        o << ind << "  const T k_" << i << " = hi_ ? " << cur[h + i] << " : " << cur[i] << ";"
          << " const T s_" << i << " = hi_ ? " << cur[i] << " : " << cur[h + i] << ";\n";
        nxt.push_back(nm);
      }
      for (size_t i = 0; i < h; ++i) o << ind << "  " << nxt[i] << " = k_" << i << " + __shfl_xor(s_" << i << ", " << off << ", 64);\n";
      o << ind << "}\n";
      // declare the next-level names before the block: patch by emitting declarations up front
      cur = nxt;
      off >>= 1;
      ++step;
    }
    // the declarations of r*_* must precede the blocks: handled by the caller through gy_decls()
    for (; off >= 1; off >>= 1)
      for (auto& c : cur) o << ind << c << " += __shfl_xor(" << c << ", " << off << ", 64);\n";
    // store: lane holds cur.size() consecutive values starting at gy_idx (computed once per thread)
    // After the butterfly every lane of a residual group holds the same totals, so all of them may
    // store (same value to the same address): no branch is needed unless the value list was padded
    // or some lanes must stay silent.  Keeping the tail of the edge body free of control flow also
    // keeps the compiler from sinking the gx accumulation below it.
    const bool padded = N2 != n;
    if (dup) {
      // no lane condition at all: a lane whose value index lies in the padding stores gy[0] (fetched from the first
      // lane of its sample's group, which holds it) to word 0 once more
      if (padded) {
        o << ind << "{ const T g0_ = __shfl(" << cur[0] << ", lane & " << (64 - M.G) << ", 64);\n";
        for (size_t i = 0; i < cur.size(); ++i)
          o << ind << "  { const bool in_ = gy_idx + " << i << " < " << n << "; " << gyb << "[in_ ? gy_idx + " << i << " : 0] = in_ ? " << cur[i] << " : g0_; }\n";
        o << ind << "}\n";
      } else {
        for (size_t i = 0; i < cur.size(); ++i) o << ind << "  " << gyb << "[gy_idx + " << i << "] = " << cur[i] << ";\n";
      }
      return;
    }
    std::string c2 = std::string(cond) == "gy_store" ? std::string() : std::string(cond).substr(std::string("gy_store && ").size());
    if (!c2.empty()) o << ind << "if (" << c2 << ") {\n";
    for (size_t i = 0; i < cur.size(); ++i) {
      o << ind << "  ";
      if (padded) o << "if (gy_idx + " << i << " < " << n << ") ";
      o << gyb << "[gy_idx + " << i << "] = " << cur[i] << ";\n";
    }
    if (!c2.empty()) o << ind << "}\n";
  }
  // declarations for reduce_store_gy (must be emitted in an enclosing scope before it)
  void gy_reduce_decls(const char* ind) {
    const int n = (int)P.dim_y();
    int N2 = 1;
    while (N2 < n) N2 <<= 1;
    int off = M.G / 2, step = 0;
    size_t sz = (size_t)N2;
    while (off >= 1 && sz > 1) {
      sz /= 2;
      o << ind << "T";
      for (size_t i = 0; i < sz; ++i) o << (i ? ", " : " ") << "r" << step << "_" << i;
      o << ";\n";
      off >>= 1;
      ++step;
    }
  }
  // per-thread constants: first value index held after the halving steps, and whether this lane stores
  void gy_lane_consts(const char* ind) {
    const int n = (int)P.dim_y();
    int N2 = 1;
    while (N2 < n) N2 <<= 1;
    o << ind << "int gy_idx = 0; bool gy_store = true;\n";
    int off = M.G / 2;
    int sz = N2;
    while (off >= 1 && sz > 1) {
      sz /= 2;
      o << ind << "if (lane & " << off << ") gy_idx += " << sz << ";\n";
      off >>= 1;
    }
    if (off >= 1) o << ind << "gy_store = (lane & " << (2 * off - 1) << ") == 0;\n";
  }
  void declare_gy(const char* ind, bool zero) {
    std::vector<std::string> v;
    for (int j : used_y_words()) v.push_back(GY(j));
    declare(v, ind, zero);
  }
  void zero_gy(const char* ind) {
    for (int j : used_y_words()) o << ind << GY(j) << " = (T)0;\n";
  }
};

// Runs `f` with the emitter's stream redirected and returns what it wrote.
template <class F>
std::string capture(Em& E, F f) {
  std::string before = E.o.str();
  E.o.str("");
  f();
  std::string text = E.o.str();
  E.o.str(before);
  E.o.seekp(0, std::ios::end);
  return text;
}

// Second operand set of a double-buffered kernel: every x / w / y operand name gets a suffix.
std::string rename_operands(const std::string& text, const char* sfx, bool backward = false) {
  static const std::regex fwd("\\b(x[0-9]+_[0-9]+_[0-9]+|w[0-9]+_[0-9]+|y[0-9]+)\\b");
  static const std::regex bwd("\\b(z[0-9]+_[0-9]+_[0-9]+|w[0-9]+_[0-9]+|y[0-9]+)\\b");  // gz rows are named z*
  return std::regex_replace(text, backward ? bwd : fwd, std::string("$1") + sfx);
}

std::string occ_attr(const LaneMap& M, const Schedule& S = Schedule()) {
  const int occ = S.occ > 0 ? S.occ : M.occ;
  return occ > 0 ? "__attribute__((amdgpu_waves_per_eu(" + std::to_string(occ) + "))) " : std::string();
}

// Common head of every kernel: lane ids and the wave's global index.
// xcd_blocks: workgroups are handed to the 8 XCDs round-robin (workgroup b runs on XCD b % 8, each XCD with an L2
// of its own).  The convolution kernels renumber their workgroups so that the workgroups of one XCD own one
// contiguous eighth of the edge ranges: the node rows gathered by neighbouring ranges then meet in the same L2
// when node numbering has any locality.  The renumbering is a bijection of [0, gridDim.x) for every grid size.
void head(Em& E, int waves_per_wg, bool uniform_wave, bool xcd_blocks = false) {
  E.o << "  const int lane = threadIdx.x & 63;\n";
  E.o << "  int vz = 0; asm volatile(\"\" : \"+v\"(vz));\n";
  E.o << "  const int g_ = lane & " << (E.M.G - 1) << ";\n";
  std::string blk = "blockIdx.x";
  if (xcd_blocks && env_int("CGTP_XCD_BLOCKS", 1)) {
    E.o << "  const unsigned bq_ = gridDim.x >> 3, br_ = gridDim.x & 7u, bx_ = blockIdx.x & 7u;\n";
    E.o << "  const unsigned blk_ = bx_ * bq_ + (bx_ < br_ ? bx_ : br_) + (blockIdx.x >> 3);\n";
    blk = "blk_";
  }
  if (xcd_blocks && E.M.spw > 1)
    // convolution with a multiplicity that fills only part of a wave: every group of G lanes is a worker of its
    // own with its own edge range ("wave" then numbers workers and is not uniform across the wavefront)
    E.o << "  const i64 wave = ((i64)" << blk << " * " << waves_per_wg << " + (threadIdx.x >> 6)) * " << E.M.spw << " + (lane / " << E.M.G << ");\n";
  else if (uniform_wave)
    E.o << "  const i64 wave = (i64)" << blk << " * " << waves_per_wg << " + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));\n";
  else
    E.o << "  const i64 wave = (i64)" << blk << " * " << waves_per_wg << " + (threadIdx.x >> 6);\n";
  E.o << "  const i64 nwave = (i64)gridDim.x * " << waves_per_wg << ";\n";
}

}  // namespace

// Cuts a set of segments (in order) into at most `n` groups of similar total width sum(2l+1).
static std::vector<std::set<int>> cut_phases(const std::set<int>& used, const std::vector<Irrep>& ir, int n) {
  std::vector<int> segs(used.begin(), used.end());
  int total = 0;
  for (int s : segs) total += 2 * ir[s].l + 1;
  std::vector<std::set<int>> out;
  n = std::min<int>(n, (int)segs.size());
  if (n <= 1) return {used};
  int acc = 0;
  size_t at = 0;
  for (int g = 0; g < n; ++g) {
    std::set<int> grp;
    const int target = (total * (g + 1) + n - 1) / n;
    while (at < segs.size() && (grp.empty() || acc + (2 * ir[segs[at]].l + 1) <= target || g == n - 1)) {
      acc += 2 * ir[segs[at]].l + 1;
      grp.insert(segs[at++]);
    }
    if (!grp.empty()) out.push_back(grp);
  }
  return out;
}
static std::vector<std::set<int>> x_phases(const Em& E, int n) { return cut_phases(E.all_used_x(), E.P.irx, n); }
static std::vector<std::set<int>> z_phases(const Em& E, int n) { return cut_phases(E.all_used_z(), E.P.irz, n); }

// ---------------------------------------------------------------------------------------
// Batched forward (paper Alg. 1 + 2) and fused convolution forward (paper Alg. 4).
static void emit_uvu_forward_impl(const Plan& P, bool conv, Kernel& K, bool atomic) {
  const LaneMap& M = P.map[atomic ? CGTP_K_CONV_FWD_ATOMIC : conv ? CGTP_K_CONV_FWD : CGTP_K_TP_FWD];
  Em E(P, M, K.sched);
  K.wg = 256;
  const int wpw = K.wg / 64;
  K.name = atomic ? "cgtp_conv_fwd_atomic" : conv ? "cgtp_conv_fwd" : "cgtp_tp_fwd";
  E.preamble();
  if (conv && !atomic && M.spw == 1) E.emit_row_of();
  const int DX = (int)P.dim_x(), DY = (int)P.dim_y(), DZ = (int)P.dim_z();
  const i64 NW = P.n_w;
  auto& o = E.o;
  if (!conv) {
    o << "extern \"C\" __global__ void __launch_bounds__(" << K.wg << ") " << occ_attr(M) << K.name
      << "(const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, T* __restrict__ z, i64 B)\n{\n";
    head(E, wpw, true);   // the wave index is wave-uniform also when a wave holds several samples
    E.nt_all = env_int("CGTP_NT_TP", 0);
    E.dup = true;
    o << "  const int sub_ = lane / " << M.G << ";\n";
    o << "  for (i64 s0 = wave * " << M.spw << "; s0 < B; s0 += nwave * " << M.spw << ") {\n";
    // lanes without a sample of their own (ragged end of the batch) work on the last sample once more
    o << "    const i64 b = s0 + sub_ < B ? s0 + sub_ : B - 1;\n";
    o << "    {\n";
    o << "      const T* xb = x + b * " << DX << "; const T* yb = y + b * " << DY << "; const T* wb = W + b * " << NW
      << "; T* zb = z + b * " << DZ << ";\n";
    E.load_y("yb", "      ");
    if (M.npass > 1) o << "      #pragma unroll 1\n";
    o << "      for (int pass = 0; pass < " << M.npass << "; ++pass) {\n";
    o << "        const int u0 = (pass * " << M.G << " + g_) * " << M.cpl << ";\n";
    E.load_x("xb", "        ");
    E.declare_z("        ");
    E.forward_paths("wb", "        ");
    E.store_z("zb", "        ");
    o << "      }\n    }\n  }\n}\n";
  } else {
    // One wave owns the contiguous edge range [e0, e1) of the row-sorted edge list and keeps a
    // running accumulator per output row (paper Alg. 4).  A row that lies entirely inside the
    // range is written straight to z; the piece of a row that started in an earlier range goes
    // to part[wave][0], the piece of a row that continues into a later range to part[wave][1];
    // a second kernel adds the pieces of each split row in wave order.  Rows without edges are
    // zero-filled by the wave whose range they precede (or end).
    // The atomic variant (paper Sec. 3.5, second algorithm) takes the edges in any order: the
    // running accumulator is added to z[recv] with float atomics whenever the receiver changes
    // (at the latest at the end of the wave's range), so runs of edges with the same receiver
    // cost one atomic update; z is zero-filled by the host beforehand.
    if (atomic)
      o << "extern \"C\" __global__ void __launch_bounds__(" << K.wg << ") " << occ_attr(M) << K.name
        << "(const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, T* __restrict__ z,\n"
           "   const i64* __restrict__ recv, const i64* __restrict__ col, i64 E, i64 nchunk, const i64* __restrict__ eperm)\n{\n";
    else
    o << "extern \"C\" __global__ void __launch_bounds__(" << K.wg << ") " << occ_attr(M) << K.name
      << "(const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, T* __restrict__ z,\n"
         "   const i64* __restrict__ row_ptr, const i64* __restrict__ col, i64 V, i64 E, T* __restrict__ part, i64 nchunk,\n"
         "   const i64* __restrict__ eperm)\n{\n";
    head(E, wpw, true, true);
    E.stream_nt = env_int("CGTP_STREAM_NT", 1) != 0;  // measured: 3-5 % on the backward, neutral on the forward
    E.dup = M.spw == 1;
    o << "  if (wave >= nchunk) return;\n";
    o << "  const i64 e0 = (wave * E) / nchunk, e1 = ((wave + 1) * E) / nchunk;\n";
    if (atomic) {
      o << "  if (e1 <= e0) return;\n";
    } else {
    o << "  i64 rstart = 0;\n";
    if (M.spw == 1) o << "  if (wave > 0) rstart = row_of(row_ptr, V, e0);\n";
    else
    o << "  if (wave > 0) { i64 lo = 0, hi = V; while (hi - lo > 1) { const i64 mid = (lo + hi) >> 1; if (row_ptr[mid] <= e0) lo = mid; else hi = mid; } rstart = lo; }\n";
    }
    if (M.npass > 1) o << "  #pragma unroll 1\n";
    o << "  for (int pass = 0; pass < " << M.npass << "; ++pass) {\n";
    o << "    const int u0 = (pass * " << M.G << " + g_) * " << M.cpl << ";\n";
    // Phases (paper Alg. 4: the outer loop over the segments of the schedule): the output segments are cut into
    // groups; a phase walks the whole edge range with the accumulators of its own segments only and reads just the
    // x segments and weights its paths need.  y and the graph arrays are read again by every phase.
    const auto zph = z_phases(E, std::max(1, Em::knob("CGTP_PHASES_CONV_FWD", K.sched.phases, 1)));
    auto emit_phase = [&]() {
    E.kahan = P.kahan_conv;
    E.declare_z("    ");
    if (E.kahan) E.declare_z_sums("    ");
    if (atomic) {
      o << "    i64 cur = recv[e0];\n";
    } else {
    o << "    i64 r = rstart;\n";
    o << "    i64 rbeg = row_ptr[r], rend = row_ptr[r + 1];\n";
    }
    // flush macro as a lambda-like block emitted twice
    auto flush = [&](const char* ind) {
      std::string in2 = std::string(ind) + "  ";
      if (atomic) {
        o << ind << "{ T* dst_ = z + cur * " << DZ << ";\n";
        E.atomic_store = true;
        E.store_z("dst_", in2.c_str());
        E.atomic_store = false;
      } else {
      o << ind << "{ T* dst_ = (rbeg >= e0 && rend <= e1) ? z + r * " << DZ << " : part + (wave * 2 + (rbeg < e0 ? 0 : 1)) * " << DZ << ";\n";
      E.store_z("dst_", in2.c_str());
      }
      if (E.kahan) E.zero_z_sums(in2.c_str());
      else E.zero_z(in2.c_str());
      o << ind << "}\n";
    };
    auto row_change = [&](const char* ind) {
      std::string in2 = std::string(ind) + "  ";
      if (atomic) {
        o << ind << "{ const i64 rc_ = recv[e < e0 ? e0 : e];\n";
        o << ind << "  if (rc_ != cur) {\n";
        flush((in2 + "  ").c_str());
        o << ind << "    cur = rc_;\n" << ind << "  }\n" << ind << "}\n";
      } else {
        o << ind << "while (e >= rend && r + 1 < V) {\n";
        flush(in2.c_str());
        o << ind << "  ++r; rbeg = rend; rend = row_ptr[r + 1];\n";
        o << ind << "}\n";
      }
    };
    if (Em::knob("CGTP_PREFETCH_CONV_FWD", K.sched.prefetch, 1) != 0) {
      // Software pipeline over the edges of the range: two register sets of (x, W, y); the loads
      // of edge e+1 are issued before the arithmetic of edge e, so a wave always has one edge's
      // row in flight while it computes.  The loop body is written out twice (set A, set B)
      // instead of copying registers.
      E.do_load = false;
      std::string decl = capture(E, [&] {
        E.load_y("", "    ");
        E.load_x("", "    ");
        for (size_t p = 0; p < P.paths.size(); ++p)
          if (E.sel(P.paths[p])) E.load_w_path("", p, "    ");
      });
      E.do_load = true;
      E.do_decl = false;
      std::string loads = capture(E, [&] {
        o << "        const i64 c = col[en]; const i64 er_ = eperm ? eperm[en] : en;\n";
        o << "        const T* xb = x + c * " << DX << "; const T* yb = y + er_ * " << DY << "; const T* wb = W + er_ * " << NW << ";\n";
        E.load_y("yb", "        ");
        E.load_x("xb", "        ");
        for (size_t p = 0; p < P.paths.size(); ++p)
          if (E.sel(P.paths[p])) E.load_w_path("wb", p, "        ");
      });
      E.do_decl = true;
      std::string compute = capture(E, [&] {
        if (E.kahan) E.zero_z("      ");
        E.forward_paths(nullptr, "      ");
        if (E.kahan) E.kahan_add_z("      ");
      });
      std::string flushes = capture(E, [&] { row_change("      "); });
      o << decl << rename_operands(decl, "B");
      // The loop leaves only at its bottom, after a whole pair of edges: with an exit between the loads of a set
      // and the arithmetic that uses them, the compiler moves the loads behind that exit (they are not needed on
      // the path that leaves) and the wave waits for them with nothing else in flight.  A range with an odd number
      // of edges therefore starts one position early with a phantom edge on the zero-initialised first operand set,
      // which adds exact zeros to the accumulators.
      o << "    i64 e = e0;\n";
      o << "    if (e < e1) {\n";
      o << "      if (((e1 - e0) & 1) == 0) {\n        const i64 en = e;\n" << loads << "      } else {\n        e = e0 - 1;\n      }\n";
      o << "    for (;;) {\n";
      o << flushes;
      o << "      { const i64 en = e + 1;\n" << rename_operands(loads, "B") << "      }\n      __builtin_amdgcn_sched_barrier(0);\n";
      o << compute;
      o << "      ++e;\n";
      o << flushes;
      // unconditional (clamped) prefetch: a branch around the loads would force the wait for the
      // current operands to cover the path on which no newer loads were issued
      o << "      { const i64 en = e + 1 < e1 ? e + 1 : e;\n" << loads << "      }\n      __builtin_amdgcn_sched_barrier(0);\n";
      o << rename_operands(compute, "B");
      o << "      if (++e >= e1) break;\n";
      o << "    }\n    }\n";
    } else {
    o << "    for (i64 e = e0; e < e1; ++e) {\n";
    row_change("      ");
    o << "      const i64 c = col[e]; const i64 er_ = eperm ? eperm[e] : e;\n";
    o << "      const T* xb = x + c * " << DX << "; const T* yb = y + er_ * " << DY << "; const T* wb = W + er_ * " << NW << ";\n";
    E.load_y("yb", "      ");
    E.load_x("xb", "      ");
    if (E.kahan) E.zero_z("      ");
    E.forward_paths("wb", "      ");
    if (E.kahan) E.kahan_add_z("      ");
    o << "    }\n";
    }
    flush("    ");
    if (!atomic) {
    o << "    ++r;\n";
    o << "    while (r < V && row_ptr[r + 1] <= e1) {\n";
    o << "      { T* dst_ = z + r * " << DZ << ";\n";
    E.store_z("dst_", "        ");
    o << "      }\n";
    o << "      ++r;\n";
    o << "    }\n";
    }
    };
    for (size_t ph = 0; ph < zph.size(); ++ph) {
      if (zph.size() > 1) {
        o << "    { // phase " << ph << "\n";
        E.zsel = zph[ph];
        E.store_unused = ph == 0;
      }
      emit_phase();
      if (zph.size() > 1) {
        o << "    }\n    __builtin_amdgcn_sched_barrier(0);\n";
        E.zsel.clear();
        E.store_unused = true;
      }
    }
    o << "  }\n}\n";
  }
  K.source = o.str();
  K.screen_divergence = true;
}

void emit_uvu_forward(const Plan& P, bool conv, Kernel& K) { emit_uvu_forward_impl(P, conv, K, false); }

// ---------------------------------------------------------------------------------------
// Batched backward (paper Alg. 3) and fused convolution backward (paper Sec. 3.5: the same walk
// over the transposed adjacency; x of the sender row and its gx accumulator stay resident).
void emit_uvu_backward(const Plan& P, bool conv, Kernel& K) {
  const LaneMap& M = P.map[conv ? CGTP_K_CONV_BWD : CGTP_K_TP_BWD];
  Em E(P, M, K.sched);
  K.wg = 256;
  const int wpw = K.wg / 64;
  K.name = conv ? "cgtp_conv_bwd" : "cgtp_tp_bwd";
  E.preamble();
  if (conv && M.spw == 1) E.emit_row_of();
  const int DX = (int)P.dim_x(), DY = (int)P.dim_y(), DZ = (int)P.dim_z();
  const i64 NW = P.n_w;
  auto& o = E.o;
  if (!conv) {
    o << "extern \"C\" __global__ void __launch_bounds__(" << K.wg << ") " << occ_attr(M) << K.name
      << "(const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, const T* __restrict__ gz,\n"
         "   T* __restrict__ gx, T* __restrict__ gy, T* __restrict__ gW, i64 B)\n{\n";
    head(E, wpw, true);   // the wave index is wave-uniform also when a wave holds several samples
    E.nt_all = env_int("CGTP_NT_TP", 0);
    E.dup = true;
    o << "  const int sub_ = lane / " << M.G << ";\n";
    E.gy_lane_consts("  ");
    // all lanes of a wave run the same trip count; lanes without a sample of their own work on the last sample once more
    o << "  for (i64 s0 = wave * " << M.spw << "; s0 < B; s0 += nwave * " << M.spw << ") {\n";
    o << "    const i64 b_ = s0 + sub_;\n";
    o << "    const i64 b = b_ < B ? b_ : (B - 1);\n";
    o << "    const T* xb = x + b * " << DX << "; const T* yb = y + b * " << DY << "; const T* wb = W + b * " << NW
      << "; const T* gzb = gz + b * " << DZ << ";\n";
    o << "    T* gxb = gx + b * " << DX << "; T* gyb = gy + b * " << DY << "; T* gwb = gW + b * " << NW << ";\n";
    E.load_y("yb", "    ");
    E.declare_gy("    ", true);
    E.gy_reduce_decls("    ");
    if (M.npass > 1) o << "    #pragma unroll 1\n";
    o << "    for (int pass = 0; pass < " << M.npass << "; ++pass) {\n";
    o << "      const int u0 = (pass * " << M.G << " + g_) * " << M.cpl << ";\n";
    if (M.npass > 1 && env_int("CGTP_Y_PER_PASS", 1)) {
      std::vector<std::string> yy;
      for (int j = *E.used_y_words().begin(); j <= *E.used_y_words().rbegin(); ++j) yy.push_back(Em::Y(j));
      E.pin(yy, "      ");
    }
    // Phases (paper Sec. 3.1, computation schedule): the used x segments are cut into groups of similar
    // register weight; a phase holds only its own x rows and gx accumulators and visits the paths that
    // read them.  gy stays in registers across phases, gz segments are read again by each phase.
    const auto phases = x_phases(E, std::max(1, Em::knob("CGTP_PHASES_TP_BWD", K.sched.phases, 1)));
    for (size_t ph = 0; ph < phases.size(); ++ph) {
      if (phases.size() > 1) {
        o << "      { // phase " << ph << "\n";
        E.xsel = phases[ph];
        E.store_unused = ph == 0;
      }
      E.load_x("xb", "      ");
      E.declare_gx("      ");
      E.backward_paths("wb", "gzb", "gwb", "      ");
      E.store_gx("gxb", "      ");
      if (phases.size() > 1) {
        o << "      }\n      __builtin_amdgcn_sched_barrier(0);\n";
        E.xsel.clear();
        E.store_unused = true;
      }
    }
    o << "    }\n";
    E.reduce_store_gy("gyb", "    ");
    o << "  }\n}\n";
  } else {
    o << "extern \"C\" __global__ void __launch_bounds__(" << K.wg << ") " << occ_attr(M) << K.name
      << "(const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, const T* __restrict__ gz,\n"
         "   T* __restrict__ gx, T* __restrict__ gy, T* __restrict__ gW,\n"
         "   const i64* __restrict__ t_row_ptr, const i64* __restrict__ t_perm, const i64* __restrict__ t_recv,\n"
         "   i64 V, i64 E, T* __restrict__ part, i64 nchunk, const i64* __restrict__ eperm, T* __restrict__ dummy)\n{\n";
    head(E, wpw, true, true);
    E.stream_nt = env_int("CGTP_STREAM_NT", 1) != 0;  // measured: 3-5 % on the backward, neutral on the forward
    E.dup = M.spw == 1;
    E.pin_accumulators = true;
    o << "  if (wave >= nchunk) return;\n";
    E.gy_lane_consts("  ");
    o << "  const i64 e0 = (wave * E) / nchunk, e1 = ((wave + 1) * E) / nchunk;\n";
    o << "  i64 rstart = 0;\n";
    if (M.spw == 1) o << "  if (wave > 0) rstart = row_of(t_row_ptr, V, e0);\n";
    else
    o << "  if (wave > 0) { i64 lo = 0, hi = V; while (hi - lo > 1) { const i64 mid = (lo + hi) >> 1; if (t_row_ptr[mid] <= e0) lo = mid; else hi = mid; } rstart = lo; }\n";
    if (M.npass > 1) o << "  #pragma unroll 1\n";
    o << "  for (int pass = 0; pass < " << M.npass << "; ++pass) {\n";
    o << "    const int u0 = (pass * " << M.G << " + g_) * " << M.cpl << ";\n";
    // Phases: the x segments are cut into groups; a phase walks the whole range of the transposed order with
    // the x rows and gx accumulators of its own segments and visits only the paths that read them (their W, gW
    // and the gz segments they need); gy of an edge is completed phase by phase.
    const auto xph = x_phases(E, std::max(1, Em::knob("CGTP_PHASES_CONV_BWD", K.sched.phases, 1)));
    int phase_index = 0;
    auto emit_phase = [&]() {
    E.kahan = P.kahan_conv;
    E.declare_gx("    ");
    if (E.kahan) E.declare_gx_sums("    ");
    E.load_x("", "    ", true, false);  // x of the current sender row stays in registers
    o << "    i64 r = rstart, rx = -1;\n";
    o << "    i64 rbeg = t_row_ptr[r], rend = t_row_ptr[r + 1];\n";
    auto flush = [&](const char* ind) {
      std::string in2 = std::string(ind) + "  ";
      o << ind << "{ T* dst_ = (rbeg >= e0 && rend <= e1) ? gx + r * " << DX << " : part + (wave * 2 + (rbeg < e0 ? 0 : 1)) * " << DX << ";\n";
      E.store_gx("dst_", in2.c_str());
      if (E.kahan) E.zero_gx_sums(in2.c_str());
      else E.zero_gx(in2.c_str());
      o << ind << "}\n";
    };
    // pipelined walk: a range with an odd number of edges starts with a phantom edge at position e0 - 1 whose operands
    // are zero; what it "computes" (zeros) is stored to a dummy row
    bool phantom = false;
    auto emit_compute = [&](const char* wb_, const char* gzb_) {
      if (phantom) {
        o << "      { const bool ph_ = q < e0; const i64 qq_ = ph_ ? e0 : q;\n";
        o << "      const i64 e = eperm ? eperm[t_perm[qq_]] : t_perm[qq_];\n";
        o << "      T* gyb = ph_ ? dummy : gy + e * " << DY << "; T* gwb = ph_ ? dummy + " << ((DY + 63) / 64 * 64) << " : gW + e * " << NW << ";\n";
      } else {
      o << "      { const i64 e = eperm ? eperm[t_perm[q]] : t_perm[q];\n";
      o << "      T* gyb = gy + e * " << DY << "; T* gwb = gW + e * " << NW << ";\n";
      }
      E.declare_gy("      ", true);
      E.gy_reduce_decls("      ");
      if (E.kahan) E.zero_gx("      ");
      E.backward_paths(wb_, gzb_, "gwb", "      ");
      if (E.kahan) E.kahan_add_gx("      ");
      if (M.npass > 1 || phase_index > 0) {
        // each pass owns a disjoint channel block and each phase a disjoint set of paths; gy needs the sum
        // over all of them: every pass / phase after the first adds to what the earlier ones stored
        o << "      if (" << (phase_index > 0 ? "true" : "pass > 0") << ") {\n";
        for (int j : E.used_y_words()) {
          if (E.dup)   // every lane reads the word, one lane adds it (no lane-conditional region)
            o << "        { const T o_ = __hip_atomic_load(gyb + " << j << ", __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); " << Em::GY(j)
              << " += g_ == 0 ? o_ : (T)0; }\n";
          else
          o << "        if (g_ == 0) " << Em::GY(j) << " += __hip_atomic_load(gyb + " << j << ", __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);\n";
        }
        o << "      }\n";
      }
      E.reduce_store_gy("gyb", "      ");
      o << "      }\n";
    };
    auto emit_pre = [&]() {
      o << "      while (q >= rend && r + 1 < V) {\n";
      flush("        ");
      o << "        ++r; rbeg = rend; rend = t_row_ptr[r + 1];\n";
      o << "      }\n";
      o << "      if (r != rx) {\n";
      o << "        const T* xb = x + r * " << DX << ";\n";
      E.load_x("xb", "        ", false, true);
      o << "        rx = r;\n";
      o << "      }\n";
    };
    // Optional software pipeline (two register sets of y, W, gz; the loads of the next edge are issued
    // before the arithmetic of the current one).
    // (measured: no gain for the backward, in either precision, so off by default)
    const int pf_mode = Em::knob("CGTP_PREFETCH_CONV_BWD", K.sched.prefetch, 0);  // 1: y, W and gz; 2: y and W only
    const bool pipelined = pf_mode != 0;
    const bool pf_gz = pf_mode == 1;
    if (pipelined) {
      E.do_load = false;
      std::string decl = capture(E, [&] {
        E.load_y("", "    ");
        for (size_t p = 0; p < P.paths.size(); ++p)
          if (E.sel(P.paths[p])) E.load_w_path("", p, "    ");
        if (pf_gz)
          for (int sz : E.used_z()) E.load_gz_seg("", sz, "    ");
      });
      E.do_load = true;
      E.do_decl = false;
      std::string loads = capture(E, [&] {
        o << "        const i64 en_ = eperm ? eperm[t_perm[qn]] : t_perm[qn]; const i64 jn_ = t_recv[qn];\n";
        o << "        const T* yb = y + en_ * " << DY << "; const T* wb = W + en_ * " << NW << "; const T* gzb = gz + jn_ * " << DZ << ";\n";
        E.load_y("yb", "        ");
        for (size_t p = 0; p < P.paths.size(); ++p)
          if (E.sel(P.paths[p])) E.load_w_path("wb", p, "        ");
        if (pf_gz)
          for (int sz : E.used_z()) E.load_gz_seg("gzb", sz, "        ");
      });
      E.do_load = false;   // operands are in registers: the path code must not load or declare them
      E.gz_in_path_code = !pf_gz;
      phantom = true;
      std::string compute = capture(E, [&] {
        o << "      {\n";
        if (!pf_gz) o << "      const T* gzb = gz + t_recv[q < e0 ? e0 : q] * " << DZ << ";\n";
        emit_compute("", "gzb");
        o << "      }\n";
      });
      phantom = false;
      E.gz_in_path_code = false;
      E.do_load = true;
      E.do_decl = true;
      std::string pre = capture(E, emit_pre);
      o << decl << rename_operands(decl, "B", true);
      // the loop leaves only at its bottom, after a pair of edges (an exit between the loads of an operand set and
      // their use lets the compiler move the loads behind the exit, where nothing else is in flight while the wave
      // waits for them); odd ranges start with a phantom edge on the zero-initialised first operand set
      o << "    i64 q = e0;\n";
      o << "    if (q < e1) {\n";
      o << "      if (((e1 - e0) & 1) == 0) {\n        const i64 qn = q;\n" << loads << "      } else {\n        q = e0 - 1;\n      }\n";
      o << "    for (;;) {\n";
      o << pre;
      o << "      { const i64 qn = q + 1;\n" << rename_operands(loads, "B", true) << "      }\n      __builtin_amdgcn_sched_barrier(0);\n";
      o << compute;
      o << "      ++q;\n";
      o << pre;
      o << "      { const i64 qn = q + 1 < e1 ? q + 1 : q;\n" << loads << "      }\n      __builtin_amdgcn_sched_barrier(0);\n";
      o << rename_operands(compute, "B", true);
      o << "      if (++q >= e1) break;\n";
      o << "    }\n    }\n";
    } else {
      o << "    for (i64 q = e0; q < e1; ++q) {\n";
      emit_pre();
      o << "      const i64 en_ = eperm ? eperm[t_perm[q]] : t_perm[q];\n";
      o << "      const i64 j = t_recv[q];\n";
      o << "      const T* yb = y + en_ * " << DY << "; const T* wb = W + en_ * " << NW << "; const T* gzb = gz + j * " << DZ << ";\n";
      E.load_y("yb", "      ");
      emit_compute("wb", "gzb");
      o << "    }\n";
    }
    flush("    ");
    o << "    ++r;\n";
    o << "    while (r < V && t_row_ptr[r + 1] <= e1) {\n";
    o << "      { T* dst_ = gx + r * " << DX << ";\n";
    E.store_gx("dst_", "        ");
    o << "      }\n";
    o << "      ++r;\n";
    o << "    }\n";
    };
    for (size_t ph = 0; ph < xph.size(); ++ph) {
      phase_index = (int)ph;
      if (xph.size() > 1) {
        o << "    { // phase " << ph << "\n";
        E.xsel = xph[ph];
        E.store_unused = ph == 0;
      }
      emit_phase();
      if (xph.size() > 1) {
        // the next phase reads back the gy this one stored
        o << "    }\n    __threadfence();\n    __builtin_amdgcn_sched_barrier(0);\n";
        E.xsel.clear();
        E.store_unused = true;
      }
    }
    if (M.npass > 1) o << "    __threadfence();\n";
    o << "  }\n}\n";
  }
  K.source = o.str();
  K.screen_divergence = true;
}

// Nondeterministic convolution for unsorted edge lists (paper Sec. 3.5, the variant "omitted for
// brevity"): one tensor product per edge as in the batched kernels, x gathered by sender, and the
// result added to the receiver's row with one atomic per word; needs neither sorted edges nor the
// transpose permutation.  Outputs are zero-filled by the host side before the launch.
void emit_uvu_atomic(const Plan& P, bool backward, Kernel& K) {
  const LaneMap& M = P.map[backward ? CGTP_K_CONV_BWD_ATOMIC : CGTP_K_CONV_FWD_ATOMIC];
  Em E(P, M, K.sched);
  K.wg = 256;
  const int wpw = K.wg / 64;
  K.name = backward ? "cgtp_conv_bwd_atomic" : "cgtp_conv_fwd_atomic";
  E.preamble();
  const int DX = (int)P.dim_x(), DY = (int)P.dim_y(), DZ = (int)P.dim_z();
  const i64 NW = P.n_w;
  auto& o = E.o;
  if (!backward) {
    emit_uvu_forward_impl(P, true, K, true);
    return;
  } else {
    o << "extern \"C\" __global__ void __launch_bounds__(" << K.wg << ") " << occ_attr(M) << K.name
      << "(const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, const T* __restrict__ gz,\n"
         "   T* __restrict__ gx, T* __restrict__ gy, T* __restrict__ gW,\n"
         "   const i64* __restrict__ recv, const i64* __restrict__ send, i64 B)\n{\n";
    head(E, wpw, true);   // the wave index is wave-uniform also when a wave holds several samples
    E.dup = true;
    E.atomic_live = "live";
    o << "  const int sub_ = lane / " << M.G << ";\n";
    E.gy_lane_consts("  ");
    o << "  for (i64 s0 = wave * " << M.spw << "; s0 < B; s0 += nwave * " << M.spw << ") {\n";
    o << "    const i64 b_ = s0 + sub_;\n";
    o << "    const bool live = b_ < B;\n";
    o << "    const i64 b = live ? b_ : (B - 1);\n";
    o << "    const i64 sn_ = send[b], rc_ = recv[b];\n";
    o << "    const T* xb = x + sn_ * " << DX << "; const T* yb = y + b * " << DY << "; const T* wb = W + b * " << NW
      << "; const T* gzb = gz + rc_ * " << DZ << ";\n";
    o << "    T* gxb = gx + sn_ * " << DX << "; T* gyb = gy + b * " << DY << "; T* gwb = gW + b * " << NW << ";\n";
    E.load_y("yb", "    ");
    E.declare_gy("    ", true);
    E.gy_reduce_decls("    ");
    if (M.npass > 1) o << "    #pragma unroll 1\n";
    o << "    for (int pass = 0; pass < " << M.npass << "; ++pass) {\n";
    o << "      const int u0 = (pass * " << M.G << " + g_) * " << M.cpl << ";\n";
    if (M.npass > 1 && env_int("CGTP_Y_PER_PASS", 1)) {
      std::vector<std::string> yy;
      for (int j = *E.used_y_words().begin(); j <= *E.used_y_words().rbegin(); ++j) yy.push_back(Em::Y(j));
      E.pin(yy, "      ");
    }
    E.load_x("xb", "      ");
    E.declare_gx("      ");
    E.backward_paths("wb", "gzb", "gwb", "      ");
    E.atomic_store = true;    // lanes without a sample of their own (and duplicate channels) add zeros
    E.store_gx("gxb", "      ");
    E.atomic_store = false;
    o << "    }\n";
    E.reduce_store_gy("gyb", "    ");
    o << "  }\n}\n";
  }
  K.source = o.str();
  K.screen_divergence = true;
}

// Fused double backward of the batched product (paper Sec. 3.4): one kernel reads x, y, W, gz and
// the three incoming gradients once and writes dL/dx, dL/dy, dL/dW, dL/dgz.
void emit_uvu_double_backward(const Plan& P, Kernel& K) {
  const LaneMap& M = P.map[CGTP_K_TP_DBL_BWD];
  Em E(P, M, K.sched);
  K.wg = 256;
  const int wpw = K.wg / 64;
  K.name = "cgtp_tp_dbl_bwd";
  E.preamble();
  const int DX = (int)P.dim_x(), DY = (int)P.dim_y(), DZ = (int)P.dim_z();
  const i64 NW = P.n_w;
  auto& o = E.o;
  o << "extern \"C\" __global__ void __launch_bounds__(" << K.wg << ") " << occ_attr(M, K.sched) << K.name
    << "(const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, const T* __restrict__ gz,\n"
       "   const T* __restrict__ La, const T* __restrict__ Lb, const T* __restrict__ LC,\n"
       "   T* __restrict__ Lx, T* __restrict__ Ly, T* __restrict__ LW, T* __restrict__ Lgz, i64 B)\n{\n";
  head(E, wpw, true);   // the wave index is wave-uniform also when a wave holds several samples
  E.nt_all = env_int("CGTP_NT_TP", 0);
  E.dup = true;
  o << "  const int sub_ = lane / " << M.G << ";\n";
  E.gy_lane_consts("  ");
  // all lanes of a wave run the same trip count so that the cross-lane sums stay convergent
  o << "  for (i64 s0 = wave * " << M.spw << "; s0 < B; s0 += nwave * " << M.spw << ") {\n";
  o << "    const i64 b_ = s0 + sub_;\n";
  o << "    const i64 b = b_ < B ? b_ : (B - 1);   // lanes without a sample of their own: the last sample once more\n";
  o << "    const T* xb = x + b * " << DX << "; const T* yb = y + b * " << DY << "; const T* wb = W + b * " << NW
    << "; const T* gzb = gz + b * " << DZ << ";\n";
  o << "    const T* axb = La + b * " << DX << "; const T* byb = Lb + b * " << DY << "; const T* cwb = LC + b * " << NW << ";\n";
  o << "    T* lxb = Lx + b * " << DX << "; T* lyb = Ly + b * " << DY << "; T* lwb = LW + b * " << NW
    << "; T* lgzb = Lgz + b * " << DZ << ";\n";
  E.load_y("yb", "    ");
  E.load_y("byb", "    ", "b");
  E.declare_gy("    ", true);
  E.gy_reduce_decls("    ");
  if (M.npass > 1) o << "    #pragma unroll 1\n";
  o << "    for (int pass = 0; pass < " << M.npass << "; ++pass) {\n";
  o << "      const int u0 = (pass * " << M.G << " + g_) * " << M.cpl << ";\n";
  if (M.npass > 1) {
    // y and bbar are the same in every pass; claiming to modify them here keeps the compiler from hoisting
    // the products v * y[j] of all paths out of the pass loop (hundreds of registers held across it)
    std::vector<std::string> yy;
    for (int j = *E.used_y_words().begin(); j <= *E.used_y_words().rbegin(); ++j) {
      yy.push_back(Em::Y(j));
      yy.push_back("b" + Em::Y(j));
    }
    E.pin(yy, "      ");
  }
  // Phases over the x segments (as in the batched backward): x, abar and dL/dx of a phase's segments only;
  // dL/dy stays in registers, dL/dgz is completed in memory phase by phase, gz segments are read again.
  const auto phases = x_phases(E, std::max(1, Em::knob("CGTP_PHASES_DBL", K.sched.phases, 1)));
  for (size_t ph = 0; ph < phases.size(); ++ph) {
    if (phases.size() > 1) {
      o << "      { // phase " << ph << "\n";
      E.xsel = phases[ph];
      E.store_unused = ph == 0;
    }
    E.load_x("xb", "      ");
    E.load_x("axb", "      ", true, true, &Em::AX);
    E.declare_gx("      ");
    E.double_backward_paths("wb", "cwb", "gzb", "lwb", "lgzb", "      ");
    E.store_gx("lxb", "      ");
    if (phases.size() > 1) {
      o << "      }\n      __builtin_amdgcn_sched_barrier(0);\n";
      E.xsel.clear();
      E.store_unused = true;
    }
  }
  E.written_z.clear();
  o << "    }\n";
  E.reduce_store_gy("lyb", "    ");
  o << "  }\n}\n";
  K.source = o.str();
  K.screen_divergence = true;
}

// Second-order pass of the fused convolution (paper Sec. 3.4 applied to Eq. 4), in two kernels as the paper
// fuses its seven dispatches into a forward-like and a backward-like one:
//   cgtp_conv_dbl_fwd  walks the receiver-sorted edges like the convolution forward and accumulates
//                      dL/dgz[j] = sum_e TP(abar_k, y_e, W_e) + TP(x_k, bbar_e, W_e) + TP(x_k, y_e, cbar_e);
//   cgtp_conv_dbl_bwd  walks the transposed order like the convolution backward, keeps x_k and abar_k of the
//                      sender row in registers and produces dL/dx[k] (row sums), dL/dy[e] and dL/dW[e].
// Split rows go through the same side buffer and merge kernel as the first-order kernels.
void emit_uvu_conv_double(const Plan& P, bool backward_like, Kernel& K) {
  const LaneMap& M = P.map[backward_like ? CGTP_K_CONV_DBL_BWD : CGTP_K_CONV_DBL_FWD];
  Em E(P, M, K.sched);
  K.wg = 256;
  const int wpw = K.wg / 64;
  K.name = backward_like ? "cgtp_conv_dbl_bwd" : "cgtp_conv_dbl_fwd";
  E.preamble();
  if (M.spw == 1) E.emit_row_of();
  const int DX = (int)P.dim_x(), DY = (int)P.dim_y(), DZ = (int)P.dim_z();
  const i64 NW = P.n_w;
  auto& o = E.o;
  if (!backward_like) {
    o << "extern \"C\" __global__ void __launch_bounds__(" << K.wg << ") " << occ_attr(M, K.sched) << K.name
      << "(const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, const T* __restrict__ La,\n"
         "   const T* __restrict__ Lb, const T* __restrict__ LC, T* __restrict__ z,\n"
         "   const i64* __restrict__ row_ptr, const i64* __restrict__ col, i64 V, i64 E, T* __restrict__ part, i64 nchunk)\n{\n";
    head(E, wpw, true, true);
    E.stream_nt = env_int("CGTP_STREAM_NT", 1) != 0;
    E.dup = M.spw == 1;
    o << "  if (wave >= nchunk) return;\n";
    o << "  const i64 e0 = (wave * E) / nchunk, e1 = ((wave + 1) * E) / nchunk;\n";
    o << "  i64 rstart = 0;\n";
    if (M.spw == 1) o << "  if (wave > 0) rstart = row_of(row_ptr, V, e0);\n";
    else
    o << "  if (wave > 0) { i64 lo = 0, hi = V; while (hi - lo > 1) { const i64 mid = (lo + hi) >> 1; if (row_ptr[mid] <= e0) lo = mid; else hi = mid; } rstart = lo; }\n";
    if (M.npass > 1) o << "  #pragma unroll 1\n";
    o << "  for (int pass = 0; pass < " << M.npass << "; ++pass) {\n";
    o << "    const int u0 = (pass * " << M.G << " + g_) * " << M.cpl << ";\n";
    E.declare_z("    ");
    o << "    i64 r = rstart;\n";
    o << "    i64 rbeg = row_ptr[r], rend = row_ptr[r + 1];\n";
    auto flush = [&](const char* ind) {
      std::string in2 = std::string(ind) + "  ";
      o << ind << "{ T* dst_ = (rbeg >= e0 && rend <= e1) ? z + r * " << DZ << " : part + (wave * 2 + (rbeg < e0 ? 0 : 1)) * " << DZ << ";\n";
      E.store_z("dst_", in2.c_str());
      E.zero_z(in2.c_str());
      o << ind << "}\n";
    };
    o << "    for (i64 e = e0; e < e1; ++e) {\n";
    o << "      while (e >= rend && r + 1 < V) {\n";
    flush("        ");
    o << "        ++r; rbeg = rend; rend = row_ptr[r + 1];\n";
    o << "      }\n";
    o << "      const i64 c = col[e];\n";
    o << "      const T* xb = x + c * " << DX << "; const T* axb = La + c * " << DX << "; const T* yb = y + e * " << DY
      << "; const T* byb = Lb + e * " << DY << "; const T* wb = W + e * " << NW << "; const T* cwb = LC + e * " << NW << ";\n";
    E.load_y("yb", "      ");
    E.load_y("byb", "      ", "b");
    E.load_x("xb", "      ");
    E.load_x("axb", "      ", true, true, &Em::AX);
    E.double_forward_paths("wb", "cwb", "      ");
    o << "    }\n";
    flush("    ");
    o << "    ++r;\n";
    o << "    while (r < V && row_ptr[r + 1] <= e1) {\n";
    o << "      { T* dst_ = z + r * " << DZ << ";\n";
    E.store_z("dst_", "        ");
    o << "      }\n";
    o << "      ++r;\n";
    o << "    }\n";
    o << "  }\n}\n";
  } else {
    o << "extern \"C\" __global__ void __launch_bounds__(" << K.wg << ") " << occ_attr(M, K.sched) << K.name
      << "(const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, const T* __restrict__ gz,\n"
         "   const T* __restrict__ La, const T* __restrict__ Lb, const T* __restrict__ LC,\n"
         "   T* __restrict__ gx, T* __restrict__ gy, T* __restrict__ gW,\n"
         "   const i64* __restrict__ t_row_ptr, const i64* __restrict__ t_perm, const i64* __restrict__ t_recv,\n"
         "   i64 V, i64 E, T* __restrict__ part, i64 nchunk)\n{\n";
    head(E, wpw, true, true);
    E.stream_nt = env_int("CGTP_STREAM_NT", 1) != 0;
    E.dup = M.spw == 1;
    E.emit_lz = false;
    o << "  if (wave >= nchunk) return;\n";
    E.gy_lane_consts("  ");
    o << "  const i64 e0 = (wave * E) / nchunk, e1 = ((wave + 1) * E) / nchunk;\n";
    o << "  i64 rstart = 0;\n";
    if (M.spw == 1) o << "  if (wave > 0) rstart = row_of(t_row_ptr, V, e0);\n";
    else
    o << "  if (wave > 0) { i64 lo = 0, hi = V; while (hi - lo > 1) { const i64 mid = (lo + hi) >> 1; if (t_row_ptr[mid] <= e0) lo = mid; else hi = mid; } rstart = lo; }\n";
    if (M.npass > 1) o << "  #pragma unroll 1\n";
    o << "  for (int pass = 0; pass < " << M.npass << "; ++pass) {\n";
    o << "    const int u0 = (pass * " << M.G << " + g_) * " << M.cpl << ";\n";
    E.declare_gx("    ");
    E.load_x("", "    ", true, false);              // x and abar of the current sender row stay in registers
    E.load_x("", "    ", true, false, &Em::AX);
    o << "    i64 r = rstart, rx = -1;\n";
    o << "    i64 rbeg = t_row_ptr[r], rend = t_row_ptr[r + 1];\n";
    auto flush = [&](const char* ind) {
      std::string in2 = std::string(ind) + "  ";
      o << ind << "{ T* dst_ = (rbeg >= e0 && rend <= e1) ? gx + r * " << DX << " : part + (wave * 2 + (rbeg < e0 ? 0 : 1)) * " << DX << ";\n";
      E.store_gx("dst_", in2.c_str());
      E.zero_gx(in2.c_str());
      o << ind << "}\n";
    };
    o << "    for (i64 q = e0; q < e1; ++q) {\n";
    o << "      while (q >= rend && r + 1 < V) {\n";
    flush("        ");
    o << "        ++r; rbeg = rend; rend = t_row_ptr[r + 1];\n";
    o << "      }\n";
    o << "      if (r != rx) {\n";
    o << "        const T* xb = x + r * " << DX << "; const T* axb = La + r * " << DX << ";\n";
    E.load_x("xb", "        ", false, true);
    E.load_x("axb", "        ", false, true, &Em::AX);
    o << "        rx = r;\n";
    o << "      }\n";
    o << "      const i64 e = t_perm[q];\n";
    o << "      const i64 j = t_recv[q];\n";
    o << "      const T* yb = y + e * " << DY << "; const T* byb = Lb + e * " << DY << "; const T* wb = W + e * " << NW
      << "; const T* cwb = LC + e * " << NW << "; const T* gzb = gz + j * " << DZ << ";\n";
    o << "      T* gyb = gy + e * " << DY << "; T* gwb = gW + e * " << NW << ";\n";
    E.load_y("yb", "      ");
    E.load_y("byb", "      ", "b");
    o << "      {\n";
    E.declare_gy("      ", true);
    E.gy_reduce_decls("      ");
    E.double_backward_paths("wb", "cwb", "gzb", "gwb", "", "      ");
    if (M.npass > 1) {
      // each pass owns a disjoint channel block; dL/dy needs the sum over all of them
      o << "      if (pass > 0) {\n";
      for (int jj : E.used_y_words()) {
        if (E.dup)
          o << "        { const T o_ = __hip_atomic_load(gyb + " << jj << ", __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); " << Em::GY(jj)
            << " += g_ == 0 ? o_ : (T)0; }\n";
        else
        o << "        if (g_ == 0) " << Em::GY(jj) << " += __hip_atomic_load(gyb + " << jj << ", __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);\n";
      }
      o << "      }\n";
    }
    E.reduce_store_gy("gyb", "      ");
    o << "      }\n";
    o << "    }\n";
    flush("    ");
    o << "    ++r;\n";
    o << "    while (r < V && t_row_ptr[r + 1] <= e1) {\n";
    o << "      { T* dst_ = gx + r * " << DX << ";\n";
    E.store_gx("dst_", "        ");
    o << "      }\n";
    o << "      ++r;\n";
    o << "    }\n";
    if (M.npass > 1) o << "    __threadfence();\n";
    o << "  }\n}\n";
  }
  K.source = o.str();
  K.screen_divergence = true;
}

// Merge kernel for rows split between waves: workgroup w handles the row that begins inside
// chunk w and continues past its end: out[row] = part[w][1] + sum of part[w'][0] for the
// following chunks that start inside the same row, in chunk order (deterministic).
void emit_fixup(const Plan& P, Kernel& K) {
  Em E(P, P.map[CGTP_K_CONV_FWD]);
  K.wg = 256;
  K.name = "cgtp_conv_fixup";
  E.preamble();
  E.emit_row_of();
  E.o << "extern \"C\" __global__ void __launch_bounds__(" << K.wg << ") " << K.name
      << "(T* __restrict__ out, const T* __restrict__ part, const i64* __restrict__ ptr, i64 V, i64 E, i64 nchunk, int dim)\n{\n"
         "  const i64 w = blockIdx.x;\n"
         "  const i64 e0 = (w * E) / nchunk, e1 = ((w + 1) * E) / nchunk;\n"
         "  if (e1 <= e0 || e1 >= E) return;\n"
         "  const i64 lo = row_of(ptr, V, e1 - 1);\n"
         "  const i64 rbeg = ptr[lo], rend = ptr[lo + 1];\n"
         "  if (!(rend > e1 && rbeg >= e0)) return;\n"
         "  for (int d = threadIdx.x; d < dim; d += blockDim.x) {\n"
         "    T acc = part[(w * 2 + 1) * dim + d];\n";
  if (P.kahan_conv)   // the pieces of a split row are added with the same compensated sum as the edges inside a piece
    E.o << "    T cmp = (T)0;\n"
           "    for (i64 v = w + 1; v < nchunk && (v * E) / nchunk < rend; ++v) {\n"
           "      const T y_ = part[(v * 2) * dim + d] - cmp; const T t_ = acc + y_; cmp = (t_ - acc) - y_; acc = t_;\n"
           "    }\n";
  else
    E.o << "    for (i64 v = w + 1; v < nchunk && (v * E) / nchunk < rend; ++v) acc += part[(v * 2) * dim + d];\n";
  E.o << "    out[lo * dim + d] = acc;\n"
         "  }\n}\n";
  K.source = E.o.str();
}

}  // namespace cgtp
