// HIP source generation for "uvw" problems with per-sample weights (the paper's sub-kernel C as it is used
// by models whose weights come from a per-edge network; paper Sec. 2.3 and Alg. 2, backward Alg. 3).
//
// Every sample brings its own dense tile W_p[u, w] per path, read exactly once, so the operation is a stream of
// weights through HBM with a few flops per word and nothing to reuse: no matrix cores, no weight staging.  One
// wave works on one sample at a time.
//   forward   z'_p[u, k] is formed with lane = u (unrolled nonzeros, as in the uvu kernels) and parked in LDS;
//             the weight tile is read in its memory order by lanes (g, w) = (lane / mul_z, lane % mul_z), so
//             a load covers floor(64 / mul_z) consecutive rows u; every lane accumulates W[u, w] z'[u, k] over
//             its rows, and the floor(64 / mul_z) partial sums per (w, k) are added through LDS once per
//             output segment.
//   backward  gW[u, w] = sum_k z'[u, k] gz[w, k] is lane-local in the same (g, w) layout and stored in memory
//             order.  G'[u, k] = sum_w W[u, w] gz[w, k] needs the tile the other way round: it goes through LDS
//             (written in memory order, read by lanes (h, u) = (lane / mul_x, lane % mul_x)), the partial sums
//             over h are added through LDS, and gx / gy follow from G' with lane = u as in the uvu backward.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <functional>
#include <map>
#include <set>
#include <sstream>
#include <stdexcept>

#include "plan.hpp"

namespace cgtp {

namespace {

std::string lit_ps(double v, bool f64) {
  char b[48];
  if (f64) std::snprintf(b, sizeof b, "(%.17e)", v);
  else std::snprintf(b, sizeof b, "(%.9ef)", v);
  return b;
}

struct Geo {
  int max_n3 = 1;
  int64_t zq = 1;     // words of the z' parking area (max over paths of mul_x * (2 l3 + 1))
  int64_t tile = 1;   // words of the transposed weight tile (max over paths of mul_x * (mul_z + 1))
  int64_t gzs = 1;    // words of one gz segment (max over used z segments of mul_z * (2 l3 + 1))
};

Geo geometry(const Plan& P) {
  Geo g;
  for (auto& q : P.paths) {
    if (q.mul_x > 64 || q.mul_z > 64) throw std::runtime_error("uvw with per-sample weights: multiplicities above 64 are not supported");
    const int n3 = 2 * q.l3 + 1;
    g.max_n3 = std::max(g.max_n3, n3);
    g.zq = std::max<int64_t>(g.zq, (int64_t)q.mul_x * n3);
    g.tile = std::max<int64_t>(g.tile, (int64_t)q.mul_x * (q.mul_z + 1));
    g.gzs = std::max<int64_t>(g.gzs, (int64_t)q.mul_z * n3);
  }
  return g;
}

void preamble(std::ostringstream& o, const Plan& P) {
  const bool f64 = P.dtype == CGTP_F64;
  o << "typedef " << (f64 ? "double" : "float") << " T;\ntypedef long long i64;\n";
  o << "#define FMA(a, b, c) " << (f64 ? "__builtin_fma" : "__builtin_fmaf") << "((a), (b), (c))\n";
}

// The distinct products |coeff * C| * y[j] of a path; returns per nonzero (name, negated).  `src` names the wave's
// copy of the vector ("y" or, in the second-order pass, "b" for dL/db), `loc` the per-path laundered copy, `tn` the
// products.
std::vector<std::pair<std::string, bool>> t_products(std::ostringstream& o, const Plan& P, const PathInfo& q, const char* ind,
                                                     const std::string& src = "y", const std::string& loc = "yl", const std::string& tn = "t") {
  const bool f64 = P.dtype == CGTP_F64;
  std::map<std::pair<long long, int>, std::string> seen;
  std::vector<std::pair<std::string, bool>> tr;
  int tc = 0;
  // the path's y words pass through an empty asm: products with equal literals are otherwise shared between paths
  // and stay live from the first path that forms them to the last that uses them (hundreds of registers for a plan
  // with many paths)
  {
    std::set<int> js;
    for (auto& n : q.nz) js.insert((int)P.offy[q.iy] + n.j);
    for (int j : js) o << ind << "T " << loc << j << " = " << src << j << "; asm volatile(\"\" : \"+v\"(" << loc << j << "));\n";
  }
  for (auto& n : q.nz) {
    const double c = n.v * q.coeff, a = std::fabs(c);
    auto key = std::make_pair(std::llround(a * 1e13), n.j);
    auto f = seen.find(key);
    if (f == seen.end()) {
      std::string name = loc + std::to_string((int)P.offy[q.iy] + n.j);
      if (std::fabs(a - 1.0) >= 1e-15) {
        std::string t_ = tn + std::to_string(tc++);
        o << ind << "const T " << t_ << " = " << name << " * " << lit_ps(a, f64) << ";\n";
        name = t_;
      }
      f = seen.insert({key, name}).first;
    }
    tr.push_back({f->second, c < 0});
  }
  return tr;
}

// out<k> (+)= sum over the nonzeros of tr * <xp><seg>_<i> for lane = u; `init` declares out0..out<n3-1> first
void z_prime(std::ostringstream& o, const PathInfo& q, const std::vector<std::pair<std::string, bool>>& tr, const char* ind,
             const std::string& xp = "x", const std::string& out = "zq", bool init = true) {
  const int n3 = 2 * q.l3 + 1;
  std::vector<bool> started((size_t)n3, !init);
  for (size_t m = 0; m < q.nz.size(); ++m) {
    const Nz& nz = q.nz[m];
    const std::string tt = std::string(tr[m].second ? "-" : "") + tr[m].first;
    const std::string xx = xp + std::to_string(q.ix) + "_" + std::to_string(nz.i);
    if (!started[nz.k]) {
      o << ind << "T " << out << nz.k << " = " << tt << " * " << xx << ";\n";
      started[nz.k] = true;
    } else {
      o << ind << out << nz.k << " = FMA(" << tt << ", " << xx << ", " << out << nz.k << ");\n";
    }
  }
  for (int k = 0; k < n3; ++k)
    if (!started[k]) o << ind << "T " << out << k << " = 0;\n";
}

// the wave's copies of a y-like vector (wave-uniform loads) and an x-like row (lane = u) of sample b
void load_x_y(std::ostringstream& o, const Plan& P, const std::set<int>& used_x, const std::set<int>& ywords,
              const std::string& xsrc = "x", const std::string& ysrc = "y", const std::string& xn = "x", const std::string& yn = "y") {
  const int DX = (int)P.dim_x(), DY = (int)P.dim_y();
  for (int j : ywords) o << "    const T " << yn << j << " = " << ysrc << "[b * " << DY << " + " << j << "];\n";
  for (int sx : used_x) {
    const Irrep& ir = P.irx[sx];
    const int n1 = 2 * ir.l + 1;
    o << "    T";
    for (int i = 0; i < n1; ++i) o << (i ? ", " : " ") << xn << sx << "_" << i << " = 0";
    o << ";\n    if (lane < " << ir.mul << ") { const T* p_ = " << xsrc << " + b * " << DX << " + " << P.offx[sx] << " + lane * " << n1 << ";";
    for (int i = 0; i < n1; ++i) o << " " << xn << sx << "_" << i << " = p_[" << i << "];";
    o << " }\n";
  }
}

// Waves per workgroup: the waves of these kernels never cooperate, so the workgroup size only decides how the LDS
// of a CU can be shared out: four waves while three such workgroups fit a CU, single-wave workgroups otherwise.
// `n` consecutive words, word i by lane i % 64: straight-line code, one statement per 64 words, the last one under
// a lane condition.  Not a loop over i = lane, lane + 64, ...: lanes leave such a loop at different times, the code
// after its exit runs with an empty execution mask until the mask is restored, and register-allocator spill code
// that lands there is lost (seen: a lane index copied to an accumulation register under an empty mask, read back
// as whatever the register held, and used in an address).
static void lane_strided(std::ostringstream& o, const char* ind, int n, const std::function<std::string(const std::string&)>& stmt) {
  for (int at = 0; at < n; at += 64) {
    const std::string i = at ? std::to_string(at) + " + lane" : std::string("lane");
    o << ind;
    if (at + 64 > n) o << "if (lane < " << n - at << ") ";
    o << "{ " << stmt(i) << " }\n";
  }
}

int waves_for(int64_t lds_bytes_per_wave) {
  const int forced = env_int("CGTP_UVWPS_WAVES", 0);
  if (forced > 0) return forced;
  return 4 * lds_bytes_per_wave * 3 <= 160 * 1024 ? 4 : 1;
}

// lane_(v, l): the value lane l holds (wave-uniform result); wave_sum: sum over the 64 lanes, from DPP row sums
// (quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror) and the four row totals
std::string lane_helpers(bool f64) {
  std::string hl;
  if (f64) {
    hl += "template <int ctrl> static __device__ __forceinline__ T dpp_(T v) { const long long b_ = __builtin_bit_cast(long long, v);\n"
          "  const int lo = __builtin_amdgcn_update_dpp(0, (int)b_, ctrl, 0xf, 0xf, true), hi = __builtin_amdgcn_update_dpp(0, (int)(b_ >> 32), ctrl, 0xf, 0xf, true);\n"
          "  return __builtin_bit_cast(T, ((long long)hi << 32) | (unsigned int)lo); }\n";
    hl += "static __device__ __forceinline__ T lane_(T v, const int l) { const long long b_ = __builtin_bit_cast(long long, v);\n"
          "  const int lo = __builtin_amdgcn_readlane((int)b_, l), hi = __builtin_amdgcn_readlane((int)(b_ >> 32), l);\n"
          "  return __builtin_bit_cast(T, ((long long)hi << 32) | (unsigned int)lo); }\n";
  } else {
    hl += "template <int ctrl> static __device__ __forceinline__ T dpp_(T v) { return __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, 0xf, 0xf, true)); }\n";
    hl += "static __device__ __forceinline__ T lane_(T v, const int l) { return __builtin_bit_cast(T, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l)); }\n";
  }
  hl += "#define ROWSTEP(v, c) v += dpp_<c>(v)\n";
  hl += "static __device__ __forceinline__ T wave_sum(T v) { ROWSTEP(v, 0xB1); ROWSTEP(v, 0x4E); ROWSTEP(v, 0x141); ROWSTEP(v, 0x140);\n"
        "  return (lane_(v, 0) + lane_(v, 16)) + (lane_(v, 32) + lane_(v, 48)); }\n";
  return hl;
}

// Paths in processing order (grouped by output segment) and the issue of a path's weight loads: all steps of
// the tile are requested at once into registers w<p>_<st> (a load covers R = floor(64 / mul_z) rows in memory
// order; lanes past the tile get 0), one path ahead when both tiles fit a register budget, so that a wave never
// waits a memory round trip per few rows.
struct Order {
  std::vector<int> seq;   // path indices
};
Order processing_order(const Plan& P) {
  Order od;
  for (size_t sz = 0; sz < P.irz.size(); ++sz)
    for (size_t p = 0; p < P.paths.size(); ++p)
      if (P.paths[p].iz == (int)sz) od.seq.push_back((int)p);
  return od;
}
int tile_steps(const PathInfo& q) { const int R = 64 / q.mul_z; return (q.mul_x + R - 1) / R; }
void declare_weight_registers(std::ostringstream& o, const Plan& P, const std::string& pre = "w") {
  for (size_t p = 0; p < P.paths.size(); ++p) {
    o << "    T";
    for (int st = 0; st < tile_steps(P.paths[p]); ++st) o << (st ? ", " : " ") << pre << p << "_" << st;
    o << ";\n";
  }
}
void issue_weight_loads(std::ostringstream& o, const Plan& P, int p, const char* ind, const std::string& src = "W", const std::string& pre = "w") {
  const PathInfo& q = P.paths[p];
  const int Wd = q.mul_z, R = 64 / Wd, U = q.mul_x, steps = tile_steps(q);
  // (a scheduling fence: without it every load of the sample is moved to the top and holds a register from there)
  o << ind << "__builtin_amdgcn_sched_barrier(0);\n";
  // unconditional loads (a load under a lane condition becomes a branch of its own): lanes past the rows of a
  // step re-read its first word and are set to 0 where a partial last step would otherwise mix them in
  o << ind << "{ const T* wp_ = " << src << " + (b * " << P.n_w << " + " << q.w_off << "); const int lc_ = lane < " << R * Wd << " ? lane : 0;\n";
  for (int st = 0; st < steps; ++st) {
    const int full = std::min(R, U - st * R) * Wd;   // lanes of this load that lie inside the tile
    if (full == R * Wd) {
      o << ind << "  " << pre << p << "_" << st << " = (wp_ + " << st * R * Wd << ")[lc_];\n";   // wave-uniform base, 32-bit lane index
    } else {
      o << ind << "  " << pre << p << "_" << st << " = (wp_ + " << st * R * Wd << ")[lane < " << full << " ? lane : 0];\n";
      o << ind << "  " << pre << p << "_" << st << " = lane < " << full << " ? " << pre << p << "_" << st << " : (T)0;\n";
    }
  }
  o << ind << "}\n";
}
// emits the loads of the path after position idx if they may run ahead; returns whether it did
bool fits_ahead(const Plan& P, int p_cur, int p_next, int tiles = 1) {
  const int words = tiles * (tile_steps(P.paths[p_cur]) + tile_steps(P.paths[p_next])) * (P.dtype == CGTP_F64 ? 2 : 1);
  return words <= env_int("CGTP_UVWPS_AHEAD", 112);
}

void head(std::ostringstream& o, const Plan& P, const std::string& name, const std::string& args, const Geo& g, bool backward,
          int kWavesPS, const std::string& helpers = std::string(), int zq_areas = 1, int occ_request = 0) {
  preamble(o, P);
  o << helpers;
  const int occ = env_int(backward ? "CGTP_UVWPS_OCC_BWD" : "CGTP_UVWPS_OCC_FWD", occ_request);
  o << "extern \"C\" __global__ void __launch_bounds__(" << 64 * kWavesPS << ") "
    << (occ > 0 ? "__attribute__((amdgpu_waves_per_eu(" + std::to_string(occ) + "))) " : std::string()) << name << "(" << args << ", i64 B)\n{\n";
  o << "  __shared__ T lds_zq[" << kWavesPS << "][" << zq_areas * g.zq << "];\n";
  o << "  __shared__ T lds_red[" << kWavesPS << "][" << 64 * g.max_n3 << "];\n";
  if (backward) {
    o << "  __shared__ T lds_wt[" << kWavesPS << "][" << g.tile << "];\n";
    o << "  __shared__ T lds_gz[" << kWavesPS << "][" << g.gzs << "];\n";
  }
  o << "  const int lane0 = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);\n";
  o << "  T* zq = lds_zq[wv];\n  T* red = lds_red[wv];\n";
  if (backward) o << "  T* wt = lds_wt[wv];\n  T* gzs = lds_gz[wv];\n";
  o << "  #pragma unroll 1\n";
  o << "  for (i64 b = (i64)blockIdx.x * " << kWavesPS << " + wv; b < B; b += (i64)gridDim.x * " << kWavesPS << ") {\n";
  // The lane index passes through an empty asm per sample, per output segment and per path: everything derived
  // from it alone (masks, LDS offsets) is otherwise computed once before the sample loop for all paths together
  // and kept, hundreds of values for a plan with many paths.
  o << "    int lane = lane0; asm volatile(\"\" : \"+v\"(lane));\n";
}
const char* kRelaunder = "int ln_ = lane; asm volatile(\"\" : \"+v\"(ln_)); { const int lane = ln_;\n";

}  // namespace

// dbl: the forward-like half of the second-order pass (paper Sec. 3.4), dL/dgz = TP(La, y, W) + TP(x, Lb, W) + TP(x, y, LC)
// in one sweep: with S = z'(La, y) + z'(x, Lb) and Z = z'(x, y) the output is sum_u W[u, w] S[u, k] + LC[u, w] Z[u, k],
// so W and LC are streamed once each instead of W twice and LC once.
static void forward_like(const Plan& P, Kernel& K, bool dbl) {
  const Geo g = geometry(P);
  const int64_t lds_wave = ((dbl ? 2 : 1) * g.zq + 64 * g.max_n3) * (int64_t)P.elt();
  if (lds_wave > 160 * 1024) throw std::runtime_error("uvw with per-sample weights: LDS areas exceed 160 KB");
  const int kWavesPS = waves_for(lds_wave);
  const int DZ = (int)P.dim_z();
  K.wg = 64 * kWavesPS;
  K.name = dbl ? "cgtp_tp_dbl_fwd_uvw_ps" : "cgtp_tp_fwd_uvw_ps";
  std::ostringstream o;
  head(o, P, K.name, dbl ? "const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, const T* __restrict__ La,\n"
                           "   const T* __restrict__ Lb, const T* __restrict__ LC, T* __restrict__ z"
                         : "const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, T* __restrict__ z", g, false,
       kWavesPS, lane_helpers(P.dtype == CGTP_F64), dbl ? 2 : 1);
  std::set<int> used_x, used_z, ywords;
  for (auto& q : P.paths) {
    used_x.insert(q.ix);
    used_z.insert(q.iz);
    for (auto& n : q.nz) ywords.insert((int)P.offy[q.iy] + n.j);
  }
  load_x_y(o, P, used_x, ywords);
  declare_weight_registers(o, P);
  if (dbl) {
    load_x_y(o, P, used_x, ywords, "La", "Lb", "a", "b");
    declare_weight_registers(o, P, "c");
  }
  auto issue = [&](int pp, const char* ind) {
    issue_weight_loads(o, P, pp, ind);
    if (dbl) issue_weight_loads(o, P, pp, ind, "LC", "c");
  };
  const Order od = processing_order(P);
  std::vector<bool> issued(P.paths.size(), false);
  std::vector<int> pos(P.paths.size(), 0);
  for (size_t i = 0; i < od.seq.size(); ++i) pos[od.seq[i]] = (int)i;
  for (size_t sz = 0; sz < P.irz.size(); ++sz) {
    const Irrep& ir = P.irz[sz];
    const int n3 = 2 * ir.l + 1, Wd = ir.mul;
    if (!used_z.count((int)sz)) {
      lane_strided(o, "    ", ir.dim(), [&](const std::string& i) { return "z[b * " + std::to_string(DZ) + " + " + std::to_string(P.offz[sz]) + " + " + i + "] = 0;"; });
      continue;
    }
    const int R = 64 / Wd;
    o << "    { // output segment " << sz << ": lanes (g, w), g < " << R << ", w < " << Wd << "\n";
    o << "      " << kRelaunder;
    o << "      const int g = lane / " << Wd << ", w = lane - g * " << Wd << ";\n";
    o << "      const bool act = g < " << R << ";\n";
    for (int k = 0; k < n3; ++k) o << "      T acc" << k << " = 0;\n";
    for (size_t p = 0; p < P.paths.size(); ++p) {
      const PathInfo& q = P.paths[p];
      if (q.iz != (int)sz) continue;
      const int U = q.mul_x, steps = (U + R - 1) / R;
      o << "      { // path " << p << ": l=(" << q.l1 << "," << q.l2 << "," << q.l3 << "), tile " << U << " x " << Wd << "\n";
      o << "        " << kRelaunder;
      if (!issued[p]) { issue((int)p, "        "); issued[p] = true; }
      auto tr = t_products(o, P, q, "        ");
      z_prime(o, q, tr, "        ");
      if (dbl) {
        auto trb = t_products(o, P, q, "        ", "b", "bl", "s");
        z_prime(o, q, tr, "        ", "a", "sq", true);
        z_prime(o, q, trb, "        ", "x", "sq", false);
      }
      if (R > 1) {   // several rows per load: z' of the lane's row comes from LDS
        o << "        __builtin_amdgcn_wave_barrier();\n";
        o << "        if (lane < " << U << ") {";
        for (int k = 0; k < n3; ++k) o << " zq[lane * " << n3 << " + " << k << "] = zq" << k << ";";
        if (dbl)
          for (int k = 0; k < n3; ++k) o << " zq[" << g.zq << " + lane * " << n3 << " + " << k << "] = sq" << k << ";";
        o << " }\n";
        o << "        __builtin_amdgcn_wave_barrier();\n";
      }
      if ((size_t)pos[p] + 1 < od.seq.size()) {
        const int nx = od.seq[pos[p] + 1];
        if (fits_ahead(P, (int)p, nx, dbl ? 2 : 1)) { issue(nx, "        "); issued[nx] = true; }
      }
      for (int st = 0; st < steps; ++st) {
        const std::string zs = dbl ? "sq" : "zq";   // the vector the W tile multiplies
        if (R == 1) {   // one row per load: z'[st, k] is wave-uniform, read from lane st
          o << "        {";
          for (int k = 0; k < n3; ++k) o << " acc" << k << " = FMA(w" << p << "_" << st << ", lane_(" << zs << k << ", " << st << "), acc" << k << ");";
          if (dbl)
            for (int k = 0; k < n3; ++k) o << " acc" << k << " = FMA(c" << p << "_" << st << ", lane_(zq" << k << ", " << st << "), acc" << k << ");";
          o << " }\n";
        } else {
          // lanes past the tile carry w = 0 and read row 0 of z'
          o << "        { const int u_ = " << st * R << " + g; const T* zr = zq + (act && u_ < " << U << " ? u_ : 0) * " << n3 << ";";
          for (int k = 0; k < n3; ++k) o << " acc" << k << " = FMA(w" << p << "_" << st << ", zr[" << (dbl ? g.zq : 0) + k << "], acc" << k << ");";
          if (dbl)
            for (int k = 0; k < n3; ++k) o << " acc" << k << " = FMA(c" << p << "_" << st << ", zr[" << k << "], acc" << k << ");";
          o << " }\n";
        }
        if ((st + 1) % std::min(8, std::max(1, 24 / n3)) == 0) o << "        __builtin_amdgcn_sched_barrier(0);\n";
      }
      o << "      } }\n";
    }
    if (R > 1) {
      o << "      __builtin_amdgcn_wave_barrier();\n";
      for (int k = 0; k < n3; ++k) o << "      red[lane * " << n3 << " + " << k << "] = acc" << k << ";\n";
      o << "      __builtin_amdgcn_wave_barrier();\n";
      o << "      if (lane < " << Wd << ") {\n";
      for (int k = 0; k < n3; ++k) {
        o << "        T s" << k << " = red[lane * " << n3 << " + " << k << "];\n";
        for (int gg = 1; gg < R; ++gg) o << "        s" << k << " += red[(" << gg * Wd << " + lane) * " << n3 << " + " << k << "];\n";
      }
      o << "        T* p_ = z + b * " << DZ << " + " << P.offz[sz] << " + lane * " << n3 << ";\n";
      for (int k = 0; k < n3; ++k) o << "        p_[" << k << "] = s" << k << ";\n";
      o << "      }\n";
      o << "      __builtin_amdgcn_wave_barrier();\n";
    } else {
      o << "      if (lane < " << Wd << ") { T* p_ = z + b * " << DZ << " + " << P.offz[sz] << " + lane * " << n3 << ";";
      for (int k = 0; k < n3; ++k) o << " p_[" << k << "] = acc" << k << ";";
      o << " }\n";
    }
    o << "    } }\n";
  }
  o << "  }\n}\n";
  K.source = o.str();
}

void emit_uvw_ps_forward(const Plan& P, Kernel& K) { forward_like(P, K, false); }
void emit_uvw_ps_double_forward(const Plan& P, Kernel& K) { forward_like(P, K, true); }

// dbl: the backward-like half of the second-order pass (paper Sec. 3.4): dL/dx, dL/dy and dL/dW of the four
// backward dispatches in one sweep.  With S = z'(La, y) + z'(x, Lb), G = W gz and H = LC gz (both per (u, k)):
//   dL/dW[u, w] = sum_k S[u, k] gz[w, k],  dL/dx[u, i] = sum C (Lb_j G[u, k] + y_j H[u, k]),
//   dL/dy[j] = sum_u sum C (La[u, i] G[u, k] + x[u, i] H[u, k]).
// W and LC are streamed once each and dL/dW written once (the four dispatches read four tiles and write four).
static void backward_like(const Plan& P, Kernel& K, bool dbl) {
  const bool f64 = P.dtype == CGTP_F64;
  const Geo g = geometry(P);
  const bool one = dbl && K.sched.one_kernel > 0;   // dL/dgz too: the forward-like half runs on the weight tiles while they are in registers
  const int64_t lds_wave = ((one ? 2 : 1) * g.zq + 64 * g.max_n3 + g.tile + g.gzs) * (int64_t)P.elt();
  if (lds_wave > 160 * 1024)
    throw std::runtime_error("uvw with per-sample weights: the backward's LDS tiles exceed 160 KB for these degrees and multiplicities");
  const int kWavesPS = waves_for(lds_wave);
  const int DX = (int)P.dim_x(), DY = (int)P.dim_y(), DZ = (int)P.dim_z();
  K.wg = 64 * kWavesPS;
  K.name = dbl ? "cgtp_tp_dbl_bwd_uvw_ps" : "cgtp_tp_bwd_uvw_ps";
  if (DY > 64) throw std::runtime_error("uvw with per-sample weights: more than 64 y words are not supported");
  std::ostringstream o;
  const std::string hl = lane_helpers(f64);
  head(o, P, K.name, dbl ? std::string("const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, const T* __restrict__ gz,\n")+
                           "   const T* __restrict__ La, const T* __restrict__ Lb, const T* __restrict__ LC,\n"
                           "   T* __restrict__ gx, T* __restrict__ gy, T* __restrict__ gW" + std::string(one ? ", T* __restrict__ gzo" : "")
                         : "const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, const T* __restrict__ gz,\n"
                           "   T* __restrict__ gx, T* __restrict__ gy, T* __restrict__ gW", g, true, kWavesPS, hl, one ? 2 : 1,
       K.sched.occ > 0 ? K.sched.occ : 0);   // waves per SIMD asked of the compiler, set by the planner
  std::set<int> used_x, used_z, ywords;
  for (auto& q : P.paths) {
    used_x.insert(q.ix);
    used_z.insert(q.iz);
    for (auto& n : q.nz) ywords.insert((int)P.offy[q.iy] + n.j);
  }
  load_x_y(o, P, used_x, ywords);
  for (int sx : used_x)
    for (int i = 0; i < 2 * P.irx[sx].l + 1; ++i) o << "    T gx" << sx << "_" << i << " = 0;\n";
  for (int j : ywords) o << "    T gy" << j << " = 0;\n";
  declare_weight_registers(o, P);
  if (dbl) {
    load_x_y(o, P, used_x, ywords, "La", "Lb", "a", "b");
    declare_weight_registers(o, P, "c");
  }
  auto issue = [&](int pp, const char* ind) {
    issue_weight_loads(o, P, pp, ind);
    if (dbl) issue_weight_loads(o, P, pp, ind, "LC", "c");
  };
  const Order od = processing_order(P);
  std::vector<bool> issued(P.paths.size(), false);
  std::vector<int> pos(P.paths.size(), 0);
  for (size_t i = 0; i < od.seq.size(); ++i) pos[od.seq[i]] = (int)i;
  for (size_t sz = 0; sz < P.irz.size(); ++sz) {
    if (!used_z.count((int)sz)) {
      if (one) lane_strided(o, "    ", P.irz[sz].dim(), [&](const std::string& i) { return "gzo[b * " + std::to_string(DZ) + " + " + std::to_string(P.offz[sz]) + " + " + i + "] = 0;"; });
      continue;
    }
    const Irrep& ir = P.irz[sz];
    const int n3 = 2 * ir.l + 1, Wd = ir.mul;
    const int R = 64 / Wd;
    o << "    { // output segment " << sz << "\n";
    o << "      " << kRelaunder;
    // the gz segment of this sample: in LDS (read by w from every layout) and, for the lanes (g, w), in registers
    o << "      __builtin_amdgcn_wave_barrier();\n";
    lane_strided(o, "      ", Wd * n3, [&](const std::string& i) { return "gzs[" + i + "] = gz[b * " + std::to_string(DZ) + " + " + std::to_string(P.offz[sz]) + " + " + i + "];"; });
    o << "      __builtin_amdgcn_wave_barrier();\n";
    o << "      const int g = lane / " << Wd << ", w = lane - g * " << Wd << ";\n";
    o << "      const bool act = g < " << R << ";\n";
    for (int k = 0; k < n3; ++k) o << "      const T gzl" << k << " = gzs[w * " << n3 << " + " << k << "];\n";
    if (one)
      for (int k = 0; k < n3; ++k) o << "      T fa" << k << " = 0;\n";      // dL/dgz[w, k] of the lane's rows
    for (size_t p = 0; p < P.paths.size(); ++p) {
      const PathInfo& q = P.paths[p];
      if (q.iz != (int)sz) continue;
      const int U = q.mul_x, steps = (U + R - 1) / R, n1 = 2 * q.l1 + 1;
      (void)n1;
      const int R2 = 64 / U, steps2 = (Wd + R2 - 1) / R2, pitch = Wd + 1;
      o << "      { // path " << p << ": l=(" << q.l1 << "," << q.l2 << "," << q.l3 << "), tile " << U << " x " << Wd << "\n";
      o << "        " << kRelaunder;
      if (!issued[p]) { issue((int)p, "        "); issued[p] = true; }
      auto tr = t_products(o, P, q, "        ");
      std::vector<std::pair<std::string, bool>> trb;
      if (dbl) {   // the vector whose outer product with gz is dL/dW
        trb = t_products(o, P, q, "        ", "b", "bl", "s");
        z_prime(o, q, tr, "        ", "a", "zq", true);
        z_prime(o, q, trb, "        ", "x", "zq", false);
        if (one) z_prime(o, q, tr, "        ", "x", "zz", true);      // Z = z'(x, y), the vector LC multiplies in dL/dgz
      } else {
        z_prime(o, q, tr, "        ");
      }
      o << "        __builtin_amdgcn_wave_barrier();\n";
      o << "        if (lane < " << U << ") {";
      for (int k = 0; k < n3; ++k) o << " zq[lane * " << n3 << " + " << k << "] = zq" << k << ";";
      if (one && R > 1)
        for (int k = 0; k < n3; ++k) o << " zq[" << g.zq << " + lane * " << n3 << " + " << k << "] = zz" << k << ";";
      o << " }\n";
      o << "        __builtin_amdgcn_wave_barrier();\n";
      // gW in memory order, and the weight tile into LDS for the transposed read
      o << "        T* gwp = gW + (b * " << P.n_w << " + " << q.w_off << ");\n";
      // the lanes inside the rows of a load work under one condition (a condition per step is a branch per step)
      auto gw_step = [&](int st, const char* ind) {
        if (R == 1) {   // one row per load: z'[st, k] is wave-uniform, read from lane st
          o << ind << "{ T v_ = lane_(zq0, " << st << ") * gzl0;";
          for (int k = 1; k < n3; ++k) o << " v_ = FMA(lane_(zq" << k << ", " << st << "), gzl" << k << ", v_);";
          // rows beyond the tile's width (mul_x > mul_z) sit in lanes the store condition switches off: a lane's value
          // may only be read across lanes while that lane is active (the compiler is free to compute z' under the
          // condition of its readers), so there the condition guards the stores alone
          if (one)      // dL/dgz[w, k] += W[st, w] S[st, k] + LC[st, w] Z[st, k] (lanes past the tile's width never store theirs)
            for (int k = 0; k < n3; ++k)
              o << " fa" << k << " = FMA(w" << p << "_" << st << ", lane_(zq" << k << ", " << st << "), fa" << k << "); fa" << k << " = FMA(c" << p << "_" << st
                << ", lane_(zz" << k << ", " << st << "), fa" << k << ");";
          if (U > Wd) o << " if (lane < " << Wd << ") {";
          o << " (gwp + " << st * R * Wd << ")[lane] = v_; wt[" << st * pitch << " + w] = w" << p << "_" << st << ";";
          o << (U > Wd ? " } }\n" : " }\n");
        } else {
          o << ind << "{ const T* zr = zq + (" << st * R << " + g) * " << n3 << "; T v_ = zr[0] * gzl0;";
          for (int k = 1; k < n3; ++k) o << " v_ = FMA(zr[" << k << "], gzl" << k << ", v_);";
          if (one)
            for (int k = 0; k < n3; ++k)
              o << " fa" << k << " = FMA(w" << p << "_" << st << ", zr[" << k << "], fa" << k << "); fa" << k << " = FMA(c" << p << "_" << st << ", zr["
                << g.zq + k << "], fa" << k << ");";
          o << " (gwp + " << st * R * Wd << ")[lane] = v_; wt[(" << st * R << " + g) * " << pitch << " + w] = w" << p << "_" << st << "; }\n";
        }
      };
      const int full_steps = U / R;
      if (full_steps > 0) {
        const bool per_step = R == 1 && U > Wd;   // condition inside each step, see gw_step
        o << (per_step ? "        {\n" : "        if (lane < " + std::to_string(R * Wd) + ") {\n");
        for (int st = 0; st < full_steps; ++st) {
          gw_step(st, "          ");
          if ((st + 1) % std::min(8, std::max(1, 24 / n3)) == 0) o << "          __builtin_amdgcn_sched_barrier(0);\n";
        }
        o << "        }\n";
      }
      if (full_steps < steps) {
        o << "        if (lane < " << (U - full_steps * R) * Wd << ") {\n";
        gw_step(full_steps, "          ");
        o << "        }\n";
      }
      o << "        __builtin_amdgcn_wave_barrier();\n";
      // the next tile's loads run during the transposed pass and the VALU part of this path
      if ((size_t)pos[p] + 1 < od.seq.size()) {
        const int nx = od.seq[pos[p] + 1];
        if (fits_ahead(P, (int)p, nx, dbl ? 2 : 1)) { issue(nx, "        "); issued[nx] = true; }
      }
      // G'[u, k] = sum_w W[u, w] gz[w, k]: lanes (h, u) take w = h, h + R2, ...
      o << "        const int h = lane / " << U << ", uu = lane - h * " << U << ";\n";
      o << "        const bool act2 = h < " << R2 << ";\n";
      auto transposed_pass = [&](const std::string& G) {
      for (int k = 0; k < n3; ++k) o << "        T " << G << k << " = 0;\n";
      o << "        #pragma unroll 8\n";
      o << "        for (int sw = 0; sw < " << steps2 << "; ++sw) {\n";
      if (R2 == 1) {   // one column per step: gz[sw, k] is wave-uniform, read from lane sw (lanes >= mul_x are zeroed below)
        o << "          const T a_ = wt[uu * " << pitch << " + sw];\n";
        for (int k = 0; k < n3; ++k) o << "          " << G << k << " = FMA(a_, lane_(gzl" << k << ", sw), " << G << k << ");\n";
      } else {
        o << "          const int w2 = sw * " << R2 << " + h;\n";
        o << "          const bool ok = act2 && w2 < " << Wd << ";\n";
        o << "          T a_ = wt[uu * " << pitch << " + (ok ? w2 : 0)];\n";
        o << "          a_ = ok ? a_ : (T)0;\n";
        o << "          const T* gr = gzs + (ok ? w2 : 0) * " << n3 << ";\n";
        for (int k = 0; k < n3; ++k) o << "          " << G << k << " = FMA(a_, gr[" << k << "], " << G << k << ");\n";
      }
      o << "        }\n";
      if (R2 > 1) {
        o << "        __builtin_amdgcn_wave_barrier();\n";
        for (int k = 0; k < n3; ++k) o << "        red[lane * " << n3 << " + " << k << "] = " << G << k << ";\n";
        o << "        __builtin_amdgcn_wave_barrier();\n";
        for (int k = 0; k < n3; ++k) {
          o << "        " << G << k << " = 0;\n";
        }
        o << "        if (lane < " << U << ") {\n";
        for (int k = 0; k < n3; ++k) {
          o << "          " << G << k << " = red[lane * " << n3 << " + " << k << "];\n";
          for (int hh = 1; hh < R2; ++hh) o << "          " << G << k << " += red[(" << hh * U << " + lane) * " << n3 << " + " << k << "];\n";
        }
        o << "        }\n";
      } else {
        o << "        if (lane >= " << U << ") {";
        for (int k = 0; k < n3; ++k) o << " " << G << k << " = 0;";
        o << " }\n";
      }
      };
      transposed_pass("G");
      if (dbl) {   // the LC tile takes the place of the W tile in LDS, same pass again -> H = LC gz
        o << "        __builtin_amdgcn_wave_barrier();\n";
        const int full_steps2 = U / R;
        if (full_steps2 > 0) {
          o << "        if (lane < " << R * Wd << ") {\n";
          for (int st = 0; st < full_steps2; ++st)
            o << "          wt[(" << st * R << " + g) * " << pitch << " + w] = c" << p << "_" << st << ";\n";
          o << "        }\n";
        }
        if (full_steps2 < steps)
          o << "        if (lane < " << (U - full_steps2 * R) * Wd << ") wt[(" << full_steps2 * R << " + g) * " << pitch << " + w] = c" << p << "_" << full_steps2 << ";\n";
        o << "        __builtin_amdgcn_wave_barrier();\n";
        transposed_pass("H");
      }
      // gx, gy from G' with lane = u (lanes >= mul_x hold G' = 0 and x = 0)
      std::map<std::pair<int, long long>, std::vector<size_t>> groups;
      for (size_t m = 0; m < q.nz.size(); ++m) groups[{q.nz[m].j, std::llround(std::fabs(q.nz[m].v * q.coeff) * 1e13)}].push_back(m);
      for (size_t m = 0; m < q.nz.size(); ++m) {
        const Nz& nz = q.nz[m];
        const std::string tt = std::string(tr[m].second ? "-" : "") + tr[m].first;
        if (dbl) {
          const std::string tb = std::string(trb[m].second ? "-" : "") + trb[m].first;
          o << "        gx" << q.ix << "_" << nz.i << " = FMA(" << tb << ", G" << nz.k << ", gx" << q.ix << "_" << nz.i << ");\n";
          o << "        gx" << q.ix << "_" << nz.i << " = FMA(" << tt << ", H" << nz.k << ", gx" << q.ix << "_" << nz.i << ");\n";
        } else {
          o << "        gx" << q.ix << "_" << nz.i << " = FMA(" << tt << ", G" << nz.k << ", gx" << q.ix << "_" << nz.i << ");\n";
        }
      }
      int gi = 0;
      for (auto& kv : groups) {
        const std::string sn = "sg" + std::to_string(gi++);
        bool first = true;
        for (size_t m : kv.second) {
          const Nz& nz = q.nz[m];
          const bool neg = nz.v * q.coeff < 0;
          const std::string sg_ = neg ? "-" : "";
          const std::string xx = sg_ + "x" + std::to_string(q.ix) + "_" + std::to_string(nz.i);
          const std::string aa = sg_ + "a" + std::to_string(q.ix) + "_" + std::to_string(nz.i);
          if (dbl) {
            if (first) o << "        T " << sn << " = " << aa << " * G" << nz.k << ";\n";
            else o << "        " << sn << " = FMA(" << aa << ", G" << nz.k << ", " << sn << ");\n";
            o << "        " << sn << " = FMA(" << xx << ", H" << nz.k << ", " << sn << ");\n";
          } else {
            if (first) o << "        T " << sn << " = " << xx << " * G" << nz.k << ";\n";
            else o << "        " << sn << " = FMA(" << xx << ", G" << nz.k << ", " << sn << ");\n";
          }
          first = false;
        }
        o << "        gy" << (int)P.offy[q.iy] + kv.first.first << " = FMA(" << sn << ", " << lit_ps(std::fabs(q.nz[kv.second[0]].v * q.coeff), f64) << ", gy"
          << (int)P.offy[q.iy] + kv.first.first << ");\n";
      }
      {
        // the accumulators are read at the end of the sample only: an empty asm brings them up to date here, so that
        // their updates (and every operand those need) are not postponed until then
        std::set<std::string> pins;
        for (auto& nz : q.nz) pins.insert("gx" + std::to_string(q.ix) + "_" + std::to_string(nz.i));
        for (auto& kv : groups) pins.insert("gy" + std::to_string((int)P.offy[q.iy] + kv.first.first));
        std::vector<std::string> pv(pins.begin(), pins.end());
        for (size_t at = 0; at < pv.size(); at += 12) {
          o << "        asm volatile(\"\" :";
          for (size_t t = at; t < pv.size() && t < at + 12; ++t) o << (t > at ? ", " : " ") << "\"+v\"(" << pv[t] << ")";
          o << ");\n";
        }
      }
      o << "        __builtin_amdgcn_wave_barrier();\n";
      o << "      } }\n";
    }
    if (one) {      // dL/dgz of this segment: the partial sums of the lane groups are added through LDS, lanes w < mul_z store
      if (R > 1) {
        o << "      __builtin_amdgcn_wave_barrier();\n";
        for (int k = 0; k < n3; ++k) o << "      red[lane * " << n3 << " + " << k << "] = fa" << k << ";\n";
        o << "      __builtin_amdgcn_wave_barrier();\n";
        o << "      if (lane < " << Wd << ") {\n";
        for (int k = 0; k < n3; ++k) {
          o << "        T s" << k << " = red[lane * " << n3 << " + " << k << "];\n";
          for (int gg = 1; gg < R; ++gg) o << "        s" << k << " += red[(" << gg * Wd << " + lane) * " << n3 << " + " << k << "];\n";
        }
        o << "        T* p_ = gzo + b * " << DZ << " + " << P.offz[sz] << " + lane * " << n3 << ";\n";
        for (int k = 0; k < n3; ++k) o << "        p_[" << k << "] = s" << k << ";\n";
        o << "      }\n";
        o << "      __builtin_amdgcn_wave_barrier();\n";
      } else {
        o << "      if (lane < " << Wd << ") { T* p_ = gzo + b * " << DZ << " + " << P.offz[sz] << " + lane * " << n3 << ";";
        for (int k = 0; k < n3; ++k) o << " p_[" << k << "] = fa" << k << ";";
        o << " }\n";
      }
    }
    o << "    } }\n";
  }
  // gx rows (lane = u), zeros for unused segments
  for (size_t sx = 0; sx < P.irx.size(); ++sx) {
    const Irrep& ir = P.irx[sx];
    const int n1 = 2 * ir.l + 1;
    if (!used_x.count((int)sx)) {
      lane_strided(o, "    ", ir.dim(), [&](const std::string& i) { return "gx[b * " + std::to_string(DX) + " + " + std::to_string(P.offx[sx]) + " + " + i + "] = 0;"; });
      continue;
    }
    o << "    if (lane < " << ir.mul << ") { T* p_ = gx + b * " << DX << " + " << P.offx[sx] << " + lane * " << n1 << ";";
    for (int i = 0; i < n1; ++i) o << " p_[" << i << "] = gx" << sx << "_" << i << ";";
    o << " }\n";
  }
  // gy: sum over the wave, lane j stores word j (words no path touches are zero)
  o << "    { T out_ = 0;\n";
  for (int j = 0; j < DY; ++j)
    if (ywords.count(j)) o << "      { const T s_ = wave_sum(gy" << j << "); out_ = lane == " << j << " ? s_ : out_; }\n";
  o << "      if (lane < " << DY << ") gy[b * " << DY << " + lane] = out_;\n";
  o << "    }\n";
  o << "  }\n}\n";
  K.source = o.str();
}

void emit_uvw_ps_backward(const Plan& P, Kernel& K) { backward_like(P, K, false); }
void emit_uvw_ps_double_backward(const Plan& P, Kernel& K) { backward_like(P, K, true); }

}  // namespace cgtp
