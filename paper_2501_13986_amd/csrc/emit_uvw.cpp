// HIP source generation for "uvw" problems with shared weights (the paper's sub-kernel C: after
// the sparse contraction, the channels u of x are mixed into the channels w of z by a dense
// weight tile; paper Sec. 2.3, Alg. 2 "compute Z += W . Z'").
//
// With one weight tensor for the whole batch this is a real GEMM: rows = (sample, k),
// inner dimension = (path, u), columns = w.  The paper multiplies through shared memory with
// all threads of a warp; here the product runs on the matrix cores:
//   - a wave owns a tile of 16 samples; lane t works for sample t%16 and channel phase t/16;
//   - per step c the lane forms z'_p[u, k] for u = 4c + t/16 with the unrolled CG nonzeros
//     (VALU), which is exactly the A operand layout of v_mfma_f32_16x16x4_f32 (row t%16, k t/16);
//   - B comes from the weight tensor, resident in LDS for the whole workgroup;
//   - the 16x16 accumulators (sample x w) for every (output segment, k, half of w) stay in
//     registers over the whole channel loop, then go through LDS to coalesced row stores.
// x tiles are staged in LDS with an odd row pitch (lanes of one MFMA row group read different
// samples) and the z tile reuses the same LDS region.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <map>
#include <set>
#include <sstream>
#include <stdexcept>

#include "plan.hpp"

namespace cgtp {

namespace {
constexpr int kTile = 16;   // samples per wave tile (MFMA M)
constexpr int kWaves = 4;   // waves per workgroup
int odd_pitch(int64_t d) { return (int)(d | 1); }
std::string lit(double v) {
  char b[48];
  std::snprintf(b, sizeof b, "(%.9ef)", v);
  return b;
}
}  // namespace

namespace {
// names[0..n) <- n consecutive words at p_ (4-byte aligned): widest loads first
void wide_load(std::ostringstream& o, const std::vector<std::string>& names) {
  static const char* comp[4] = {"x", "y", "z", "w"};
  size_t at = 0, n = names.size();
  while (at < n) {
    size_t w = n - at >= 4 ? 4 : (n - at >= 2 ? 2 : 1);
    if (w == 1) {
      o << " " << names[at] << " = p_[" << at << "];";
    } else {
      o << " { const u" << w << " v_ = *(const u" << w << "*)(p_ + " << at << ");";
      for (size_t c = 0; c < w; ++c) o << " " << names[at + c] << " = v_." << comp[c] << ";";
      o << " }";
    }
    at += w;
  }
}
}  // namespace

int64_t uvw_tile_samples(const Plan&) { return (int64_t)kTile * kWaves; }

void emit_uvw_forward(const Plan& P, Kernel& K) {
  if (P.dtype != CGTP_F32) throw std::runtime_error("uvw plans are implemented in fp32 only");
  if (!P.shared_w) throw std::runtime_error("uvw plans need shared weights");
  int maxmul = 0;
  for (auto& q : P.paths) {
    if (q.mul_x % 4) throw std::runtime_error("uvw: mul_x must be a multiple of 4");
    if (q.mul_z % 16) throw std::runtime_error("uvw: mul_z must be a multiple of 16");
    maxmul = std::max(maxmul, q.mul_x);
  }
  const int DX = (int)P.dim_x(), DY = (int)P.dim_y(), DZ = (int)P.dim_z();
  const int XS = odd_pitch(DX), ZS = odd_pitch(DZ);
  // direct mode (default): x and z go straight between global memory and registers, LDS holds only the
  // weights, two workgroups share a CU.  Staged mode (CGTP_UVW_STAGED=1): x and z tiles pass through LDS
  // (coalesced rows), one workgroup per CU.
  const bool staged = env_int("CGTP_UVW_STAGED", 0) != 0;
  const int region = staged ? kTile * std::max(XS, ZS) : 0;
  const int64_t lds_bytes = 4 * (P.n_w + (int64_t)kWaves * region);
  if (lds_bytes > 160 * 1024) throw std::runtime_error("uvw: weights + tiles exceed the 160 KB of LDS");
  K.wg = 64 * kWaves;
  K.name = "cgtp_tp_fwd_uvw";
  std::ostringstream o;
  o << "typedef float T;\ntypedef long long i64;\n";
  o << "typedef float f4 __attribute__((ext_vector_type(4)));\n";
  o << "typedef float u4 __attribute__((ext_vector_type(4), aligned(4)));\n";
  o << "typedef float u2 __attribute__((ext_vector_type(2), aligned(4)));\n";
  o << "#define FMA(a, b, c) __builtin_fmaf((a), (b), (c))\n";
  o << "extern \"C\" __global__ void __launch_bounds__(" << K.wg << ") " << (staged ? "" : "__attribute__((amdgpu_waves_per_eu(" + std::to_string(env_int("CGTP_UVW_OCC", 2)) + "))) ") << K.name
    << "(const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, T* __restrict__ z, i64 B)\n{\n";
  o << "  __shared__ __attribute__((aligned(16))) T lds_w[" << P.n_w << "];\n";
  if (staged) o << "  __shared__ T lds_t[" << kWaves << "][" << region << "];\n";
  // weights -> LDS once per workgroup (the grid is one workgroup per CU slot): all loads of a thread
  // are in flight before its first LDS write
  if (P.n_w % 4 == 0) {
    const int nv = (int)(P.n_w / 4), per = (nv + K.wg - 1) / K.wg;
    o << "  { f4 v_[" << per << "];\n";
    o << "    #pragma unroll\n";
    o << "    for (int it = 0; it < " << per << "; ++it) { const int i4 = it * " << K.wg << " + threadIdx.x; v_[it] = i4 < " << nv
      << " ? *(const f4*)(W + 4 * i4) : (f4){0.0f, 0.0f, 0.0f, 0.0f}; }\n";
    o << "    #pragma unroll\n";
    o << "    for (int it = 0; it < " << per << "; ++it) { const int i4 = it * " << K.wg << " + threadIdx.x; if (i4 < " << nv
      << ") *(f4*)(lds_w + 4 * i4) = v_[it]; }\n";
    o << "  }\n";
  } else {
    o << "  for (int i = threadIdx.x; i < " << P.n_w << "; i += " << K.wg << ") lds_w[i] = W[i];\n";
  }
  o << "  __syncthreads();\n";
  o << "  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;\n";
  o << "  const int s = lane & 15, q = lane >> 4;\n";
  if (staged) o << "  T* tile = lds_t[wv];\n";
  else o << "  (void)wv;\n";
  o << "  const i64 ntile = (B + " << kTile - 1 << ") / " << kTile << ";\n";
  // direct mode: y and the first channel step of x of the NEXT tile are loaded while the current tile computes
  // (a wave would otherwise expose a full memory latency at every tile start); the values travel in yn* / xn*
  const bool carry = !staged && env_int("CGTP_UVW_TILE_PREFETCH", 1) != 0;
  std::set<int> ywords0, used_x0;
  for (auto& p : P.paths) {
    used_x0.insert(p.ix);
    for (auto& n : p.nz) ywords0.insert((int)P.offy[p.iy] + n.j);
  }
  auto emit_tile_loads = [&](const char* tvar, const char* ind) {
    // row of this lane in tile `tvar` (rows past the batch read the tile's first row), then y and x step 0
    o << ind << "{ const i64 bn_ = (" << tvar << ") * " << kTile << "; const int rn_ = (int)((B - bn_) < " << kTile << " ? (B - bn_) : " << kTile
      << "); const i64 row_ = bn_ + (s < rn_ ? s : 0);\n";
    o << ind << "  const T* yb_ = y + row_ * " << DY << ";\n";
    for (int j : ywords0) o << ind << "  yn" << j << " = yb_[" << j << "];\n";
    for (int sx : used_x0) {
      const int n1 = 2 * P.irx[sx].l + 1;
      o << ind << "  { const T* p_ = x + row_ * " << DX << " + " << P.offx[sx] << " + q * " << n1 << ";";
      std::vector<std::string> nm;
      for (int i = 0; i < n1; ++i) nm.push_back("xn" + std::to_string(sx) + "_" + std::to_string(i));
      wide_load(o, nm);
      o << " }\n";
    }
    o << ind << "}\n";
  };
  const std::string t_first = "(i64)blockIdx.x * " + std::to_string(kWaves) + " + wv";
  const std::string t_stride = "(i64)gridDim.x * " + std::to_string(kWaves);
  if (carry) {
    for (int j : ywords0) o << "  T yn" << j << " = 0.0f;\n";
    for (int sx : used_x0) {
      o << "  T";
      for (int i = 0; i < 2 * P.irx[sx].l + 1; ++i) o << (i ? ", " : " ") << "xn" << sx << "_" << i << " = 0.0f";
      o << ";\n";
    }
    o << "  if (" << t_first << " < ntile) {\n";
    emit_tile_loads(t_first.c_str(), "    ");
    o << "  }\n";
  }
  o << "  for (i64 t_ = " << t_first << "; t_ < ntile; t_ += " << t_stride << ") {\n";
  o << "    const i64 b0 = t_ * " << kTile << ";\n";
  o << "    const int rows = (int)((B - b0) < " << kTile << " ? (B - b0) : " << kTile << ");\n";
  if (carry) o << "    const i64 tn_ = t_ + " << t_stride << " < ntile ? t_ + " << t_stride << " : t_;\n";
  if (staged) {
  // stage the x tile: the 16 rows are one contiguous block in memory; all of a lane's loads are
  // issued before the first LDS write (a load -> store loop would pay the memory latency per
  // iteration); LDS pitch is odd so that the 16 samples of an MFMA row group hit different banks
  o << "    __builtin_amdgcn_wave_barrier();\n";
  if (DX % 4 == 0) {
    const int nv = kTile * DX / 4;             // float4 per tile
    const int per = (nv + 63) / 64;
    o << "    { f4 v_[" << per << "];\n";
    o << "      #pragma unroll\n";
    o << "      for (int it = 0; it < " << per << "; ++it) { const int i4 = it * 64 + lane; const int r_ = i4 / " << DX / 4
      << "; v_[it] = (i4 < " << nv << " && r_ < rows) ? *(const f4*)(x + b0 * " << DX << " + 4 * (i64)i4) : (f4){0.0f, 0.0f, 0.0f, 0.0f}; }\n";
    o << "      #pragma unroll\n";
    o << "      for (int it = 0; it < " << per << "; ++it) { const int i4 = it * 64 + lane; if (i4 < " << nv << ") { const int r_ = i4 / " << DX / 4
      << ", c_ = 4 * (i4 - r_ * " << DX / 4 << "); T* d_ = tile + r_ * " << XS
      << " + c_; d_[0] = v_[it][0]; d_[1] = v_[it][1]; d_[2] = v_[it][2]; d_[3] = v_[it][3]; } }\n";
    o << "    }\n";
  } else {
    o << "    for (int i = lane; i < " << kTile * DX << "; i += 64) { const int r_ = i / " << DX << ", c_ = i - r_ * " << DX
      << "; tile[r_ * " << XS << " + c_] = r_ < rows ? x[b0 * " << DX << " + i] : 0.0f; }\n";
  }
  o << "    __builtin_amdgcn_wave_barrier();\n";
  }
  // y of the lane's sample and the coefficient products
  std::set<int> ywords;
  for (auto& p : P.paths)
    for (auto& n : p.nz) ywords.insert((int)P.offy[p.iy] + n.j);
  o << "    const bool live = s < rows;\n";
  o << "    const T* yb = y + (b0 + (live ? s : 0)) * " << DY << ";\n";
  // rows past the end of the batch read the tile's first row instead (their results are never stored and
  // matrix rows do not mix), so no load needs a branch
  if (carry) {
    for (int j : ywords) o << "    const T y" << j << " = yn" << j << ";\n";
  } else {
    for (int j : ywords) o << "    const T y" << j << " = yb[" << j << "];\n";
  }
  // accumulators
  std::set<int> used_z;
  for (auto& p : P.paths) used_z.insert(p.iz);
  for (int sz : used_z) {
    const Irrep& ir = P.irz[sz];
    for (int k = 0; k < 2 * ir.l + 1; ++k)
      for (int h = 0; h < ir.mul / 16; ++h) o << "    f4 acc" << sz << "_" << k << "_" << h << " = {0.0f, 0.0f, 0.0f, 0.0f};\n";
  }
  // coefficient products, once per tile
  int tcount = 0;
  std::vector<std::vector<std::pair<std::string, bool>>> tref(P.paths.size());
  for (size_t p = 0; p < P.paths.size(); ++p) {
    const PathInfo& pq = P.paths[p];
    std::map<std::pair<long long, int>, std::string> seen;
    for (auto& n : pq.nz) {
      double c = n.v * pq.coeff, a = std::fabs(c);
      auto key = std::make_pair(std::llround(a * 1e13), n.j);
      auto it = seen.find(key);
      if (it == seen.end()) {
        std::string name;
        std::string yv = "y" + std::to_string((int)P.offy[pq.iy] + n.j);
        if (std::fabs(a - 1.0) < 1e-15) {
          name = yv;
        } else {
          name = "t" + std::to_string(tcount++);
          o << "    const T " << name << " = " << yv << " * " << lit(a) << ";\n";
        }
        it = seen.insert({key, name}).first;
      }
      tref[p].push_back({it->second, c < 0});
    }
  }
  if (!staged) o << "    const T* xrow = x + (b0 + (live ? s : 0)) * " << DX << ";\n";
  if (carry) {
    // row of this lane in the next tile: the last channel step prefetches from there
    o << "    const i64 bnx_ = tn_ * " << kTile << "; const int rnx_ = (int)((B - bnx_) < " << kTile << " ? (B - bnx_) : " << kTile << ");\n";
    o << "    const T* xrow_n = x + (bnx_ + (s < rnx_ ? s : 0)) * " << DX << ";\n";
    // y of the next tile: in flight during the whole channel loop
    o << "    { const T* yb_ = y + (bnx_ + (s < rnx_ ? s : 0)) * " << DY << ";";
    for (int j : ywords) o << " yn" << j << " = yb_[" << j << "];";
    o << " }\n";
  }
  if (!staged && !carry) {
    std::set<int> ux;
    for (auto& p : P.paths) ux.insert(p.ix);
    for (int sx : ux) {
      const Irrep& ir = P.irx[sx];
      const int n1 = 2 * ir.l + 1;
      o << "    T";
      for (int i = 0; i < n1; ++i) o << (i ? ", " : " ") << "xn" << sx << "_" << i;
      o << ";\n";
      o << "    { const T* p_ = xrow + " << P.offx[sx] << " + q * " << n1 << ";";
      {
        std::vector<std::string> nm;
        for (int i = 0; i < n1; ++i) nm.push_back("xn" + std::to_string(sx) + "_" + std::to_string(i));
        wide_load(o, nm);
      }
      o << " }\n";
    }
  }
  // channel loop: 4 channels of x per step (one per lane group q)
  o << "    #pragma unroll " << env_int("CGTP_UVW_UNROLL", 4) << "\n";
  o << "    for (int c = 0; c < " << maxmul / 4 << "; ++c) {\n";
  o << "      const int u = 4 * c + q;\n";
  std::set<int> used_x;
  for (auto& p : P.paths) used_x.insert(p.ix);
  if (staged) {
    for (int sx : used_x) {
      const Irrep& ir = P.irx[sx];
      const int n1 = 2 * ir.l + 1;
      o << "      T";
      for (int i = 0; i < n1; ++i) o << (i ? ", " : " ") << "x" << sx << "_" << i << " = 0.0f";
      o << ";\n";
      o << "      " << (ir.mul < maxmul ? "if (4 * c < " + std::to_string(ir.mul) + ") " : std::string()) << "{ const T* p_ = tile + s * " << XS
        << " + " << P.offx[sx] << " + u * " << n1 << ";";
      for (int i = 0; i < n1; ++i) o << " x" << sx << "_" << i << " = p_[" << i << "];";
      o << " }\n";
    }
  } else {
    // operands of this step were loaded one step ahead; issue the loads of the next step now
    for (int sx : used_x) {
      const int n1 = 2 * P.irx[sx].l + 1;
      o << "      const T";
      for (int i = 0; i < n1; ++i) o << (i ? ", " : " ") << "x" << sx << "_" << i << " = xn" << sx << "_" << i;
      o << ";\n";
    }
    if (carry)
      o << "      { const bool last_ = c + 1 >= " << maxmul / 4 << "; const int cn = last_ ? 0 : c + 1; const int un = 4 * cn + q; const T* xr_ = last_ ? xrow_n : xrow;\n";
    else
    o << "      { const int cn = c + 1 < " << maxmul / 4 << " ? c + 1 : c; const int un = 4 * cn + q; const T* xr_ = xrow;\n";
    for (int sx : used_x) {
      const Irrep& ir = P.irx[sx];
      const int n1 = 2 * ir.l + 1;
      // a segment with fewer channels than the longest one re-reads its last channel block in the extra steps
      // (those steps skip its paths), so the address stays inside the row
      o << "        { const int us_ = " << (ir.mul < maxmul ? "(4 * cn < " + std::to_string(ir.mul) + " ? un : " + std::to_string(ir.mul - 4) + " + q)" : std::string("un"))
        << "; const T* p_ = xr_ + " << P.offx[sx] << " + us_ * " << n1 << ";";
      {
        std::vector<std::string> nm;
        for (int i = 0; i < n1; ++i) nm.push_back("xn" + std::to_string(sx) + "_" + std::to_string(i));
        wide_load(o, nm);
      }
      o << " }\n";
    }
    o << "      }\n";
  }
  // the weight operands of the whole step are read from LDS together, ahead of the first product: a read just
  // before its MFMAs leaves the matrix pipe idle for the LDS latency (the wave issues in order)
  // (measured on the 32-channel benchmark plan: 0.101 ms with the reads pinned ahead, 0.109 ms with reads the
  // compiler is free to sink, 0.108 ms with reads at their uses; forming all z' values of a step before its
  // first MFMA, so that the two waves of a SIMD alternate whole phases, gave 0.104-0.107 ms and was dropped)
  const bool w_ahead = env_int("CGTP_UVW_W_AHEAD", 2) != 0;
  if (w_ahead)
    for (size_t p = 0; p < P.paths.size(); ++p) {
      const PathInfo& pq = P.paths[p];
      // a path with fewer channels than the longest segment skips the extra steps; its (unused) reads are clamped
      const std::string uu = pq.mul_x < maxmul ? "(4 * c < " + std::to_string(pq.mul_x) + " ? u : q)" : std::string("u");
      for (int h = 0; h < pq.mul_z / 16; ++h)
        o << "      const T bw" << p << "_" << h << " = lds_w[" << pq.w_off << " + " << uu << " * " << pq.mul_z << " + s + " << 16 * h << "];\n";
    }
  if (w_ahead && env_int("CGTP_UVW_W_AHEAD", 2) >= 2) {
    // an empty asm that reads them keeps the compiler from sinking the reads back to their uses
    std::vector<std::string> all;
    for (size_t p = 0; p < P.paths.size(); ++p)
      for (int h = 0; h < P.paths[p].mul_z / 16; ++h) all.push_back("bw" + std::to_string(p) + "_" + std::to_string(h));
    for (size_t at = 0; at < all.size(); at += 12) {
      o << "      asm volatile(\"\" ::";
      for (size_t t = at; t < all.size() && t < at + 12; ++t) o << (t > at ? ", " : " ") << "\"v\"(" << all[t] << ")";
      o << ");\n";
    }
  }
  for (size_t p = 0; p < P.paths.size(); ++p) {
    const PathInfo& pq = P.paths[p];
    const int n3 = 2 * pq.l3 + 1;
    o << "      " << (pq.mul_x < maxmul ? "if (4 * c < " + std::to_string(pq.mul_x) + ") " : std::string()) << "{ // path " << p << ": l=("
      << pq.l1 << "," << pq.l2 << "," << pq.l3 << ")\n";
    std::vector<bool> started((size_t)n3, false);
    for (size_t n = 0; n < pq.nz.size(); ++n) {
      const Nz& nz = pq.nz[n];
      std::string tt = std::string(tref[p][n].second ? "-" : "") + tref[p][n].first;
      std::string xx = "x" + std::to_string(pq.ix) + "_" + std::to_string(nz.i);
      if (!started[nz.k]) {
        o << "        T q" << nz.k << " = " << tt << " * " << xx << ";\n";
        started[nz.k] = true;
      } else {
        o << "        q" << nz.k << " = FMA(" << tt << ", " << xx << ", q" << nz.k << ");\n";
      }
    }
    o << "        const T* wp_ = lds_w + " << pq.w_off << " + u * " << pq.mul_z << " + s;\n";
    for (int h = 0; h < pq.mul_z / 16; ++h) {
      if (w_ahead) o << "        { const T b_ = bw" << p << "_" << h << ";\n";
      else
      o << "        { const T b_ = wp_[" << 16 * h << "];\n";
      for (int k = 0; k < n3; ++k)
        if (started[k])
          o << "          acc" << pq.iz << "_" << k << "_" << h << " = __builtin_amdgcn_mfma_f32_16x16x4f32(q" << k << ", b_, acc" << pq.iz
            << "_" << k << "_" << h << ", 0, 0, 0);\n";
      o << "        }\n";
    }
    o << "      }\n";
  }
  o << "    }\n";
  if (staged) {
  // z tile through LDS: accumulator register i of lane (s, q) is sample 4q+i, column w = 16h+s
  o << "    __builtin_amdgcn_wave_barrier();\n";
  for (size_t sz = 0; sz < P.irz.size(); ++sz) {
    const Irrep& ir = P.irz[sz];
    const int n3 = 2 * ir.l + 1;
    if (!used_z.count((int)sz)) {
      o << "    for (int i = lane; i < " << kTile * ir.dim() << "; i += 64) tile[(i / " << ir.dim() << ") * " << ZS << " + " << P.offz[sz]
        << " + i % " << ir.dim() << "] = 0.0f;\n";
      continue;
    }
    for (int k = 0; k < n3; ++k)
      for (int h = 0; h < ir.mul / 16; ++h)
        for (int i = 0; i < 4; ++i)
          o << "    tile[(4 * q + " << i << ") * " << ZS << " + " << P.offz[sz] << " + (" << 16 * h << " + s) * " << n3 << " + " << k << "] = acc"
            << sz << "_" << k << "_" << h << "[" << i << "];\n";
  }
  o << "    __builtin_amdgcn_wave_barrier();\n";
  if (DZ % 4 == 0) {
    const int nv = kTile * DZ / 4;
    const int per = (nv + 63) / 64;
    o << "    #pragma unroll\n";
    o << "    for (int it = 0; it < " << per << "; ++it) { const int i4 = it * 64 + lane; const int r_ = i4 / " << DZ / 4
      << "; if (i4 < " << nv << " && r_ < rows) { const int c_ = 4 * (i4 - r_ * " << DZ / 4 << "); const T* s_ = tile + r_ * " << ZS
      << " + c_; f4 v_ = {s_[0], s_[1], s_[2], s_[3]}; *(f4*)(z + b0 * " << DZ << " + 4 * (i64)i4) = v_; } }\n";
  } else {
    o << "    for (int i = lane; i < rows * " << DZ << "; i += 64) { const int r_ = i / " << DZ << ", c_ = i - r_ * " << DZ << "; z[b0 * " << DZ
      << " + i] = tile[r_ * " << ZS << " + c_]; }\n";
  }
  } else {
    // accumulator register i of lane (s, q) is sample 4q+i, column w = 16h+s: scattered 4-byte stores that
    // the L2 merges into full lines (z is 1 KB per sample)
    for (size_t sz = 0; sz < P.irz.size(); ++sz) {
      const Irrep& ir = P.irz[sz];
      const int n3 = 2 * ir.l + 1;
      if (!used_z.count((int)sz)) {
        o << "    for (int i = lane; i < rows * " << ir.dim() << "; i += 64) z[(b0 + i / " << ir.dim() << ") * " << DZ << " + " << P.offz[sz]
          << " + i % " << ir.dim() << "] = 0.0f;\n";
        continue;
      }
      // the 2l+1 components of one (sample, channel) are adjacent in memory: one wide store each
      for (int i = 0; i < 4; ++i) {
        o << "    if (4 * q + " << i << " < rows) { T* p_ = z + (b0 + 4 * q + " << i << ") * " << DZ << " + " << P.offz[sz] << " + s * " << n3 << ";\n";
        for (int h = 0; h < ir.mul / 16; ++h) {
          int k = 0;
          static const char* comp[4] = {"x", "y", "z", "w"};
          while (k < n3) {
            const int w = n3 - k >= 4 ? 4 : (n3 - k >= 2 ? 2 : 1);
            if (w == 1) {
              o << "      p_[" << 16 * h * n3 + k << "] = acc" << sz << "_" << k << "_" << h << "[" << i << "];\n";
            } else {
              o << "      { u" << w << " v_;";
              for (int c = 0; c < w; ++c) o << " v_." << comp[c] << " = acc" << sz << "_" << k + c << "_" << h << "[" << i << "];";
              o << " *(u" << w << "*)(p_ + " << 16 * h * n3 + k << ") = v_; }\n";
            }
            k += w;
          }
        }
        o << "    }\n";
      }
    }
  }
  o << "  }\n}\n";
  K.source = o.str();
}


// ---------------------------------------------------------------------------------------------
// Backward of the shared-weight uvw product (paper Alg. 3, the general dense-W case):
//   G'[s,u,k] = sum_w W_p[u,w] gz[s,w,k]          GEMM over w on the matrix cores
//   gx[s,u,i] += sum C y[j] G'[s,u,k],  gy[s,j] += sum_u sum C x[u,i] G'[s,u,k]     (VALU, unrolled nonzeros)
//   gW_p[u,w]  = sum_s sum_k z'_p[s,u,k] gz[s,w,k]  GEMM over (s,k) on the matrix cores, summed over the batch
// A wave owns tiles of 16 samples.  The output layout of the first GEMM (lane (c,q): samples 4q..4q+3,
// channel u = 16h+c) is the lane map of the VALU part, and z' computed there is the A operand of the second
// GEMM as it stands.  gW accumulates in registers over all tiles of the wave; per-wave partial sums are
// written once and added in a fixed order by a second kernel (deterministic, no atomics).
void emit_uvw_backward(const Plan& P, Kernel& K, Kernel& Kred) {
  if (P.dtype != CGTP_F32) throw std::runtime_error("uvw plans are implemented in fp32 only");
  for (auto& q : P.paths)
    if (q.mul_x % 16 || q.mul_z % 16) throw std::runtime_error("uvw backward: mul_x and mul_z must be multiples of 16");
  const int DX = (int)P.dim_x(), DY = (int)P.dim_y(), DZ = (int)P.dim_z();
  const int ZS = odd_pitch(DZ);
  std::vector<int64_t> wp(P.paths.size() + 1, 0);  // padded LDS offsets: path p is [mul_x][mul_z + 1]
  for (size_t p = 0; p < P.paths.size(); ++p) wp[p + 1] = wp[p] + (int64_t)P.paths[p].mul_x * (P.paths[p].mul_z + 1);
  const int YS = odd_pitch(DY);
  const int64_t lds_bytes = 4 * (wp.back() + (int64_t)kWaves * kTile * (ZS + YS));
  if (lds_bytes > 160 * 1024) throw std::runtime_error("uvw backward: weights + tiles exceed the 160 KB of LDS");
  K.wg = 64 * kWaves;
  K.name = "cgtp_tp_bwd_uvw";
  std::ostringstream o;
  o << "typedef float T;\ntypedef long long i64;\n";
  o << "typedef float f4 __attribute__((ext_vector_type(4)));\n";
  o << "#define FMA(a, b, c) __builtin_fmaf((a), (b), (c))\n";
  o << "#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_16x16x4f32((a), (b), (c), 0, 0, 0)\n";
  o << "extern \"C\" __global__ void __launch_bounds__(" << K.wg << ") " << K.name
    << "(const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, const T* __restrict__ gz,\n"
       "   T* __restrict__ gx, T* __restrict__ gy, T* __restrict__ gwpart, i64 B)\n{\n";
  o << "  __shared__ T lds_w[" << wp.back() << "];\n";
  o << "  __shared__ T lds_g[" << kWaves << "][" << kTile * ZS << "];\n";
  o << "  __shared__ T lds_y[" << kWaves << "][" << kTile * YS << "];\n";
  for (size_t p = 0; p < P.paths.size(); ++p) {
    const PathInfo& pq = P.paths[p];
    o << "  for (int i = threadIdx.x; i < " << pq.mul_x * pq.mul_z << "; i += " << K.wg << ") lds_w[" << wp[p] << " + (i / " << pq.mul_z
      << ") * " << pq.mul_z + 1 << " + i % " << pq.mul_z << "] = W[" << pq.w_off << " + i];\n";
  }
  o << "  __syncthreads();\n";
  o << "  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;\n";
  o << "  const int s = lane & 15, q = lane >> 4;\n";
  o << "  T* tile = lds_g[wv];\n";
  o << "  T* ytile = lds_y[wv];\n";
  // gW partial sums: every wave owns a private slice of the workspace, laid out [block][lane][4] (block =
  // (path, h, h2)), and adds the 16x16 block results of each tile to it with plain loads and stores.
  // (Keeping all blocks in registers across tiles costs 176 accumulators and drives the rest to scratch.)
  std::vector<int> blk(P.paths.size() + 1, 0);
  for (size_t p = 0; p < P.paths.size(); ++p) blk[p + 1] = blk[p] + (P.paths[p].mul_x / 16) * (P.paths[p].mul_z / 16);
  o << "  const i64 gwave = (i64)blockIdx.x * " << kWaves << " + wv;\n";
  o << "  f4* part = (f4*)gwpart + gwave * " << blk.back() * 64 << " + lane;\n";
  o << "  for (int b_ = 0; b_ < " << blk.back() << "; ++b_) part[b_ * 64] = (f4){0.0f, 0.0f, 0.0f, 0.0f};\n";
  std::set<int> used_x, ywords;
  for (auto& p : P.paths) {
    used_x.insert(p.ix);
    for (auto& n : p.nz) ywords.insert((int)P.offy[p.iy] + n.j);
  }
  o << "  const i64 ntile = (B + " << kTile - 1 << ") / " << kTile << ";\n";
  o << "  #pragma unroll 1\n";
  o << "  for (i64 t_ = gwave; t_ < ntile; t_ += (i64)gridDim.x * " << kWaves << ") {\n";
  o << "    const i64 b0 = t_ * " << kTile << ";\n";
  o << "    const int rows = (int)((B - b0) < " << kTile << " ? (B - b0) : " << kTile << ");\n";
  // stage gz tile
  o << "    __builtin_amdgcn_wave_barrier();\n";
  if (DZ % 4 == 0) {
    const int nv = kTile * DZ / 4, per = (nv + 63) / 64;
    o << "    { f4 v_[" << per << "];\n      #pragma unroll\n";
    o << "      for (int it = 0; it < " << per << "; ++it) { const int i4 = it * 64 + lane; const int r_ = i4 / " << DZ / 4
      << "; v_[it] = (i4 < " << nv << " && r_ < rows) ? *(const f4*)(gz + b0 * " << DZ << " + 4 * (i64)i4) : (f4){0.0f, 0.0f, 0.0f, 0.0f}; }\n";
    o << "      #pragma unroll\n";
    o << "      for (int it = 0; it < " << per << "; ++it) { const int i4 = it * 64 + lane; if (i4 < " << nv << ") { const int r_ = i4 / " << DZ / 4
      << ", c_ = 4 * (i4 - r_ * " << DZ / 4 << "); T* d_ = tile + r_ * " << ZS << " + c_; d_[0] = v_[it][0]; d_[1] = v_[it][1]; d_[2] = v_[it][2]; d_[3] = v_[it][3]; } }\n";
    o << "    }\n";
  } else {
    o << "    for (int i = lane; i < " << kTile * DZ << "; i += 64) { const int r_ = i / " << DZ << ", c_ = i - r_ * " << DZ
      << "; tile[r_ * " << ZS << " + c_] = r_ < rows ? gz[b0 * " << DZ << " + i] : 0.0f; }\n";
  }
  // y of the 16 samples goes to LDS too (re-read per path: 36 registers less than keeping it)
  o << "    for (int i = lane; i < " << kTile * DY << "; i += 64) { const int r_ = i / " << DY << ", c_ = i - r_ * " << DY
    << "; ytile[r_ * " << YS << " + c_] = r_ < rows ? y[b0 * " << DY << " + i] : 0.0f; }\n";
  o << "    __builtin_amdgcn_wave_barrier();\n";
  // per-lane samples 4q+i: y, liveness, accumulators
  for (int i = 0; i < 4; ++i) {
    o << "    const bool live" << i << " = 4 * q + " << i << " < rows;\n";
    o << "    const i64 row" << i << " = b0 + (live" << i << " ? 4 * q + " << i << " : 0);\n";
    for (int j : ywords) o << "    T gy" << i << "_" << j << " = 0.0f;\n";
  }
  auto store_gx_seg = [&](int sx) {
    const Irrep& ir = P.irx[sx];
    const int n1 = 2 * ir.l + 1;
    for (int i = 0; i < 4; ++i) {
      o << "    if (live" << i << ") { T* p_ = gx + row" << i << " * " << DX << " + " << P.offx[sx] << " + s * " << n1 << ";\n";
      for (int h = 0; h < ir.mul / 16; ++h)
        for (int c = 0; c < n1; ++c) o << "      p_[" << 16 * h * n1 + c << "] = gx" << sx << "_" << h << "_" << i << "_" << c << ";\n";
      o << "    }\n";
    }
    o << "    }\n";   // closes the scope opened at the first path of the segment
  };
  for (size_t p = 0; p < P.paths.size(); ++p) {
    const PathInfo& pq = P.paths[p];
    const int n1 = 2 * pq.l1 + 1, n3 = 2 * pq.l3 + 1;
    const int HX = pq.mul_x / 16, HZ = pq.mul_z / 16;
    if (p == 0 || P.paths[p - 1].ix != pq.ix) {
      o << "    { // x segment " << pq.ix << "\n";
      const Irrep& ir = P.irx[pq.ix];
      for (int h = 0; h < ir.mul / 16; ++h)
        for (int i = 0; i < 4; ++i)
          for (int c = 0; c < 2 * ir.l + 1; ++c) o << "    T gx" << pq.ix << "_" << h << "_" << i << "_" << c << " = 0.0f;\n";
      // x of the lane's (sample, channel) pairs for this segment: loaded once, all loads in flight together
      // (per-path loads would each expose a full memory latency: one wave per SIMD has nothing else to run)
      for (int i = 0; i < 4; ++i)
        for (int h = 0; h < ir.mul / 16; ++h) {
          o << "    const T* xp" << i << "_" << h << " = x + row" << i << " * " << DX << " + " << P.offx[pq.ix] << " + (" << 16 * h << " + s) * " << n1 << ";\n";
          for (int c = 0; c < n1; ++c)
            o << "    const T xv" << i << "_" << h << "_" << c << " = live" << i << " ? xp" << i << "_" << h << "[" << c << "] : 0.0f;\n";
        }
    }
    o << "    { // path " << p << ": l=(" << pq.l1 << "," << pq.l2 << "," << pq.l3 << ")\n";
    for (int k = 0; k < n3; ++k)
      for (int h = 0; h < HX; ++h) o << "      f4 G" << k << "_" << h << " = {0.0f, 0.0f, 0.0f, 0.0f};\n";
    for (int h = 0; h < HX; ++h)
      for (int h2 = 0; h2 < HZ; ++h2) {
        o << "      f4 aw" << p << "_" << h << "_" << h2 << " = {0.0f, 0.0f, 0.0f, 0.0f};\n";
        o << "      const f4 pw" << h << "_" << h2 << " = part[" << (blk[p] + h * HZ + h2) * 64 << "];\n";
      }
    o << "      #pragma unroll\n";
    o << "      for (int st = 0; st < " << pq.mul_z / 4 << "; ++st) {\n";
    o << "        const T* a_ = tile + s * " << ZS << " + " << P.offz[pq.iz] << " + (4 * st + q) * " << n3 << ";\n";
    o << "        const T* b_ = lds_w + " << wp[p] << " + s * " << pq.mul_z + 1 << " + 4 * st + q;\n";
    for (int h = 0; h < HX; ++h) o << "        const T bv" << h << " = b_[" << 16 * h * (pq.mul_z + 1) << "];\n";
    for (int k = 0; k < n3; ++k) {
      o << "        { const T av = a_[" << k << "];";
      for (int h = 0; h < HX; ++h) o << " G" << k << "_" << h << " = MFMA(av, bv" << h << ", G" << k << "_" << h << ");";
      o << " }\n";
    }
    o << "      }\n";
    o << "      __builtin_amdgcn_sched_barrier(0);\n";
    // VALU part per sample i and channel block h
    // group nonzeros for gy
    std::map<std::pair<int, long long>, std::vector<size_t>> groups;
    for (size_t n = 0; n < pq.nz.size(); ++n)
      groups[{pq.nz[n].j, std::llround(std::fabs(pq.nz[n].v * pq.coeff) * 1e13)}].push_back(n);
    for (int i = 0; i < 4; ++i) {
      o << "      { // sample 4q+" << i << "\n";
      std::map<std::pair<long long, int>, std::string> seen;
      std::vector<std::pair<std::string, bool>> tr;
      std::set<int> seen_y;
      int tc = 0;
      for (auto& n : pq.nz) {
        double c = n.v * pq.coeff, a = std::fabs(c);
        auto key = std::make_pair(std::llround(a * 1e13), n.j);
        auto it = seen.find(key);
        if (it == seen.end()) {
          // y passes through an empty asm so that products with equal literals are not merged across
          // paths (merged, the products of all four samples of the lane stay live through the whole tile)
          std::string yv = "yo" + std::to_string(n.j);
          if (!seen_y.count(n.j)) {
            if (seen_y.empty())   // opaque pointer: the loads are redone here instead of being kept from an earlier path
              o << "        const T* yp_ = ytile + (4 * q + " << i << ") * " << YS << " + " << P.offy[pq.iy] << "; asm volatile(\"\" : \"+v\"(yp_));\n";
            o << "        const T " << yv << " = yp_[" << n.j << "];\n";
            seen_y.insert(n.j);
          }
          std::string name = yv;
          if (std::fabs(a - 1.0) >= 1e-15) {
            name = "t" + std::to_string(tc++);
            o << "        const T " << name << " = " << yv << " * " << lit(a) << ";\n";
          }
          it = seen.insert({key, name}).first;
        }
        tr.push_back({it->second, c < 0});
      }
      for (int h = 0; h < HX; ++h) {
        o << "        {\n";
        for (int c = 0; c < n1; ++c) o << "          const T xv" << c << " = xv" << i << "_" << h << "_" << c << ";\n";
        std::vector<bool> started((size_t)n3, false);
        for (size_t n = 0; n < pq.nz.size(); ++n) {
          const Nz& nz = pq.nz[n];
          std::string tt = std::string(tr[n].second ? "-" : "") + tr[n].first;
          std::string g = "G" + std::to_string(nz.k) + "_" + std::to_string(h) + "[" + std::to_string(i) + "]";
          std::string gxn = "gx" + std::to_string(pq.ix) + "_" + std::to_string(h) + "_" + std::to_string(i) + "_" + std::to_string(nz.i);
          o << "          " << gxn << " = FMA(" << tt << ", " << g << ", " << gxn << ");\n";
          if (!started[nz.k]) {
            o << "          T zq" << nz.k << " = " << tt << " * xv" << nz.i << ";\n";
            started[nz.k] = true;
          } else {
            o << "          zq" << nz.k << " = FMA(" << tt << ", xv" << nz.i << ", zq" << nz.k << ");\n";
          }
        }
        int gi = 0;
        for (auto& kv : groups) {
          std::string sn = "sg" + std::to_string(gi++);
          bool first = true;
          for (size_t n : kv.second) {
            const Nz& nz = pq.nz[n];
            bool neg = nz.v * pq.coeff < 0;
            std::string xx = std::string(neg ? "-" : "") + "xv" + std::to_string(nz.i);
            std::string g = "G" + std::to_string(nz.k) + "_" + std::to_string(h) + "[" + std::to_string(i) + "]";
            if (first) o << "          T " << sn << " = " << xx << " * " << g << ";\n";
            else o << "          " << sn << " = FMA(" << xx << ", " << g << ", " << sn << ");\n";
            first = false;
          }
          std::string gyn = "gy" + std::to_string(i) + "_" + std::to_string((int)P.offy[pq.iy] + kv.first.first);
          o << "          " << gyn << " = FMA(" << sn << ", " << lit(std::fabs(pq.nz[kv.second[0]].v * pq.coeff)) << ", " << gyn << ");\n";
        }
        // gW: A = z' (row u = 16h+s, inner index q <-> sample 4q+i), B = gz of the same samples
        for (int k = 0; k < n3; ++k) {
          if (!started[k]) continue;
          o << "          { const T* g_ = tile + (4 * q + " << i << ") * " << ZS << " + " << P.offz[pq.iz] << " + s * " << n3 << " + " << k << ";\n";
          for (int h2 = 0; h2 < HZ; ++h2)
            o << "            aw" << p << "_" << h << "_" << h2 << " = MFMA(zq" << k << ", g_[" << 16 * h2 * n3 << "], aw" << p << "_" << h << "_" << h2 << ");\n";
          o << "          }\n";
        }
        o << "        }\n";
        // the accumulators are only read at the end of the tile: pin them so that their updates (and all the
        // operands those need) are not postponed until then
        {
          std::vector<std::string> pins;
          for (auto& kv : groups) pins.push_back("gy" + std::to_string(i) + "_" + std::to_string((int)P.offy[pq.iy] + kv.first.first));
          for (int c = 0; c < n1; ++c) pins.push_back("gx" + std::to_string(pq.ix) + "_" + std::to_string(h) + "_" + std::to_string(i) + "_" + std::to_string(c));
          std::sort(pins.begin(), pins.end());
          pins.erase(std::unique(pins.begin(), pins.end()), pins.end());
          for (size_t at = 0; at < pins.size(); at += 12) {
            o << "        asm volatile(\"\" :";
            for (size_t t = at; t < pins.size() && t < at + 12; ++t) o << (t > at ? ", " : " ") << "\"+v\"(" << pins[t] << ")";
            o << ");\n";
          }
        }
        o << "        __builtin_amdgcn_sched_barrier(0);\n";
      }
      o << "      }\n";
    }
    for (int h = 0; h < HX; ++h)
      for (int h2 = 0; h2 < HZ; ++h2)
        o << "      part[" << (blk[p] + h * HZ + h2) * 64 << "] = pw" << h << "_" << h2 << " + aw" << p << "_" << h << "_" << h2 << ";\n";
    o << "    }\n";
    // x-segment finished (paths are sorted by x segment): its gx rows leave the registers now
    if (p + 1 == P.paths.size() || P.paths[p + 1].ix != pq.ix) store_gx_seg(pq.ix);
  }
  // store gx
  for (size_t sx = 0; sx < P.irx.size(); ++sx) {
    const Irrep& ir = P.irx[sx];
    const int n1 = 2 * ir.l + 1;
    if (!used_x.count((int)sx)) {
      o << "    for (int i = lane; i < rows * " << ir.dim() << "; i += 64) gx[(b0 + i / " << ir.dim() << ") * " << DX << " + " << P.offx[sx]
        << " + i % " << ir.dim() << "] = 0.0f;\n";
      continue;
    }
    (void)n1;
  }
  // gy: sum over the 16 lanes that share q (channels), every lane stores the same total
  for (int i = 0; i < 4; ++i) {
    for (int j = 0; j < DY; ++j) {
      if (!ywords.count(j)) {
        o << "    if (live" << i << ") gy[row" << i << " * " << DY << " + " << j << "] = 0.0f;\n";
        continue;
      }
      std::string v = "gy" + std::to_string(i) + "_" + std::to_string(j);
      for (int off = 8; off >= 1; off >>= 1) o << "    " << v << " += __shfl_xor(" << v << ", " << off << ", 64);\n";
      o << "    if (live" << i << ") gy[row" << i << " * " << DY << " + " << j << "] = " << v << ";\n";
    }
  }
  o << "    __builtin_amdgcn_wave_barrier();\n";
  o << "  }\n";
  o << "}\n";
  K.source = o.str();

  Kred.wg = 256;
  Kred.name = "cgtp_uvw_gw_reduce";
  std::ostringstream r;
  r << "typedef float T;\ntypedef long long i64;\n";
  r << "extern \"C\" __global__ void __launch_bounds__(256) cgtp_uvw_gw_reduce(const T* __restrict__ part, T* __restrict__ gW, i64 nparts, i64 n)\n{\n"
       "  // 64 outputs per workgroup; the four waves each add every fourth partial, then the four sums are\n"
       "  // combined in a fixed order through LDS\n"
       "  __shared__ T red[4][64];\n"
       "  const int c = threadIdx.x & 63, rr = threadIdx.x >> 6;\n"
       "  const i64 i = (i64)blockIdx.x * 64 + c;\n"
       "  T acc = 0.0f;\n"
       "  if (i < n) {\n"
       "  int woff = 0, mz = 1, hz = 1, b0 = 0;\n";
  for (size_t p = 0; p < P.paths.size(); ++p)
    r << "  if (i >= " << P.paths[p].w_off << ") { woff = " << P.paths[p].w_off << "; mz = " << P.paths[p].mul_z << "; hz = " << P.paths[p].mul_z / 16
      << "; b0 = " << blk[p] << "; }\n";
  r << "  const int u = (int)(i - woff) / mz, w = (int)(i - woff) % mz;\n"
       "  // accumulator register ii of lane (s, q) of block (h, h2) is row u = 16h + 4q + ii, column w = 16h2 + s\n"
       "  const i64 src = ((i64)(b0 + (u / 16) * hz + w / 16) * 64 + ((u % 16) / 4) * 16 + w % 16) * 4 + u % 4;\n"
       "  const i64 stride = " << (int64_t)blk.back() * 256 << ";\n"
       "  T a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;\n"
       "  i64 v = rr;\n"
       "  for (; v + 12 < nparts; v += 16) { a0 += part[v * stride + src]; a1 += part[(v + 4) * stride + src]; a2 += part[(v + 8) * stride + src]; a3 += part[(v + 12) * stride + src]; }\n"
       "  for (; v < nparts; v += 4) a0 += part[v * stride + src];\n"
       "  acc = (a0 + a1) + (a2 + a3);\n"
       "  }\n"
       "  red[rr][c] = acc;\n"
       "  __syncthreads();\n"
       "  if (rr == 0 && i < n) gW[i] = (red[0][c] + red[1][c]) + (red[2][c] + red[3][c]);\n}\n";
  Kred.source = r.str();
}

}  // namespace cgtp
