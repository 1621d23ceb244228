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
//     registers over the whole channel loop and are stored from there.
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
  // The tiles are dealt to the waves round-robin.  The last, incomplete round would leave most SIMDs idle while a
  // few finish a whole tile (B = 100 000: 6 250 tiles over 2 048 waves, 7 tile times on the busiest SIMD against
  // 6.1 on average), so its tiles are worked on by a whole workgroup each: the four waves split the (output
  // segment, k) accumulators of the tile between them (emit_tail below).
  const bool tail = !staged && env_int("CGTP_UVW_TAIL", 1) != 0;
  if (tail)
    o << "  i64 nmain = ntile - ntile % ((i64)gridDim.x * " << kWaves << ");\n"
         "  if (ntile - nmain > (i64)gridDim.x) nmain = ntile;   // more tail tiles than workgroups: whole tiles are cheaper\n";
  else o << "  const i64 nmain = ntile;\n";
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
    o << "  if (" << t_first << " < nmain) {\n";
    emit_tile_loads(t_first.c_str(), "    ");
    o << "  }\n";
  }
  if (env_int("CGTP_UVW_W_AHEAD", 3) == 3)   // weight operands of channel step 0 (the same for every tile)
    for (size_t p = 0; p < P.paths.size(); ++p)
      for (int h = 0; h < P.paths[p].mul_z / 16; ++h)
        o << "  T bwn" << p << "_" << h << " = lds_w[" << P.paths[p].w_off << " + q * " << P.paths[p].mul_z << " + s + " << 16 * h << "];\n";
  o << "  for (i64 t_ = " << t_first << "; t_ < nmain; t_ += " << t_stride << ") {\n";
  o << "    const i64 b0 = t_ * " << kTile << ";\n";
  o << "    const int rows = (int)((B - b0) < " << kTile << " ? (B - b0) : " << kTile << ");\n";
  if (carry) o << "    const i64 tn_ = t_ + " << t_stride << " < nmain ? t_ + " << t_stride << " : t_;\n";
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
  // unrolled twice: with four copies the kernel needs 48 bytes of private memory at its 256-register budget (the
  // time is the same within the run-to-run spread: 0.096-0.100 ms on the 32-channel benchmark plan either way)
  o << "    #pragma unroll " << env_int("CGTP_UVW_UNROLL", 2) << "\n";
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
  // (measured on the 32-channel benchmark plan: 0.098 ms with the operands of step c+1 requested during step c
  // behind a scheduling fence and never waited for early (mode 3, the default), 0.102 ms with the reads of a step
  // pinned at its start by an empty asm that waits for them (mode 2), 0.109 ms with reads the compiler is free to
  // sink (mode 1), 0.108 ms with reads at their uses (mode 0); forming all z' values of a step before its first
  // MFMA, so that the two waves of a SIMD alternate whole phases, gave 0.104-0.107 ms and was dropped)
  const bool w_ahead = env_int("CGTP_UVW_W_AHEAD", 3) != 0;
  const bool w_carried = env_int("CGTP_UVW_W_AHEAD", 3) == 3;   // operands of step c+1 requested during step c, no wait
  if (w_carried) {
    const int steps = maxmul / 4;
    for (size_t p = 0; p < P.paths.size(); ++p)
      for (int h = 0; h < P.paths[p].mul_z / 16; ++h) o << "      const T bw" << p << "_" << h << " = bwn" << p << "_" << h << ";\n";
    o << "      { const int cn_ = c + 1 < " << steps << " ? c + 1 : 0; const int un_ = 4 * cn_ + q;\n";
    for (size_t p = 0; p < P.paths.size(); ++p) {
      const PathInfo& pq = P.paths[p];
      const std::string uu = pq.mul_x < maxmul ? "(4 * cn_ < " + std::to_string(pq.mul_x) + " ? un_ : q)" : std::string("un_");
      for (int h = 0; h < pq.mul_z / 16; ++h)
        o << "        bwn" << p << "_" << h << " = lds_w[" << pq.w_off << " + " << uu << " * " << pq.mul_z << " + s + " << 16 * h << "];\n";
    }
    o << "      }\n      __builtin_amdgcn_sched_barrier(0);\n";
  } else
  if (w_ahead)
    for (size_t p = 0; p < P.paths.size(); ++p) {
      const PathInfo& pq = P.paths[p];
      // a path with fewer channels than the longest segment skips the extra steps; its (unused) reads are clamped
      const std::string uu = pq.mul_x < maxmul ? "(4 * c < " + std::to_string(pq.mul_x) + " ? u : q)" : std::string("u");
      for (int h = 0; h < pq.mul_z / 16; ++h)
        o << "      const T bw" << p << "_" << h << " = lds_w[" << pq.w_off << " + " << uu << " * " << pq.mul_z << " + s + " << 16 * h << "];\n";
    }
  if (w_ahead && env_int("CGTP_UVW_W_AHEAD", 3) == 2) {
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
  o << "  }\n";
  if (tail) {
    // units of work: one (output segment, k) pair = the accumulators of that component for both halves of w; its
    // cost is one matrix instruction per path into the segment, half of w and channel step.  Longest first onto the
    // least loaded of the four waves.
    struct Unit { int sz, k, cost; };
    std::vector<Unit> units;
    for (int sz : used_z) {
      int np = 0;
      for (auto& pq : P.paths) np += pq.iz == sz;
      for (int k = 0; k < 2 * P.irz[sz].l + 1; ++k) units.push_back({sz, k, np * (P.irz[sz].mul / 16)});
    }
    std::stable_sort(units.begin(), units.end(), [](const Unit& a, const Unit& b) { return a.cost > b.cost; });
    std::vector<std::vector<Unit>> role(kWaves);
    std::vector<int> load(kWaves, 0);
    for (auto& un : units) {
      const int r = (int)(std::min_element(load.begin(), load.end()) - load.begin());
      role[r].push_back(un);
      load[r] += un.cost;
    }
    o << "  const int wvu = __builtin_amdgcn_readfirstlane(wv);\n";
    o << "  for (i64 tt_ = nmain + blockIdx.x; tt_ < ntile; tt_ += gridDim.x) {\n";
    o << "    const i64 b0 = tt_ * " << kTile << ";\n";
    o << "    const int rows = (int)((B - b0) < " << kTile << " ? (B - b0) : " << kTile << ");\n";
    o << "    const i64 row_ = b0 + (s < rows ? s : 0);\n";
    o << "    const T* yb = y + row_ * " << DY << ";\n";
    o << "    const T* xrow = x + row_ * " << DX << ";\n";
    for (int r = 0; r < kWaves; ++r) {
      o << "    " << (r ? "else " : "") << "if (wvu == " << r << ") {\n";
      std::set<std::pair<int, int>> mine;
      for (auto& un : role[r]) mine.insert({un.sz, un.k});
      std::vector<size_t> rp;   // paths with a component in this role
      for (size_t p = 0; p < P.paths.size(); ++p)
        for (int k = 0; k < 2 * P.paths[p].l3 + 1; ++k)
          if (mine.count({P.paths[p].iz, k})) { rp.push_back(p); break; }
      std::set<int> yw, xs;
      for (size_t p : rp) {
        xs.insert(P.paths[p].ix);
        for (auto& n : P.paths[p].nz)
          if (mine.count({P.paths[p].iz, n.k})) yw.insert((int)P.offy[P.paths[p].iy] + n.j);
      }
      for (int j : yw) o << "      const T y" << j << " = yb[" << j << "];\n";
      for (auto& un : role[r])
        for (int h = 0; h < P.irz[un.sz].mul / 16; ++h) o << "      f4 acc" << un.sz << "_" << un.k << "_" << h << " = {0.0f, 0.0f, 0.0f, 0.0f};\n";
      // coefficient products of the role's nonzeros
      int tc = 0;
      std::vector<std::vector<std::pair<std::string, bool>>> tr(P.paths.size());
      for (size_t p : rp) {
        const PathInfo& pq = P.paths[p];
        std::map<std::pair<long long, int>, std::string> seen;
        for (auto& n : pq.nz) {
          const double c = n.v * pq.coeff, a = std::fabs(c);
          if (!mine.count({pq.iz, n.k})) { tr[p].push_back({"", false}); continue; }
          auto key = std::make_pair(std::llround(a * 1e13), n.j);
          auto it = seen.find(key);
          if (it == seen.end()) {
            const std::string yv = "y" + std::to_string((int)P.offy[pq.iy] + n.j);
            std::string name = yv;
            if (std::fabs(a - 1.0) >= 1e-15) {
              name = "tr" + std::to_string(tc++);
              o << "      const T " << name << " = " << yv << " * " << lit(a) << ";\n";
            }
            it = seen.insert({key, name}).first;
          }
          tr[p].push_back({it->second, c < 0});
        }
      }
      o << "      #pragma unroll 2\n";
      o << "      for (int c = 0; c < " << maxmul / 4 << "; ++c) {\n";
      o << "        const int u = 4 * c + q;\n";
      for (int sx : xs) {
        const Irrep& ir = P.irx[sx];
        const int n1 = 2 * ir.l + 1;
        o << "        T";
        for (int i = 0; i < n1; ++i) o << (i ? ", " : " ") << "x" << sx << "_" << i;
        o << ";\n";
        o << "        { const int us_ = " << (ir.mul < maxmul ? "(4 * c < " + std::to_string(ir.mul) + " ? u : " + std::to_string(ir.mul - 4) + " + q)" : std::string("u"))
          << "; const T* p_ = xrow + " << P.offx[sx] << " + us_ * " << n1 << ";";
        std::vector<std::string> nm;
        for (int i = 0; i < n1; ++i) nm.push_back("x" + std::to_string(sx) + "_" + std::to_string(i));
        wide_load(o, nm);
        o << " }\n";
      }
      for (size_t p : rp) {
        const PathInfo& pq = P.paths[p];
        const int n3 = 2 * pq.l3 + 1;
        o << "        " << (pq.mul_x < maxmul ? "if (4 * c < " + std::to_string(pq.mul_x) + ") " : std::string()) << "{ // path " << p << "\n";
        std::vector<bool> started((size_t)n3, false);
        for (size_t n = 0; n < pq.nz.size(); ++n) {
          const Nz& nz = pq.nz[n];
          if (!mine.count({pq.iz, nz.k})) continue;
          const std::string tt = std::string(tr[p][n].second ? "-" : "") + tr[p][n].first;
          const std::string xx = "x" + std::to_string(pq.ix) + "_" + std::to_string(nz.i);
          if (!started[nz.k]) {
            o << "          T q" << nz.k << " = " << tt << " * " << xx << ";\n";
            started[nz.k] = true;
          } else {
            o << "          q" << nz.k << " = FMA(" << tt << ", " << xx << ", q" << nz.k << ");\n";
          }
        }
        for (int h = 0; h < pq.mul_z / 16; ++h) {
          o << "          { const T b_ = lds_w[" << pq.w_off << " + u * " << pq.mul_z << " + s + " << 16 * h << "];\n";
          for (int k = 0; k < n3; ++k)
            if (started[k])
              o << "            acc" << pq.iz << "_" << k << "_" << h << " = __builtin_amdgcn_mfma_f32_16x16x4f32(q" << k << ", b_, acc" << pq.iz
                << "_" << k << "_" << h << ", 0, 0, 0);\n";
          o << "          }\n";
        }
        o << "        }\n";
      }
      o << "      }\n";
      // accumulator register i of lane (s, q) is sample 4q+i, column w = 16h+s
      for (int i = 0; i < 4; ++i) {
        o << "      if (4 * q + " << i << " < rows) { T* p_ = z + (b0 + 4 * q + " << i << ") * " << DZ << ";\n";
        for (auto& un : role[r]) {
          const int n3 = 2 * P.irz[un.sz].l + 1;
          for (int h = 0; h < P.irz[un.sz].mul / 16; ++h)
            o << "        p_[" << P.offz[un.sz] + (int64_t)16 * h * n3 + un.k << " + s * " << n3 << "] = acc" << un.sz << "_" << un.k << "_" << h << "[" << i << "];\n";
        }
        o << "      }\n";
      }
      if (r == 0)   // output segments that no path reaches
        for (size_t sz = 0; sz < P.irz.size(); ++sz)
          if (!used_z.count((int)sz))
            o << "      for (int i = lane; i < rows * " << P.irz[sz].dim() << "; i += 64) z[(b0 + i / " << P.irz[sz].dim() << ") * " << DZ << " + "
              << P.offz[sz] << " + i % " << P.irz[sz].dim() << "] = 0.0f;\n";
      o << "    }\n";
    }
    o << "  }\n";
  }
  o << "}\n";
  K.source = o.str();
}


// ---------------------------------------------------------------------------------------------
// Backward of the shared-weight uvw product (paper Alg. 3, the general dense-W case):
//   G'[s,u,k] = sum_w W_p[u,w] gz[s,w,k]          GEMM over w on the matrix cores
//   gx[s,u,i] += sum C y[j] G'[s,u,k],  gy[s,j] += sum_u sum C x[u,i] G'[s,u,k]     (VALU, unrolled nonzeros)
//   gW_p[u,w]  = sum_s sum_k z'_p[s,u,k] gz[s,w,k]  GEMM over (s,k) on the matrix cores, summed over the batch
// Tiles are 16 samples.  The output layout of the first GEMM (lane (c,q): samples 4q..4q+3, channel u = 16h+c)
// is the lane map of the VALU part, and z' computed in that layout is the A operand of the second GEMM as it
// stands.  One partial gW per workgroup is written at the end of the kernel; a second kernel adds the partial
// sums in a fixed order (deterministic, no atomics).

namespace {
int pitch4(int64_t d) { return (int)(d + ((4 - d % 32) + 32) % 32); }  // >= d and = 4 mod 32: (row, q) pairs of a wave hit every bank twice

// Per-workgroup partial sums of gW are added by this kernel in a fixed order (deterministic, no atomics).
void emit_gw_reduce(const Plan& P, const std::vector<int>& blk, Kernel& Kred) {
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

}  // namespace

// Two kinds of waves share a workgroup of eight (two waves per SIMD, each within 256 registers) and work in
// rounds of four tiles:
//   waves 0-3 ("tile waves") each own one tile of the round: G' = gz W^T on the matrix cores, then gx and gy on
//     the VALU, per x segment and half of its channels;
//   waves 4-7 ("block waves") each own a fixed share of the 16x16 blocks of gW, cut by (path, half of u) into
//     shares of equal issue time; for each of the four tiles they form z' on the VALU and multiply by the gz
//     values of the tile.  Their accumulators live in registers for the whole kernel.
// What was measured on the 32-channel benchmark plan and shaped the code (the fp32 matrix instructions and the
// VALU do not overlap on this hardware, so the floor is the sum of their issue times, 54 k cycles per round):
//   - every LDS operand is requested one work item ahead, between scheduling fences (a read just before its use
//     leaves the wave idle for the LDS round trip);
//   - gz, y and the first x rows of a tile travel through registers a round ahead, gz split between the tile
//     wave and the block waves with the fewest x registers (staging after the barrier cost 27 k cycles a round);
//   - addresses are a wave-uniform base plus a 32-bit lane offset (64-bit lane addresses were spilled, and each
//     reload waited for every outstanding load);
//   - gy is summed over the 16 channel lanes with DPP row operations (36 x 4 dependent LDS shuffles cost 14 k
//     cycles a tile).
void emit_uvw_backward(const Plan& P, Kernel& K, Kernel& Kred) {
  if (P.dtype != CGTP_F32) throw std::runtime_error("uvw plans are implemented in fp32 only");
  for (auto& q : P.paths)
    if (q.mul_x % 16 || q.mul_z % 16) throw ShapeNotCovered("uvw backward: mul_x and mul_z must be multiples of 16");
  const int DX = (int)P.dim_x(), DY = (int)P.dim_y(), DZ = (int)P.dim_z();
  const int ZS = pitch4(DZ), YS = odd_pitch(DY);
  const int NB = 4;
  std::vector<int64_t> wp(P.paths.size() + 1, 0);
  std::vector<int> wpitch(P.paths.size());
  for (size_t p = 0; p < P.paths.size(); ++p) {
    wpitch[p] = pitch4(P.paths[p].mul_z);
    wp[p + 1] = wp[p] + (int64_t)P.paths[p].mul_x * wpitch[p];
  }
  const int64_t lds_bytes = 4 * (wp.back() + (int64_t)kWaves * kTile * (ZS + YS));
  if (lds_bytes > 160 * 1024) throw ShapeNotCovered("uvw backward: weights + tiles exceed the 160 KB of LDS");
  std::vector<int> blk(P.paths.size() + 1, 0);
  for (size_t p = 0; p < P.paths.size(); ++p) blk[p + 1] = blk[p] + (P.paths[p].mul_x / 16) * (P.paths[p].mul_z / 16);
  // units (path, h) in path order, dealt to the block waves by the midpoint of their cumulative cost
  struct Unit { int p, h; };
  std::vector<std::vector<Unit>> share(NB);
  {
    // issue cycles of a unit per sample: 32 per matrix instruction, 4 per VALU instruction (the fp32 matrix
    // instructions and the VALU do not overlap on this hardware, so both count)
    auto unit_cost = [](const PathInfo& q) {
      std::set<std::pair<long long, int>> tp;
      for (auto& n : q.nz) tp.insert({std::llround(std::fabs(n.v * q.coeff) * 1e13), n.j});
      return 32.0 * (2 * q.l3 + 1) * (q.mul_z / 16) + 4.0 * (double)(q.nz.size() + tp.size());
    };
    double total = 0;
    for (auto& q : P.paths) total += unit_cost(q) * (q.mul_x / 16);
    double cum = 0;
    for (size_t p = 0; p < P.paths.size(); ++p)
      for (int h = 0; h < P.paths[p].mul_x / 16; ++h) {
        const double c = unit_cost(P.paths[p]);
        int v = std::min(NB - 1, (int)((cum + 0.5 * c) / (total / NB)));
        share[v].push_back({(int)p, h});
        cum += c;
      }
  }
  std::set<int> used_x, ywords;
  for (auto& p : P.paths) {
    used_x.insert(p.ix);
    for (auto& n : p.nz) ywords.insert((int)P.offy[p.iy] + n.j);
  }
  K.wg = 64 * (kWaves + NB);
  K.name = "cgtp_tp_bwd_uvw";
  std::ostringstream o;
  o << "typedef float T;\ntypedef long long i64;\n";
  o << "typedef float f4 __attribute__((ext_vector_type(4)));\n";
  o << "typedef float u4 __attribute__((ext_vector_type(4), aligned(4)));\n";
  o << "typedef float u2 __attribute__((ext_vector_type(2), aligned(4)));\n";
  o << "#define FMA(a, b, c) __builtin_fmaf((a), (b), (c))\n";
  o << "#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_16x16x4f32((a), (b), (c), 0, 0, 0)\n";
  // sum over the 16 lanes of a DPP row: quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror
  o << "#define DPP_ADD(v, ctrl) ((v) + __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, (v)), (ctrl), 0xf, 0xf, true)))\n";
  o << "static __device__ __forceinline__ T row_sum(T v) { v = DPP_ADD(v, 0xB1); v = DPP_ADD(v, 0x4E); v = DPP_ADD(v, 0x141); v = DPP_ADD(v, 0x140); return v; }\n";
  o << "extern \"C\" __global__ void __launch_bounds__(" << K.wg << ") " << K.name
    << "(const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, const T* __restrict__ gz,\n"
       "   T* __restrict__ gx, T* __restrict__ gy, T* __restrict__ gwpart, i64 B)\n{\n";
  o << "  __shared__ T lds_w[" << wp.back() << "];\n";
  o << "  __shared__ __attribute__((aligned(16))) T lds_g[" << kWaves << "][" << kTile * ZS << "];\n";
  o << "  __shared__ T lds_y[" << kWaves << "][" << kTile * YS << "];\n";
  {
    // weights -> LDS (padded rows): up to 32 loads of a thread are in flight together
    struct Ld { size_t p; int k; };
    std::vector<Ld> lds;
    for (size_t p = 0; p < P.paths.size(); ++p)
      for (int k = 0; k * K.wg < P.paths[p].mul_x * P.paths[p].mul_z; ++k) lds.push_back({p, k});
    for (size_t at = 0; at < lds.size(); at += 32) {
      o << "  {\n";
      for (size_t t = at; t < lds.size() && t < at + 32; ++t) {
        const PathInfo& pq = P.paths[lds[t].p];
        const int sz = pq.mul_x * pq.mul_z;
        o << "    const int i" << t << " = threadIdx.x + " << lds[t].k * K.wg << "; const T w" << t << " = W[" << pq.w_off << " + (i" << t << " < " << sz
          << " ? i" << t << " : 0)];\n";
      }
      for (size_t t = at; t < lds.size() && t < at + 32; ++t) {
        const PathInfo& pq = P.paths[lds[t].p];
        const int sz = pq.mul_x * pq.mul_z;
        o << "    if (i" << t << " < " << sz << ") lds_w[" << wp[lds[t].p] << " + (i" << t << " / " << pq.mul_z << ") * " << wpitch[lds[t].p] << " + i" << t
          << " % " << pq.mul_z << "] = w" << t << ";\n";
      }
      o << "  }\n";
    }
  }
  o << "  __syncthreads();\n";
  o << "  const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);\n";
  o << "  const int s = lane & 15, q = lane >> 4;\n";
  o << "  const i64 ntile = (B + " << kTile - 1 << ") / " << kTile << ", nround = (ntile + " << kWaves - 1 << ") / " << kWaves << ";\n";

  // ---------------------------------------------------------------- tile waves
  o << "  if (wv < " << kWaves << ") {\n";
  o << "  T* tile = lds_g[wv];\n  T* ytile = lds_y[wv];\n";
  // The gz and y rows of the wave's next tile travel through registers: requested right after the barrier that
  // opens a round, written to LDS after the barrier that closes it (the loads are in flight during the round's
  // arithmetic).  Addresses are clamped into the arrays; rows past the end of the batch are written as zeros.
  const bool vec = DZ % 4 == 0;
  const int nvz = vec ? kTile * DZ / 4 : kTile * DZ, perz = (nvz + 63) / 64, pery = (kTile * DY + 63) / 64;
  o << "  " << (vec ? "f4" : "T") << " pf[" << perz << "];\n  T py[" << pery << "];\n";
  const int half = (perz + 1) / 2;   // the tile wave carries slots [0, half) and y, its partner block wave the rest
  auto prefetch = [&](const std::string& b0expr, const char* ind, int lo, int hi, bool with_y, const std::string& pf = "pf") {
    o << ind << "{ const i64 pb0 = " << b0expr << ";\n";
    o << ind << "  #pragma unroll\n";
    if (vec)
      o << ind << "  for (int it = " << lo << "; it < " << hi << "; ++it) { i64 a_ = pb0 * " << DZ << " + 4 * (i64)(it * 64 + lane); a_ = a_ < B * " << DZ
        << " - 4 ? a_ : B * " << DZ << " - 4; " << pf << "[it] = *(const f4*)(gz + a_); }\n";
    else
      o << ind << "  for (int it = " << lo << "; it < " << hi << "; ++it) { i64 a_ = pb0 * " << DZ << " + it * 64 + lane; a_ = a_ < B * " << DZ
        << " - 1 ? a_ : B * " << DZ << " - 1; " << pf << "[it] = gz[a_]; }\n";
    if (with_y) {
      o << ind << "  #pragma unroll\n";
      o << ind << "  for (int it = 0; it < " << pery << "; ++it) { i64 a_ = pb0 * " << DY << " + it * 64 + lane; a_ = a_ < B * " << DY
        << " - 1 ? a_ : B * " << DY << " - 1; py[it] = y[a_]; }\n";
    }
    o << ind << "}\n";
  };
  // writes the carried slots of tile `tile_` (rows past `rows` as zeros)
  auto lds_write = [&](const char* ind, int lo, int hi, bool with_y, const std::string& pf = "pf", const std::string& tile = "tile") {
    o << ind << "#pragma unroll\n";
    if (vec)
      o << ind << "for (int it = " << lo << "; it < " << hi << "; ++it) { const int i4 = it * 64 + lane; if (i4 < " << nvz << ") { const int r_2 = i4 / " << DZ / 4
        << ", c_ = 4 * (i4 - r_2 * " << DZ / 4 << "); *(f4*)(" << tile << " + r_2 * " << ZS << " + c_) = r_2 < rows ? " << pf << "[it] : (f4){0.0f, 0.0f, 0.0f, 0.0f}; } }\n";
    else
      o << ind << "for (int it = " << lo << "; it < " << hi << "; ++it) { const int i = it * 64 + lane; if (i < " << nvz << ") { const int r_2 = i / " << DZ
        << ", c_ = i - r_2 * " << DZ << "; " << tile << "[r_2 * " << ZS << " + c_] = r_2 < rows ? " << pf << "[it] : 0.0f; } }\n";
    if (with_y) {
      o << ind << "#pragma unroll\n";
      o << ind << "for (int it = 0; it < " << pery << "; ++it) { const int i = it * 64 + lane; if (i < " << kTile * DY << ") { const int r_2 = i / " << DY
        << ", c_ = i - r_2 * " << DY << "; ytile[r_2 * " << YS << " + c_] = r_2 < rows ? py[it] : 0.0f; } }\n";
    }
  };
  prefetch("((i64)blockIdx.x * " + std::to_string(kWaves) + " + wv) * " + std::to_string(kTile), "  ", 0, half, true);
  // blocks (x segment, half of its channels) in path order; the x rows of a block are requested one block ahead
  struct Blk { int sx, h; };
  std::vector<Blk> blocks;
  for (size_t p = 0; p < P.paths.size(); ++p)
    if (p == 0 || P.paths[p - 1].ix != P.paths[p].ix)
      for (int h = 0; h < P.paths[p].mul_x / 16; ++h) blocks.push_back({P.paths[p].ix, h});
  // mode 0: declare and load; 1: declare only; 2: load only (rows of the tile that starts at sample `b0expr`;
  // nothing is loaded for a tile past the end of the batch).  Addresses are a wave-uniform base plus a 32-bit
  // lane offset, rows clamped into the tile.
  auto load_x_a = [&](const Blk& bk, const char* ind, int mode = 0, const std::string& b0expr = "b0") {
    const int n1 = 2 * P.irx[bk.sx].l + 1;
    if (mode != 2)
      for (int i = 0; i < 4; ++i) {
        o << ind << "T";
        for (int c = 0; c < n1; ++c)
          o << (c ? ", " : " ") << "xv" << bk.sx << "_" << bk.h << "_" << i << "_" << c << " = 0.0f";
        o << ";\n";
      }
    if (mode == 1) return;
    o << ind << "{ const i64 xb0_ = " << b0expr << "; if (xb0_ < B) { const int xrows_ = (int)(B - xb0_ < " << kTile << " ? B - xb0_ : " << kTile
      << "); const T* xt_ = x + xb0_ * " << DX << " + " << P.offx[bk.sx] + 16 * bk.h * n1 << ";\n";
    for (int i = 0; i < 4; ++i) {
      std::vector<std::string> nm;
      for (int c = 0; c < n1; ++c) nm.push_back("xv" + std::to_string(bk.sx) + "_" + std::to_string(bk.h) + "_" + std::to_string(i) + "_" + std::to_string(c));
      o << ind << "  { const int xr_ = 4 * q + " << i << " < xrows_ ? 4 * q + " << i << " : xrows_ - 1; const T* p_ = xt_ + (xr_ * " << DX << " + s * " << n1 << ");";
      wide_load(o, nm);
      o << " }\n";
    }
    o << ind << "} }\n";
  };
  // the x rows of the first block travel with the tile (requested a round ahead)
  if (!blocks.empty()) {
    load_x_a(blocks[0], "  ", 1);
    load_x_a(blocks[0], "  ", 2, "((i64)blockIdx.x * " + std::to_string(kWaves) + " + wv) * " + std::to_string(kTile));
  }
  o << "  #pragma unroll 1\n";
  o << "  for (i64 r_ = blockIdx.x; r_ < nround; r_ += gridDim.x) {\n";
  o << "    const i64 b0 = (r_ * " << kWaves << " + wv) * " << kTile << ";\n";
  o << "    const int rows = (int)(B - b0 < 0 ? 0 : (B - b0 < " << kTile << " ? B - b0 : " << kTile << "));\n";
  lds_write("    ", 0, half, true);
  o << "    __syncthreads();\n";
  prefetch("((r_ + gridDim.x) * " + std::to_string(kWaves) + " + wv) * " + std::to_string(kTile), "    ", 0, half, true);
  o << "    if (rows > 0) {\n";
  for (int i = 0; i < 4; ++i) {
    o << "    const bool live" << i << " = 4 * q + " << i << " < rows;\n";
    for (int j : ywords) o << "    T gy" << i << "_" << j << " = 0.0f;\n";
  }
  // The work of a tile is a list of items: quarters of a path's G' = gz W^T for one half of the channels (matrix
  // cores), then the four samples of the lane (VALU).  The LDS operands of item n+1 are requested before item n is
  // worked on, between scheduling fences.
  struct AItem { int kind, p, h, part; };   // kind 0: part `part` of the product, 1: sample `part`
  // a product is cut into 1, 2 or 4 parts of at least six matrix instructions (enough to cover an LDS round trip)
  auto gemm_parts = [](const PathInfo& pq) {
    const int total = (pq.mul_z / 4) * (2 * pq.l3 + 1);
    return total >= 24 ? 4 : (total >= 12 ? 2 : 1);
  };
  for (size_t bi = 0; bi < blocks.size(); ++bi) {
    const Blk& bk = blocks[bi];
    const int n1 = 2 * P.irx[bk.sx].l + 1;
    o << "    // x segment " << bk.sx << ", channels " << 16 * bk.h << ".." << 16 * bk.h + 15 << "\n";
    for (int i = 0; i < 4; ++i)
      for (int c = 0; c < n1; ++c) o << "    T gx" << i << "_" << c << "_b" << bi << " = 0.0f;\n";
    if (bi + 1 < blocks.size()) load_x_a(blocks[bi + 1], "    ");
    if (bi > 0 && bi + 1 == blocks.size())   // the first block of the next round's tile (its registers are free by now)
      load_x_a(blocks[0], "    ", 2, "((r_ + gridDim.x) * " + std::to_string(kWaves) + " + wv) * " + std::to_string(kTile));
    std::vector<AItem> items;
    for (size_t p = 0; p < P.paths.size(); ++p) {
      if (P.paths[p].ix != bk.sx) continue;
      for (int part = 0; part < gemm_parts(P.paths[p]); ++part) items.push_back({0, (int)p, bk.h, part});
      for (int i = 0; i < 4; ++i) items.push_back({1, (int)p, bk.h, i});
    }
    auto tag = [&](size_t n) { return "b" + std::to_string(bi) + "n" + std::to_string(n); };
    auto reads = [&](size_t n) {
      const AItem& it = items[n];
      const PathInfo& pq = P.paths[it.p];
      const int n3 = 2 * pq.l3 + 1;
      if (it.kind == 0) {
        const int per = pq.mul_z / 4 / gemm_parts(pq);   // steps of this part
        for (int st = it.part * per; st < (it.part + 1) * per; ++st) {
          for (int k = 0; k < n3; ++k)
            o << "      const T ga" << tag(n) << "_" << st << "_" << k << " = tile[s * " << ZS << " + " << P.offz[pq.iz] + 4 * st * n3 + k << " + q * " << n3 << "];\n";
          o << "      const T gw" << tag(n) << "_" << st << " = lds_w[" << wp[it.p] + (int64_t)16 * it.h * wpitch[it.p] + 4 * st << " + s * " << wpitch[it.p] << " + q];\n";
        }
      } else {
        std::set<int> js;
        for (auto& nz : pq.nz) js.insert(nz.j);
        o << "      int yo" << tag(n) << " = (4 * q + " << it.part << ") * " << YS << " + " << P.offy[pq.iy] << "; asm volatile(\"\" : \"+v\"(yo" << tag(n) << "));\n";
        for (int j : js) o << "      const T y" << tag(n) << "_" << j << " = ytile[yo" << tag(n) << " + " << j << "];\n";
      }
      o << "      __builtin_amdgcn_sched_barrier(0);\n";
    };
    if (!items.empty()) reads(0);
    for (size_t n = 0; n < items.size(); ++n) {
      const AItem& it = items[n];
      const PathInfo& pq = P.paths[it.p];
      const int n3 = 2 * pq.l3 + 1;
      if (n + 1 < items.size()) reads(n + 1);
      const std::string G = "G" + std::to_string(it.p) + "_" + std::to_string(it.h) + "_";
      if (it.kind == 0) {
        if (it.part == 0)
          for (int k = 0; k < n3; ++k) o << "      f4 " << G << k << " = {0.0f, 0.0f, 0.0f, 0.0f};\n";
        const int per = pq.mul_z / 4 / gemm_parts(pq);
        for (int st = it.part * per; st < (it.part + 1) * per; ++st)
          for (int k = 0; k < n3; ++k)
            o << "      " << G << k << " = MFMA(ga" << tag(n) << "_" << st << "_" << k << ", gw" << tag(n) << "_" << st << ", " << G << k << ");\n";
      } else {
        const int i = it.part;
        o << "      { // path " << it.p << " l=(" << pq.l1 << "," << pq.l2 << "," << pq.l3 << "), sample 4q+" << i << "\n";
        std::map<std::pair<long long, int>, std::string> seen;
        std::vector<std::pair<std::string, bool>> tr;
        int tc = 0;
        for (auto& nz : pq.nz) {
          const double c = nz.v * pq.coeff, a = std::fabs(c);
          auto key = std::make_pair(std::llround(a * 1e13), nz.j);
          auto f = seen.find(key);
          if (f == seen.end()) {
            std::string name = "y" + tag(n) + "_" + std::to_string(nz.j);
            if (std::fabs(a - 1.0) >= 1e-15) {
              std::string tn = "t" + std::to_string(tc++);
              o << "        const T " << tn << " = " << name << " * " << lit(a) << ";\n";
              name = tn;
            }
            f = seen.insert({key, name}).first;
          }
          tr.push_back({f->second, c < 0});
        }
        auto xv = [&](int c) { return "xv" + std::to_string(bk.sx) + "_" + std::to_string(bk.h) + "_" + std::to_string(i) + "_" + std::to_string(c); };
        for (size_t m = 0; m < pq.nz.size(); ++m) {
          const Nz& nz = pq.nz[m];
          std::string tt = std::string(tr[m].second ? "-" : "") + tr[m].first;
          std::string gxn = "gx" + std::to_string(i) + "_" + std::to_string(nz.i) + "_b" + std::to_string(bi);
          o << "        " << gxn << " = FMA(" << tt << ", " << G << nz.k << "[" << i << "], " << gxn << ");\n";
        }
        std::map<std::pair<int, long long>, std::vector<size_t>> groups;
        for (size_t m = 0; m < pq.nz.size(); ++m)
          groups[{pq.nz[m].j, std::llround(std::fabs(pq.nz[m].v * pq.coeff) * 1e13)}].push_back(m);
        int gi = 0;
        std::vector<std::string> pins;
        for (auto& kv : groups) {
          std::string sn = "sg" + std::to_string(gi++);
          bool first = true;
          for (size_t m : kv.second) {
            const Nz& nz = pq.nz[m];
            const bool neg = nz.v * pq.coeff < 0;
            std::string xx = std::string(neg ? "-" : "") + xv(nz.i);
            std::string g = G + std::to_string(nz.k) + "[" + std::to_string(i) + "]";
            if (first) o << "        T " << sn << " = " << xx << " * " << g << ";\n";
            else o << "        " << sn << " = FMA(" << xx << ", " << g << ", " << sn << ");\n";
            first = false;
          }
          std::string gyn = "gy" + std::to_string(i) + "_" + std::to_string((int)P.offy[pq.iy] + kv.first.first);
          o << "        " << gyn << " = FMA(" << sn << ", " << lit(std::fabs(pq.nz[kv.second[0]].v * pq.coeff)) << ", " << gyn << ");\n";
          pins.push_back(gyn);
        }
        o << "      }\n";
        // the accumulators are only read at the end of the block / tile: pin them so that their updates (and the
        // operands those need) are not postponed until then
        for (int c = 0; c < n1; ++c) pins.push_back("gx" + std::to_string(i) + "_" + std::to_string(c) + "_b" + std::to_string(bi));
        std::sort(pins.begin(), pins.end());
        pins.erase(std::unique(pins.begin(), pins.end()), pins.end());
        for (size_t at = 0; at < pins.size(); at += 12) {
          o << "      asm volatile(\"\" :";
          for (size_t t = at; t < pins.size() && t < at + 12; ++t) o << (t > at ? ", " : " ") << "\"+v\"(" << pins[t] << ")";
          o << ");\n";
        }
      }
      o << "      __builtin_amdgcn_sched_barrier(0);\n";
    }
    for (int i = 0; i < 4; ++i) {
      // (the lane offset passes through an empty asm: the 64-bit lane address is formed here, not kept from the top of the round)
      o << "    if (live" << i << ") { int o_ = (4 * q + " << i << ") * " << DX << " + s * " << n1 << "; asm volatile(\"\" : \"+v\"(o_)); T* p_ = gx + b0 * " << DX << " + "
        << P.offx[bk.sx] + 16 * bk.h * n1 << " + o_;";
      for (int c = 0; c < n1; ++c) o << " p_[" << c << "] = gx" << i << "_" << c << "_b" << bi << ";";
      o << " }\n";
    }
    if (blocks.size() == 1)   // a single block: its rows for the next round can only be requested after their last use
      load_x_a(blocks[0], "    ", 2, "((r_ + gridDim.x) * " + std::to_string(kWaves) + " + wv) * " + std::to_string(kTile));
  }
  for (size_t sx = 0; sx < P.irx.size(); ++sx) {
    const Irrep& ir = P.irx[sx];
    if (used_x.count((int)sx)) continue;
    o << "    for (int i = lane; i < rows * " << ir.dim() << "; i += 64) gx[(b0 + i / " << ir.dim() << ") * " << DX << " + " << P.offx[sx]
      << " + i % " << ir.dim() << "] = 0.0f;\n";
  }
  // gy: sum over the 16 lanes of a row (the channels) with DPP row operations, every lane ends with the total;
  // lane s then stores word s (+16, +32, ...) of each of its samples
  for (int i = 0; i < 4; ++i) {
    for (int j : ywords) {
      const std::string v = "gy" + std::to_string(i) + "_" + std::to_string(j);
      o << "    " << v << " = row_sum(" << v << ");\n";
    }
    for (int c0 = 0; c0 < DY; c0 += 16) {
      o << "    { T v_ = 0.0f;\n";
      for (int j = c0; j < DY && j < c0 + 16; ++j)
        if (ywords.count(j)) o << "      v_ = s == " << j - c0 << " ? gy" << i << "_" << j << " : v_;\n";
      o << "      int o_ = (4 * q + " << i << ") * " << DY << " + " << c0 << " + s; asm volatile(\"\" : \"+v\"(o_));\n";
      o << "      if (live" << i << " && s + " << c0 << " < " << DY << ") (gy + b0 * " << DY << ")[o_] = v_;\n";
      o << "    }\n";
    }
  }
  o << "    }\n";          // rows > 0
  o << "    __syncthreads();\n";
  o << "  }\n";            // rounds
  o << "  }\n";            // tile waves

  // ---------------------------------------------------------------- block waves
  // which block wave carries the second half of which tile: the waves with the fewest x registers first
  std::vector<std::vector<int>> carried(NB);
  {
    std::vector<int> load(NB, 0);
    for (int v = 0; v < NB; ++v) {
      std::set<std::pair<int, int>> nd;
      for (auto& un : share[v]) nd.insert({P.paths[un.p].ix, un.h});
      for (auto& e : nd) load[v] += 2 * 4 * (2 * P.irx[e.first].l + 1);
      for (auto& un : share[v]) load[v] += 4 * (P.paths[un.p].mul_z / 16);
    }
    const int cost = (perz - half) * (vec ? 4 : 1);
    for (int t = 0; t < kWaves; ++t) {
      int best = 0;
      for (int v = 1; v < NB; ++v)
        if (load[v] < load[best]) best = v;
      carried[best].push_back(t);
      load[best] += cost;
    }
  }
  for (int v = 0; v < NB; ++v) {
    o << "  else if (wv == " << kWaves + v << ") {\n";
    for (auto& un : share[v])
      for (int h2 = 0; h2 < P.paths[un.p].mul_z / 16; ++h2)
        o << "    f4 aw" << un.p << "_" << un.h << "_" << h2 << " = {0.0f, 0.0f, 0.0f, 0.0f};\n";
    // the x rows this wave needs per tile, (segment, u block) pairs, held in two register sets: the rows of the
    // next tile are requested before the current tile is worked on (rows clamped into the batch: what rows past the
    // end contribute is multiplied by the zero rows of the tile)
    std::set<std::pair<int, int>> need;
    for (auto& un : share[v]) need.insert({P.paths[un.p].ix, un.h});
    auto xname = [&](int set, int sx, int h, int i, int c) {
      return std::string(set ? "xb" : "xa") + std::to_string(sx) + "_" + std::to_string(h) + "_" + std::to_string(i) + "_" + std::to_string(c);
    };
    for (int set = 0; set < 2; ++set)
      for (auto& nd : need)
        for (int i = 0; i < 4; ++i)
          for (int c = 0; c < 2 * P.irx[nd.first].l + 1; ++c) o << "    T " << xname(set, nd.first, nd.second, i, c) << " = 0.0f;\n";
    auto load_set = [&](int set, const std::string& b0expr, const char* ind) {
      o << ind << "{ const i64 nb0_ = " << b0expr << "; if (nb0_ < B) { const int nrows_ = (int)(B - nb0_ < " << kTile << " ? B - nb0_ : " << kTile
        << "); const T* xt_ = x + nb0_ * " << DX << ";\n";
      for (int i = 0; i < 4; ++i) {
        o << ind << "  const int nr" << i << " = (4 * q + " << i << " < nrows_ ? 4 * q + " << i << " : nrows_ - 1) * " << DX << ";\n";
        for (auto& nd : need) {
          const int n1 = 2 * P.irx[nd.first].l + 1;
          std::vector<std::string> nm;
          for (int c = 0; c < n1; ++c) nm.push_back(xname(set, nd.first, nd.second, i, c));
          o << ind << "  { const T* p_ = xt_ + (nr" << i << " + " << P.offx[nd.first] + 16 * nd.second * n1 << " + s * " << n1 << ");";
          wide_load(o, nm);
          o << " }\n";
        }
      }
      o << ind << "} }\n";
    };
    if (!need.empty()) load_set(0, "(i64)blockIdx.x * " + std::to_string(kWaves * kTile), "    ");
    // the second halves of the gz rows of the tiles in carried[v] travel through this wave's registers
    for (int t : carried[v]) {
      const std::string pf = "pf" + std::to_string(t);
      o << "    " << (vec ? "f4 " : "T ") << pf << "[" << perz << "];\n";
      o << "    T* tile" << t << " = lds_g[" << t << "];\n";
      prefetch("((i64)blockIdx.x * " + std::to_string(kWaves) + " + " + std::to_string(t) + ") * " + std::to_string(kTile), "    ", half, perz, false, pf);
    }
    o << "    #pragma unroll 1\n";
    o << "    for (i64 r_ = blockIdx.x; r_ < nround; r_ += gridDim.x) {\n";
    for (int t : carried[v]) {
      o << "      { const i64 b0 = (r_ * " << kWaves << " + " << t << ") * " << kTile << ";\n";
      o << "        const int rows = (int)(B - b0 < 0 ? 0 : (B - b0 < " << kTile << " ? B - b0 : " << kTile << "));\n";
      lds_write("        ", half, perz, false, "pf" + std::to_string(t), "tile" + std::to_string(t));
      o << "      }\n";
    }
    o << "      __syncthreads();\n";
    for (int t : carried[v])
      prefetch("((r_ + gridDim.x) * " + std::to_string(kWaves) + " + " + std::to_string(t) + ") * " + std::to_string(kTile), "      ", half, perz, false, "pf" + std::to_string(t));
    {
      // the four tiles of the round, one loop body (the code of a block wave is the nonzeros of its paths once per
      // sample of the lane): set a holds the rows of the current tile, set b receives those of the next
      const int set = 0;
      o << "      #pragma unroll 1\n";
      o << "      for (int tl = 0; tl < " << kWaves << "; ++tl) {\n";
      o << "        const i64 b0 = (r_ * " << kWaves << " + tl) * " << kTile << ";\n";
      if (!need.empty())
        load_set(1, "(tl + 1 < " + std::to_string(kWaves) + ") ? b0 + " + std::to_string(kTile) + " : (r_ + gridDim.x) * " + std::to_string(kWaves * kTile), "        ");
      o << "        if (b0 < B) {\n";
      o << "        const T* tile_ = lds_g[tl];\n        const T* ytile = lds_y[tl];\n";
      // The work of a tile is a list of items (path, u block, sample of the lane).  The LDS operands of item n+1
      // (its y words and the gz values that are the B operands of its products) are requested before item n is
      // worked on, between scheduling fences, so that no product waits for an LDS round trip.
      struct Item { int p, h, i; };
      std::vector<Item> items;
      for (auto& un : share[v])
        for (int i = 0; i < 4; ++i) items.push_back({un.p, un.h, i});
      auto reads = [&](size_t n) {
        const Item& it = items[n];
        const PathInfo& pq = P.paths[it.p];
        const int n3 = 2 * pq.l3 + 1, HZ = pq.mul_z / 16;
        std::set<int> js, ks;
        for (auto& nz : pq.nz) { js.insert(nz.j); ks.insert(nz.k); }
        o << "          int yo" << n << " = (4 * q + " << it.i << ") * " << YS << " + " << P.offy[pq.iy] << "; asm volatile(\"\" : \"+v\"(yo" << n << "));\n";
        for (int j : js) o << "          const T y" << n << "_" << j << " = ytile[yo" << n << " + " << j << "];\n";
        o << "          const T* g" << n << " = tile_ + (4 * q + " << it.i << ") * " << ZS << " + " << P.offz[pq.iz] << " + s * " << n3 << ";\n";
        for (int k : ks)
          for (int h2 = 0; h2 < HZ; ++h2) o << "          const T gb" << n << "_" << k << "_" << h2 << " = g" << n << "[" << k + 16 * h2 * n3 << "];\n";
        o << "          __builtin_amdgcn_sched_barrier(0);\n";
      };
      if (!items.empty()) reads(0);
      for (size_t n = 0; n < items.size(); ++n) {
        const Item& it = items[n];
        const PathInfo& pq = P.paths[it.p];
        const int n3 = 2 * pq.l3 + 1, HZ = pq.mul_z / 16;
        if (n + 1 < items.size()) reads(n + 1);
        o << "          { // path " << it.p << " l=(" << pq.l1 << "," << pq.l2 << "," << pq.l3 << "), u block " << it.h << ", sample 4q+" << it.i << "\n";
        std::map<std::pair<long long, int>, std::string> seen;
        int tc = 0;
        std::vector<bool> started((size_t)n3, false);
        for (auto& nz : pq.nz) {
          const double c = nz.v * pq.coeff, a = std::fabs(c);
          auto key = std::make_pair(std::llround(a * 1e13), nz.j);
          auto f = seen.find(key);
          if (f == seen.end()) {
            std::string name = "y" + std::to_string(n) + "_" + std::to_string(nz.j);
            if (std::fabs(a - 1.0) >= 1e-15) {
              std::string tn = "t" + std::to_string(tc++);
              o << "            const T " << tn << " = " << name << " * " << lit(a) << ";\n";
              name = tn;
            }
            f = seen.insert({key, name}).first;
          }
          std::string tt = std::string(c < 0 ? "-" : "") + f->second;
          std::string xx = xname(set, pq.ix, it.h, it.i, nz.i);
          if (!started[nz.k]) {
            o << "            T zq" << nz.k << " = " << tt << " * " << xx << ";\n";
            started[nz.k] = true;
          } else {
            o << "            zq" << nz.k << " = FMA(" << tt << ", " << xx << ", zq" << nz.k << ");\n";
          }
        }
        // A = z' (row u = 16h+s, inner index q <-> sample 4q+i), B = gz of the same samples
        for (int k = 0; k < n3; ++k) {
          if (!started[k]) continue;
          for (int h2 = 0; h2 < HZ; ++h2)
            o << "            aw" << it.p << "_" << it.h << "_" << h2 << " = MFMA(zq" << k << ", gb" << n << "_" << k << "_" << h2 << ", aw" << it.p << "_" << it.h << "_" << h2 << ");\n";
        }
        o << "          }\n";
        o << "          __builtin_amdgcn_sched_barrier(0);\n";
      }
      o << "        }\n";   // b0 < B
      for (auto& nd : need)
        for (int i = 0; i < 4; ++i)
          for (int c = 0; c < 2 * P.irx[nd.first].l + 1; ++c)
            o << "        " << xname(0, nd.first, nd.second, i, c) << " = " << xname(1, nd.first, nd.second, i, c) << ";\n";
      o << "      }\n";
    }
    o << "      __syncthreads();\n";
    o << "    }\n";
    o << "    f4* part = (f4*)gwpart + (i64)blockIdx.x * " << blk.back() * 64 << " + lane;\n";
    for (auto& un : share[v])
      for (int h2 = 0; h2 < P.paths[un.p].mul_z / 16; ++h2)
        o << "    part[" << (blk[un.p] + un.h * (P.paths[un.p].mul_z / 16) + h2) * 64 << "] = aw" << un.p << "_" << un.h << "_" << h2 << ";\n";
    o << "  }\n";
  }
  o << "}\n";
  K.source = o.str();
  emit_gw_reduce(P, blk, Kred);
}

}  // namespace cgtp
