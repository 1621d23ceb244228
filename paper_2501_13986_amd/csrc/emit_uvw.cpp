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
  const int region = kTile * std::max(XS, ZS);
  const int64_t lds_bytes = 4 * (P.n_w + (int64_t)kWaves * region);
  if (lds_bytes > 160 * 1024) throw std::runtime_error("uvw: weights + tiles exceed the 160 KB of LDS");
  K.wg = 64 * kWaves;
  K.name = "cgtp_tp_fwd";
  std::ostringstream o;
  o << "typedef float T;\ntypedef long long i64;\n";
  o << "typedef float f4 __attribute__((ext_vector_type(4)));\n";
  o << "#define FMA(a, b, c) __builtin_fmaf((a), (b), (c))\n";
  o << "extern \"C\" __global__ void __launch_bounds__(" << K.wg << ") " << K.name
    << "(const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ W, T* __restrict__ z, i64 B)\n{\n";
  o << "  __shared__ T lds_w[" << P.n_w << "];\n";
  o << "  __shared__ T lds_t[" << kWaves << "][" << region << "];\n";
  o << "  for (int i = threadIdx.x; i < " << P.n_w << "; i += " << K.wg << ") lds_w[i] = W[i];\n";
  o << "  __syncthreads();\n";
  o << "  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;\n";
  o << "  const int s = lane & 15, q = lane >> 4;\n";
  o << "  T* tile = lds_t[wv];\n";
  o << "  const i64 ntile = (B + " << kTile - 1 << ") / " << kTile << ";\n";
  o << "  for (i64 t_ = (i64)blockIdx.x * " << kWaves << " + wv; t_ < ntile; t_ += (i64)gridDim.x * " << kWaves << ") {\n";
  o << "    const i64 b0 = t_ * " << kTile << ";\n";
  o << "    const int rows = (int)((B - b0) < " << kTile << " ? (B - b0) : " << kTile << ");\n";
  // stage the x tile: rows are contiguous in memory, LDS pitch is odd
  o << "    __builtin_amdgcn_wave_barrier();\n";
  o << "    for (int i = lane; i < rows * " << DX << "; i += 64) { const int r_ = i / " << DX << ", c_ = i - r_ * " << DX
    << "; tile[r_ * " << XS << " + c_] = x[b0 * " << DX << " + i]; }\n";
  o << "    for (int i = rows * " << DX << " + lane; i < " << kTile * DX << "; i += 64) { const int r_ = i / " << DX << ", c_ = i - r_ * "
    << DX << "; tile[r_ * " << XS << " + c_] = 0.0f; }\n";
  o << "    __builtin_amdgcn_wave_barrier();\n";
  // y of the lane's sample and the coefficient products
  std::set<int> ywords;
  for (auto& p : P.paths)
    for (auto& n : p.nz) ywords.insert((int)P.offy[p.iy] + n.j);
  o << "    const bool live = s < rows;\n";
  o << "    const T* yb = y + (b0 + (live ? s : 0)) * " << DY << ";\n";
  for (int j : ywords) o << "    const T y" << j << " = live ? yb[" << j << "] : 0.0f;\n";
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
  // channel loop: 4 channels of x per step (one per lane group q)
  o << "    #pragma unroll 1\n";
  o << "    for (int c = 0; c < " << maxmul / 4 << "; ++c) {\n";
  o << "      const int u = 4 * c + q;\n";
  std::set<int> used_x;
  for (auto& p : P.paths) used_x.insert(p.ix);
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
  o << "    for (int i = lane; i < rows * " << DZ << "; i += 64) { const int r_ = i / " << DZ << ", c_ = i - r_ * " << DZ << "; z[b0 * " << DZ
    << " + i] = tile[r_ * " << ZS << " + c_]; }\n";
  o << "  }\n}\n";
  K.source = o.str();
}

}  // namespace cgtp
