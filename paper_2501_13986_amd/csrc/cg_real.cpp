// Irreps parsing and the planner's own Clebsch-Gordan generator.
//
// The coefficient blocks P^(l1,l2,l3) of paper Sec. 2.2 are produced here as nonzero lists
// that the emitters turn into literals (paper Sec. 3.2: indices and values are known when
// the kernel is generated).  Route taken: complex coupling coefficients <l1 m1 l2 m2|l3 m3>
// from Racah's single-sum formula; the coupled vector is rotated to the real basis,
// Z_real = U3 . CG . (U1^H X_real) (U2^H Y_real); the global phase (1 or i) is removed;
// the sign is fixed by making the first nonzero positive.  Since sum_{m1 m2} |CG|^2 = 1
// for every m3, the block comes out with sum_{ij} C[ijk] C[ijk'] = delta_{kk'}.
#include <cmath>
#include <complex>
#include <cstdlib>
#include <stdexcept>

#include "plan.hpp"

namespace cgtp {

int env_int(const char* name, int fallback) {
  const char* s = std::getenv(name);
  if (!s || !*s) return fallback;
  char* end = nullptr;
  long v = std::strtol(s, &end, 10);
  return (end && *end == 0) ? (int)v : fallback;
}

std::vector<Irrep> parse_irreps(const std::string& s) {
  std::vector<Irrep> out;
  size_t pos = 0;
  auto skip = [&]() { while (pos < s.size() && std::isspace((unsigned char)s[pos])) ++pos; };
  auto number = [&](long& v) {
    skip();
    size_t b = pos;
    v = 0;
    while (pos < s.size() && std::isdigit((unsigned char)s[pos])) {
      v = v * 10 + (s[pos] - '0');
      if (v > 1000000) throw std::invalid_argument("number too large in irreps '" + s + "'");
      ++pos;
    }
    return pos > b;
  };
  for (;;) {
    long a = 0, l = 0, mul = 1;
    if (!number(a)) throw std::invalid_argument("expected a number in irreps '" + s + "'");
    skip();
    if (pos < s.size() && s[pos] == 'x') {
      ++pos;
      mul = a;
      if (!number(l)) throw std::invalid_argument("expected a degree after 'x' in irreps '" + s + "'");
    } else {
      l = a;
    }
    skip();
    if (pos >= s.size() || (s[pos] != 'e' && s[pos] != 'o'))
      throw std::invalid_argument("expected parity 'e' or 'o' in irreps '" + s + "'");
    int p = s[pos] == 'e' ? 1 : -1;
    ++pos;
    if (mul <= 0) throw std::invalid_argument("multiplicity must be positive in irreps '" + s + "'");
    out.push_back(Irrep{(int)mul, (int)l, p});
    skip();
    if (pos >= s.size()) break;
    if (s[pos] != '+') throw std::invalid_argument("expected '+' in irreps '" + s + "'");
    ++pos;
  }
  return out;
}

namespace {

using cplx = std::complex<long double>;

long double fact(int n) {
  long double r = 1.0L;
  for (int t = 2; t <= n; ++t) r *= t;
  return r;
}

// <j1 m1 j2 m2 | j3 m3>, Racah's formula, integer momenta.
long double coupling(int j1, int m1, int j2, int m2, int j3, int m3) {
  if (m3 != m1 + m2 || j3 < std::abs(j1 - j2) || j3 > j1 + j2) return 0.0L;
  if (std::abs(m1) > j1 || std::abs(m2) > j2 || std::abs(m3) > j3) return 0.0L;
  long double delta = fact(j1 + j2 - j3) * fact(j1 - j2 + j3) * fact(-j1 + j2 + j3) / fact(j1 + j2 + j3 + 1);
  long double pref = (2 * j3 + 1) * delta * fact(j3 + m3) * fact(j3 - m3) * fact(j1 - m1) * fact(j1 + m1) *
                     fact(j2 - m2) * fact(j2 + m2);
  long double sum = 0.0L;
  for (int t = 0; t <= j1 + j2 - j3; ++t) {
    int a = j1 + j2 - j3 - t, b = j1 - m1 - t, c = j2 + m2 - t, d = j3 - j2 + m1 + t, e = j3 - j1 - m2 + t;
    if (a < 0 || b < 0 || c < 0 || d < 0 || e < 0) continue;
    long double term = 1.0L / (fact(t) * fact(a) * fact(b) * fact(c) * fact(d) * fact(e));
    sum += (t & 1) ? -term : term;
  }
  return std::sqrt(pref) * sum;
}

// Row m of the unitary that maps complex harmonics to real ones: only columns +-m are set.
//   m > 0 : (Y^{-m} + (-1)^m Y^{m}) / sqrt2      m < 0 : i (Y^{m} - (-1)^m Y^{-m}) / sqrt2
cplx to_real(int m, int mu) {
  const long double r = 1.0L / std::sqrt(2.0L);
  const long double sg = (std::abs(m) & 1) ? -1.0L : 1.0L;
  if (m == 0) return mu == 0 ? cplx(1, 0) : cplx(0, 0);
  if (m > 0) {
    if (mu == -m) return cplx(r, 0);
    if (mu == m) return cplx(sg * r, 0);
    return cplx(0, 0);
  }
  if (mu == m) return cplx(0, r);
  if (mu == -m) return cplx(0, -sg * r);
  return cplx(0, 0);
}

}  // namespace

std::vector<Nz> cg_nonzeros(int l1, int l2, int l3) {
  std::vector<Nz> out;
  if (l3 < std::abs(l1 - l2) || l3 > l1 + l2) return out;
  const int n1 = 2 * l1 + 1, n2 = 2 * l2 + 1, n3 = 2 * l3 + 1;
  std::vector<cplx> t((size_t)n1 * n2 * n3, cplx(0, 0));
  for (int a = -l1; a <= l1; ++a)        // real index of x
    for (int b = -l2; b <= l2; ++b)      // real index of y
      for (int c = -l3; c <= l3; ++c) {  // real index of z
        cplx acc(0, 0);
        // only mu1 = +-a, mu2 = +-b, mu3 = +-c contribute
        for (int s1 = -1; s1 <= 1; s1 += 2)
          for (int s2 = -1; s2 <= 1; s2 += 2) {
            int mu1 = s1 * a, mu2 = s2 * b;
            if ((a == 0 && s1 > 0) || (b == 0 && s2 > 0)) continue;  // count mu = 0 once
            int mu3 = mu1 + mu2;
            if (std::abs(mu3) != std::abs(c)) continue;
            long double cgv = coupling(l1, mu1, l2, mu2, l3, mu3);
            if (cgv == 0.0L) continue;
            acc += to_real(c, mu3) * cgv * std::conj(to_real(a, mu1)) * std::conj(to_real(b, mu2));
          }
        t[((size_t)(a + l1) * n2 + (b + l2)) * n3 + (c + l3)] = acc;
      }
  // global phase: the tensor is real up to a factor that is either 1 or +-i
  long double re = 0, im = 0;
  for (auto& v : t) {
    re += std::fabs(v.real());
    im += std::fabs(v.imag());
  }
  const bool imag = im > re;
  if ((imag ? re : im) > 1e-14L) throw std::runtime_error("CG block is not real up to a global phase");
  bool first = true;
  long double sign = 1.0L;
  for (int i = 0; i < n1; ++i)
    for (int j = 0; j < n2; ++j)
      for (int k = 0; k < n3; ++k) {
        cplx v = t[((size_t)i * n2 + j) * n3 + k];
        long double r = imag ? v.imag() : v.real();
        if (std::fabs(r) < 1e-13L) continue;
        if (first) {
          sign = r < 0 ? -1.0L : 1.0L;
          first = false;
        }
        out.push_back(Nz{i, j, k, (double)(sign * r)});
      }
  return out;
}

}  // namespace cgtp
