#include "scat_host3d.hpp"

#include "scat_host.hpp"

#include <cmath>

namespace scat {

namespace {

constexpr double kPi = 3.14159265358979323846264338327950288;

bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

// Real orthonormal spherical harmonics of degree l at the direction (x, y, z) / r, times
// r^l (a homogeneous harmonic polynomial, finite at r = 0): out[m + l], m = -l .. l.
// Associated Legendre functions by the standard upward recurrences in cos(theta), with
// sin^m(theta) e^{i m phi} expanded from (x + i y)^m / r^m so that no angle is formed.
void solid_harmonics(int l, double x, double y, double z, double *out) {
  const double r2 = x * x + y * y + z * z;
  const double r = std::sqrt(r2);
  if (r == 0.0) {
    for (int m = -l; m <= l; ++m) out[m + l] = 0.0;
    if (l == 0) out[0] = 1.0 / std::sqrt(4.0 * kPi);
    return;
  }
  const double ct = z / r;
  const double st = std::sqrt(std::fmax(0.0, 1.0 - ct * ct));
  const double rl = std::pow(r, l);
  // (cos phi, sin phi); the azimuth is irrelevant on the axis, where sin(theta) = 0
  const double rho = std::sqrt(x * x + y * y);
  const double cp = rho > 0 ? x / rho : 1.0, sp = rho > 0 ? y / rho : 0.0;
  double cm = 1.0, sm = 0.0;  // cos(m phi), sin(m phi)
  double pmm = 1.0;           // P_m^m(ct), Condon-Shortley phase left out (basis choice)
  for (int m = 0; m <= l; ++m) {
    if (m > 0) {
      pmm *= (2 * m - 1) * st;
      const double c2 = cm * cp - sm * sp, s2 = sm * cp + cm * sp;
      cm = c2;
      sm = s2;
    }
    // P_l^m from P_m^m by the recurrence in the degree
    double p_prev = 0.0, p = pmm;
    for (int k = m + 1; k <= l; ++k) {
      const double pn = ((2 * k - 1) * ct * p - (k + m - 1) * p_prev) / (k - m);
      p_prev = p;
      p = pn;
    }
    // normalisation sqrt((2l+1)/(4 pi) (l-m)!/(l+m)!)
    double ratio = 1.0;
    for (int k = l - m + 1; k <= l + m; ++k) ratio /= k;
    const double nlm = std::sqrt((2 * l + 1) / (4.0 * kPi) * ratio);
    if (m == 0) {
      out[l] = nlm * p * rl;
    } else {
      out[l + m] = std::sqrt(2.0) * nlm * p * cm * rl;
      out[l - m] = std::sqrt(2.0) * nlm * p * sm * rl;
    }
  }
}

}  // namespace

int validate_3d(const int *shape, int J, int L, int max_order) {
  if (J < 1 || J > 8 || L < 0 || L > 8) return 1;
  if (max_order != 1 && max_order != 2) return 1;
  for (int d = 0; d < 3; ++d) {
    if (!is_pow2(shape[d])) return 2;
    if (shape[d] < (1 << J) || shape[d] < 4 || shape[d] > 256) return 2;
  }
  return 0;
}

void build_host_plan_3d(HostPlan3D &p, const int *shape, int J, int L, int max_order) {
  for (int d = 0; d < 3; ++d) p.shape[d] = shape[d];
  p.J = J;
  p.L = L;
  p.max_order = max_order;
  p.index.clear();
  p.index.push_back(Coeff3D{0, -1, -1, -1});
  for (int j = 0; j < J; ++j)
    for (int l = 0; l <= L; ++l) p.index.push_back(Coeff3D{1, j, l, -1});
  if (max_order == 2)
    for (int j1 = 0; j1 < J; ++j1)
      for (int l = 0; l <= L; ++l)
        for (int j2 = j1 + 1; j2 < J; ++j2) p.index.push_back(Coeff3D{2, j1, l, j2});
  p.K = static_cast<int>(p.index.size());

  const size_t n = p.points();
  const int n0 = shape[0], n1 = shape[1], n2 = shape[2];
  auto freq = [](int k, int nn) { return 2.0 * kPi * (k < (nn + 1) / 2 ? k : k - nn) / nn; };
  // aliases needed: exp(-(2^j * 2 pi a)^2 / 2) is below 1e-17 beyond |a| = 2 at j = 0
  p.psi.assign(static_cast<size_t>(J) * (L + 1), std::vector<double>());
  for (int j = 0; j < J; ++j) {
    const double s = std::ldexp(1.0, j);
    const int na = j == 0 ? 2 : 1, A = 2 * na + 1;
    // scaled alias frequencies of every index along each axis
    std::vector<double> wa[3];
    for (int d = 0; d < 3; ++d) {
      wa[d].resize(static_cast<size_t>(shape[d]) * A);
      for (int k = 0; k < shape[d]; ++k)
        for (int a = -na; a <= na; ++a)
          wa[d][static_cast<size_t>(k) * A + a + na] = s * (freq(k, shape[d]) + 2.0 * kPi * a);
    }
    for (int l = 0; l <= L; ++l) {
      std::vector<double> &tab = p.psi[static_cast<size_t>(j) * (L + 1) + l];
      tab.assign(static_cast<size_t>(2 * l + 1) * n, 0.0);
      // slices of axis 0 are independent: one thread each, a few at a time
      auto slice = [&](int k0) {
        double sh[2 * 8 + 1];
        for (int k1 = 0; k1 < n1; ++k1)
          for (int k2 = 0; k2 < n2; ++k2) {
            const size_t e = (static_cast<size_t>(k0) * n1 + k1) * n2 + k2;
            for (int a0 = 0; a0 < A; ++a0) {
              const double w0 = wa[0][static_cast<size_t>(k0) * A + a0];
              if (w0 * w0 > 90.0) continue;
              for (int a1 = 0; a1 < A; ++a1) {
                const double w1 = wa[1][static_cast<size_t>(k1) * A + a1];
                if (w0 * w0 + w1 * w1 > 90.0) continue;
                for (int a2 = 0; a2 < A; ++a2) {
                  const double w2 = wa[2][static_cast<size_t>(k2) * A + a2];
                  const double r2 = w0 * w0 + w1 * w1 + w2 * w2;
                  if (r2 > 90.0) continue;  // r^8 exp(-45) < 2e-12: below fp32 resolution
                  const double g = std::exp(-0.5 * r2);
                  solid_harmonics(l, w0, w1, w2, sh);
                  for (int m = 0; m < 2 * l + 1; ++m) tab[static_cast<size_t>(m) * n + e] += g * sh[m];
                }
              }
            }
          }
      };
      parallel_for(n0, slice);
    }
  }
  // lowpass: Gaussian of std 2^J and unit mass sampled at the integers: its spectrum is
  // the alias sum of exp(-(sigma |omega + 2 pi a|)^2 / 2), a product of one sum per axis
  const double sig = std::ldexp(1.0, J);
  std::vector<double> ph[3];
  for (int d = 0; d < 3; ++d) {
    ph[d].resize(shape[d]);
    for (int k = 0; k < shape[d]; ++k) {
      double acc = 0.0;
      for (int a = -1; a <= 1; ++a) {
        const double w = freq(k, shape[d]) + 2.0 * kPi * a;
        acc += std::exp(-0.5 * sig * sig * w * w);
      }
      ph[d][k] = acc;
    }
  }
  p.phi.assign(n, 0.0);
  for (int k0 = 0; k0 < n0; ++k0)
    for (int k1 = 0; k1 < n1; ++k1)
      for (int k2 = 0; k2 < n2; ++k2)
        p.phi[(static_cast<size_t>(k0) * n1 + k1) * n2 + k2] = ph[0][k0] * ph[1][k1] * ph[2][k2];
}

}  // namespace scat
