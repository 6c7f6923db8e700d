// Host-side core: validation, index table, analytic filter bank (fp64).
//
// The wavelets are Morlet wavelets (paper section 2, "Implementation"); the paper
// gives no formula, so the construction is this library's: a Gabor function minus a
// multiple of its Gaussian envelope, the multiple chosen so the sampled, periodised
// wavelet has zero mean.  A function sampled at the integers and made N-periodic has
// as DFT its continuous Fourier transform sampled at 2 pi k / N and summed over all
// 2 pi shifts (Poisson summation), so the tables are evaluated directly in the Fourier
// domain: Gaussians centred at the wavelet's centre frequency, plus their aliases.
#include "scat_host.hpp"

#include <cmath>

namespace scat {

namespace {

constexpr double kPi = 3.14159265358979323846264338327950288;
constexpr double kMinExponent = -100.0;  // exp() below this is dropped (< 4e-44)

bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

// Number of 2 pi aliases needed on each side so that the dropped Gaussians are below
// exp(kMinExponent) everywhere: sigma_f is the narrowest spatial standard deviation.
int alias_count(double sigma_narrow) {
  double reach = std::sqrt(-2.0 * kMinExponent) / sigma_narrow;  // frequency radius
  return static_cast<int>(std::ceil(reach / (2.0 * kPi))) + 1;
}

struct Gauss2 {
  double sigma, slant, ct, st;
  double operator()(double wr, double wc) const {
    double al = wr * ct + wc * st;
    double ac = (-wr * st + wc * ct) / slant;
    double e = -0.5 * sigma * sigma * (al * al + ac * ac);
    return e < kMinExponent ? 0.0 : std::exp(e);
  }
};

// psi_hat on the n_r x n_c grid for (sigma, xi, theta, slant).
void morlet_hat_2d(std::vector<double> &out, int n_r, int n_c, double sigma, double xi,
                   double theta, double slant) {
  Gauss2 g{sigma, slant, std::cos(theta), std::sin(theta)};
  const double xr = xi * g.ct, xc = xi * g.st;
  const int A = alias_count(sigma * std::fmin(1.0, 1.0 / slant));
  double gab0 = 0.0, env0 = 0.0;
  for (int a = -A; a <= A; ++a)
    for (int b = -A; b <= A; ++b) {
      gab0 += g(2.0 * kPi * a - xr, 2.0 * kPi * b - xc);
      env0 += g(2.0 * kPi * a, 2.0 * kPi * b);
    }
  const double kappa = gab0 / env0;
  out.assign(static_cast<size_t>(n_r) * n_c, 0.0);
  // rows are independent: spread over host threads (a 512 x 512 bank takes seconds on one)
  parallel_for(n_r, [&](int kr) {
    for (int kc = 0; kc < n_c; ++kc) {
      double gab = 0.0, env = 0.0;
      for (int a = -A; a <= A; ++a) {
        double wr = 2.0 * kPi * (static_cast<double>(kr) + static_cast<double>(a) * n_r) / n_r;
        for (int b = -A; b <= A; ++b) {
          double wc = 2.0 * kPi * (static_cast<double>(kc) + static_cast<double>(b) * n_c) / n_c;
          gab += g(wr - xr, wc - xc);
          env += g(wr, wc);
        }
      }
      out[static_cast<size_t>(kr) * n_c + kc] = gab - kappa * env;
    }
  });
  out[0] = 0.0;  // exact zero mean (gab - kappa*env at the origin is 0 up to rounding)
}

// 1-D periodised Gaussian spectrum: sum_a exp(-sigma^2 (w + 2 pi a)^2 / 2) at w = 2 pi k / n.
void gauss_hat_1d(std::vector<double> &out, int n, double sigma, double centre) {
  const int A = alias_count(sigma);
  out.assign(n, 0.0);
  for (int k = 0; k < n; ++k) {
    double s = 0.0;
    for (int a = -A; a <= A; ++a) {
      double w = 2.0 * kPi * (static_cast<double>(k) + static_cast<double>(a) * n) / n - centre;
      double e = -0.5 * sigma * sigma * w * w;
      if (e >= kMinExponent) s += std::exp(e);
    }
    out[k] = s;
  }
}

void morlet_hat_1d(std::vector<double> &out, int n, double sigma, double xi) {
  std::vector<double> gab, env;
  gauss_hat_1d(gab, n, sigma, xi);
  gauss_hat_1d(env, n, sigma, 0.0);
  const double kappa = gab[0] / env[0];
  out.resize(n);
  for (int k = 0; k < n; ++k) out[k] = gab[k] - kappa * env[k];
  out[0] = 0.0;
}

// Sum the 2^r x 2^r (2-D) or 2^r (1-D, n_r == 1) Fourier blocks.
void fold_table(const FilterTable &src, int r, FilterTable &dst) {
  const int rr = src.n_r > 1 ? r : 0;
  dst.n_r = src.n_r >> rr;
  dst.n_c = src.n_c >> r;
  dst.v.assign(static_cast<size_t>(dst.n_r) * dst.n_c, 0.0);
  for (int kr = 0; kr < src.n_r; ++kr)
    for (int kc = 0; kc < src.n_c; ++kc)
      dst.v[static_cast<size_t>(kr % dst.n_r) * dst.n_c + (kc % dst.n_c)] +=
          src.v[static_cast<size_t>(kr) * src.n_c + kc];
}

void fold_1d(const std::vector<double> &src, int r, std::vector<double> &dst) {
  const size_t m = src.size() >> r;
  dst.assign(m, 0.0);
  for (size_t k = 0; k < src.size(); ++k) dst[k % m] += src[k];
}

}  // namespace

const FilterTable *HostPlan::find(int kind, int idx, int res) const {
  // In 2-D the two wavelet banks coincide, so a second-order table at resolution 0 is
  // the first-order table.
  if (dims == 2 && kind == 2 && res == 0) kind = 1;
  for (const FilterTable &t : filters)
    if (t.kind == kind && t.res == res && (kind == 0 || t.index == idx)) return &t;
  return nullptr;
}

int validate(int dims, const int *shape, int J, int LQ, int max_order) {
  if (dims != 1 && dims != 2) return 1;
  if (J < 1 || J > 24 || LQ < 1 || LQ > 64) return 1;
  if (max_order != 1 && max_order != 2) return 1;
  for (int d = 0; d < dims; ++d) {
    if (!is_pow2(shape[d])) return 2;
    if (shape[d] < (1 << J)) return 2;
    // one row or column of a transform must fit a workgroup's LDS tile (4096 points);
    // a 1-D signal is handled as a matrix with both sides at most 4096
    if (shape[d] > (dims == 2 ? 4096 : (1 << 24))) return 2;
  }
  if (dims == 1 && J > 12) return 1;
  return 0;
}

void build_host_plan(HostPlan &p, int dims, const int *shape, int J, int LQ, int max_order) {
  p.dims = dims;
  p.J = J;
  p.LQ = LQ;
  p.max_order = max_order;
  if (dims == 2) {
    p.shape[0] = shape[0];
    p.shape[1] = shape[1];
  } else {
    p.shape[0] = 1;
    p.shape[1] = shape[0];
  }
  const int n_r = p.shape[0], n_c = p.shape[1];

  // ---- index table: S0, S1 by (j1, t1), S2 by (j1, t1, j2, t2) with j2 > j1
  p.index.clear();
  p.index.push_back({0, -1, -1, -1, -1});
  const int n_first = J * LQ;  // 2-D: J*L (j, theta); 1-D: J*Q wavelets
  for (int k = 0; k < n_first; ++k) {
    int j1 = k / LQ;
    p.index.push_back({1, j1, dims == 2 ? k % LQ : k, -1, -1});
  }
  if (max_order == 2) {
    for (int k = 0; k < n_first; ++k) {
      int j1 = k / LQ;
      for (int j2 = j1 + 1; j2 < J; ++j2) {
        if (dims == 2) {
          for (int t2 = 0; t2 < LQ; ++t2) p.index.push_back({2, j1, k % LQ, j2, t2});
        } else {
          p.index.push_back({2, j1, k, j2, j2});
        }
      }
    }
  }
  p.K = static_cast<int>(p.index.size());

  // ---- filters
  p.filters.clear();
  const double sigma_low = 0.8 * std::ldexp(1.0, J);
  if (dims == 2) {
    const double slant = 4.0 / LQ;
    // first-order (= second-order) bank at full resolution
    for (int j = 0; j < J; ++j)
      for (int l = 0; l < LQ; ++l) {
        FilterTable t;
        t.kind = 1;
        t.index = j * LQ + l;
        t.res = 0;
        t.n_r = n_r;
        t.n_c = n_c;
        morlet_hat_2d(t.v, n_r, n_c, 0.8 * std::ldexp(1.0, j), 0.75 * kPi * std::ldexp(1.0, -j),
                      kPi * l / LQ, slant);
        p.filters.push_back(std::move(t));
      }
    if (max_order == 2) {
      for (int j2 = 1; j2 < J; ++j2)
        for (int l = 0; l < LQ; ++l)
          for (int r = 1; r < j2; ++r) {
            FilterTable t;
            t.kind = 2;
            t.index = j2 * LQ + l;
            t.res = r;
            fold_table(*p.find(1, j2 * LQ + l, 0), r, t);
            p.filters.push_back(std::move(t));
          }
    }
    // lowpass: separable factors per axis, folded to each resolution; also the 2-D product
    std::vector<double> row0, col0;
    gauss_hat_1d(row0, n_r, sigma_low, 0.0);
    gauss_hat_1d(col0, n_c, sigma_low, 0.0);
    p.phi_rows.assign(J, {});
    p.phi_cols.assign(J, {});
    for (int r = 0; r < J; ++r) {
      fold_1d(row0, r, p.phi_rows[r]);
      fold_1d(col0, r, p.phi_cols[r]);
      FilterTable t;
      t.kind = 0;
      t.index = 0;
      t.res = r;
      t.n_r = n_r >> r;
      t.n_c = n_c >> r;
      t.v.resize(static_cast<size_t>(t.n_r) * t.n_c);
      for (int a = 0; a < t.n_r; ++a)
        for (int b = 0; b < t.n_c; ++b)
          t.v[static_cast<size_t>(a) * t.n_c + b] = p.phi_rows[r][a] * p.phi_cols[r][b];
      p.filters.push_back(std::move(t));
    }
  } else {
    const int Q = LQ;
    for (int k = 0; k < J * Q; ++k) {
      double xi = 0.75 * kPi * std::exp2(-static_cast<double>(k) / Q);
      double sigma = Q == 1 ? 0.8 * std::ldexp(1.0, k)
                            : 0.3 * kPi / (xi * (1.0 - std::exp2(-1.0 / Q)));
      FilterTable t;
      t.kind = 1;
      t.index = k;
      t.res = 0;
      t.n_r = 1;
      t.n_c = n_c;
      morlet_hat_1d(t.v, n_c, sigma, xi);
      p.filters.push_back(std::move(t));
    }
    if (max_order == 2) {
      for (int j2 = 1; j2 < J; ++j2) {
        FilterTable full;
        full.kind = 2;
        full.index = j2;
        full.res = 0;
        full.n_r = 1;
        full.n_c = n_c;
        morlet_hat_1d(full.v, n_c, 0.8 * std::ldexp(1.0, j2), 0.75 * kPi * std::ldexp(1.0, -j2));
        for (int r = 1; r < j2; ++r) {
          FilterTable t;
          t.kind = 2;
          t.index = j2;
          t.res = r;
          fold_table(full, r, t);
          p.filters.push_back(std::move(t));
        }
        p.filters.push_back(std::move(full));
      }
    }
    FilterTable low;
    low.kind = 0;
    low.index = 0;
    low.res = 0;
    low.n_r = 1;
    low.n_c = n_c;
    gauss_hat_1d(low.v, n_c, sigma_low, 0.0);
    for (int r = 1; r < J; ++r) {
      FilterTable t;
      t.kind = 0;
      t.index = 0;
      t.res = r;
      fold_table(low, r, t);
      p.filters.push_back(std::move(t));
    }
    p.filters.push_back(std::move(low));
  }
}

}  // namespace scat
