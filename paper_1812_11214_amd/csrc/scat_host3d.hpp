// Host-side core of the 3-D solid harmonic scattering plans: validation, coefficient
// index table and the filter bank (fp64, analytic Fourier transforms).  Nothing in this
// file touches the GPU.
#pragma once

#include <vector>

namespace scat {

struct Coeff3D {
  int order, j1, l, j2;
};

// Section 2 of the paper: solid harmonic wavelets psi_{j,l,m} and the non-linearity
// rho = sqrt(sum_m |x conv psi_{j,l,m}|^2).  The modulus makes the result independent of
// the orthonormal basis chosen for the degree-l harmonics and of any unit factor, so the
// tables hold REAL functions: r^l exp(-r^2/2) times real spherical harmonics, evaluated at
// w = 2^j (omega + 2 pi a), r = |w|, and summed over the aliases a (the Fourier transform
// of the wavelet sampled at the integers), in natural frequency order, unscaled.
struct HostPlan3D {
  int shape[3] = {1, 1, 1};
  int J = 0, L = 0, max_order = 0;
  int K = 0;
  int oversampling = 0;  // the outputs are read at the samples 2^out_shift() n
  int out_shift() const { return J > oversampling ? J - oversampling : 0; }
  std::vector<Coeff3D> index;
  // psi[(j * (L+1) + l)] = (2l+1) tables of shape[0]*shape[1]*shape[2] doubles, m-major
  std::vector<std::vector<double>> psi;
  std::vector<double> phi;  // Gaussian lowpass, std 2^J, unit mass, same layout
  size_t points() const { return static_cast<size_t>(shape[0]) * shape[1] * shape[2]; }
};

// 0 on success, else a scat_status value (1 = bad argument, 2 = bad shape).
int validate_3d(const int *shape, int J, int L, int max_order);
void build_host_plan_3d(HostPlan3D &p, const int *shape, int J, int L, int max_order);

}  // namespace scat
