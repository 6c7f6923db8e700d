// Host-side core of the scattering library: argument validation, coefficient index
// table, filter-bank construction in fp64 from analytic Fourier transforms.
// Nothing in this file touches the GPU.
#pragma once

#include <cstddef>
#include <atomic>
#include <thread>
#include <vector>

namespace scat {

struct CoeffRow {
  int order, j1, t1, j2, t2;
};

// One filter's Fourier samples at one resolution, natural frequency order, unscaled.
struct FilterTable {
  int kind;   // 0 lowpass, 1 first-order wavelet, 2 second-order wavelet
  int index;  // 2-D: j*L + theta; 1-D: wavelet number; lowpass: 0
  int res;    // resolution: grid = shape >> res
  int n_r;    // rows (1 in 1-D)
  int n_c;    // columns (length in 1-D)
  std::vector<double> v;
};

struct HostPlan {
  int dims = 0;
  int shape[2] = {1, 1};  // 1-D: shape[0] = 1 rows, shape[1] = N
  int J = 0, LQ = 0, max_order = 0;
  // Oversampling o: after a wavelet of octave j the grid is shape >> res(j) with
  // res(j) = max(j - o, 0); the output grid is shape >> res(J).  o = 0: critical schedule.
  int oversampling = 0;
  int res(int j) const { return j > oversampling ? j - oversampling : 0; }
  int K = 0;
  std::vector<CoeffRow> index;
  std::vector<FilterTable> filters;
  // 2-D only: the separable factors of the lowpass, phi_hat[k_r, k_c] = row[k_r] * col[k_c],
  // folded to each resolution r = 0 .. J-1 (unscaled).
  std::vector<std::vector<double>> phi_rows, phi_cols;

  const FilterTable *find(int kind, int index, int res) const;
};

// Returns 0 on success, else a scat_status value (1 = bad argument, 2 = bad shape).
int validate(int dims, const int *shape, int J, int LQ, int max_order);

// Fills every field of `p` (validate() must have passed).
void build_host_plan(HostPlan &p, int dims, const int *shape, int J, int LQ, int max_order);

// Number of second-order wavelets below first-order octave j1, i.e. octaves j1+1 .. J-1.
inline int num_children_octaves(int J, int j1) { return J - 1 - j1; }

// Runs body(i) for i in [0, count) on up to 16 host threads (the tables of large volumes
// take seconds on one).
template <class Fn>
inline void parallel_for(int count, Fn body) {
  unsigned hw = std::thread::hardware_concurrency();
  int workers = static_cast<int>(hw == 0 ? 1 : hw > 16 ? 16 : hw);
  if (workers > count) workers = count;
  if (workers <= 1) {
    for (int i = 0; i < count; ++i) body(i);
    return;
  }
  std::atomic<int> next(0);
  std::vector<std::thread> pool;
  auto work = [&] {
    for (int i = next.fetch_add(1); i < count; i = next.fetch_add(1)) body(i);
  };
  try {
    for (int w = 1; w < workers; ++w) pool.emplace_back(work);
  } catch (...) {
    // could not start every thread: the ones that run, and this one, finish the job
  }
  work();
  for (std::thread &t : pool) t.join();
}


}  // namespace scat
