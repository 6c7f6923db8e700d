// 3-D solid harmonic scattering (paper section 2: wavelets psi_{j,l,m}, non-linearity
// rho = sqrt(sum_m |x conv psi_{j,l,m}|^2)), evaluated as the definition states it: every
// convolution on the full periodic grid through 3-D FFTs, the lowpassed result read at
// the samples 2^J n.  A 3-D transform is three passes of the plain in-place transforms of
// the backward pass (last axis as rows, the other two as columns); the pointwise steps
// are the small kernels below.
#include <hip/hip_runtime.h>

#include "scat_kernels.hpp"

namespace scat {

namespace {

unsigned blocks_for(long total) {
  long b = (total + 255) / 256;
  if (b > 65536 * 16) b = 65536 * 16;
  return static_cast<unsigned>(b < 1 ? 1 : b);
}

__global__ __launch_bounds__(256) void k3_real_to_complex(const float *__restrict__ x,
                                                          float2 *__restrict__ out, long total) {
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride)
    out[i] = make_float2(x[i], 0.f);
}

// dst[v][e] = src[v][e] * filt[e]: one real table applied to every volume of the batch
__global__ __launch_bounds__(256) void k3_mul_table(const float2 *__restrict__ src,
                                                    const float *__restrict__ filt,
                                                    float2 *__restrict__ dst, long total, long n) {
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const float f = filt[i % n];
    const float2 v = src[i];
    dst[i] = make_float2(v.x * f, v.y * f);
  }
}

// acc[i] (+)= |y[i]|^2
__global__ __launch_bounds__(256) void k3_accum_abs2(const float2 *__restrict__ y,
                                                     float *__restrict__ acc, long total,
                                                     int first) {
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const float2 v = y[i];
    const float p = v.x * v.x + v.y * v.y;
    acc[i] = first ? p : acc[i] + p;
  }
}

// out[i] = (sqrt(acc[i]), 0)
__global__ __launch_bounds__(256) void k3_sqrt(const float *__restrict__ acc,
                                               float2 *__restrict__ out, long total) {
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride)
    out[i] = make_float2(__builtin_amdgcn_sqrtf(acc[i]), 0.f);
}

// out[v][chan][a][b][c] = Re src[v][a s][b s][c s], s = 2^J
__global__ __launch_bounds__(256) void k3_sample(const float2 *__restrict__ src,
                                                 float *__restrict__ out, long volumes, int K,
                                                 int chan, int n0, int n1, int n2, int J) {
  const int m0 = n0 >> J, m1 = n1 >> J, m2 = n2 >> J;
  const long per = static_cast<long>(m0) * m1 * m2;
  const long total = volumes * per;
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const long v = i / per;
    long e = i - v * per;
    const int c = static_cast<int>(e % m2);
    e /= m2;
    const int b = static_cast<int>(e % m1);
    const int a = static_cast<int>(e / m1);
    const size_t s = ((static_cast<size_t>(v) * n0 + (static_cast<size_t>(a) << J)) * n1 +
                      (static_cast<size_t>(b) << J)) * n2 + (static_cast<size_t>(c) << J);
    out[(static_cast<size_t>(v) * K + chan) * per + (static_cast<size_t>(a) * m1 + b) * m2 + c] = src[s].x;
  }
}

}  // namespace

hipError_t launch3_fft(float2 *data, long volumes, int n0, int n1, int n2, bool inverse,
                       const float2 *tw, int tw_n, hipStream_t st) {
  hipError_t e = launch_fft_rows_inplace(data, volumes * n0 * n1, n2, inverse, tw, tw_n, st);
  if (e != hipSuccess) return e;
  e = launch_fft_cols_inplace(data, volumes * n0, n1, n2, inverse, tw, tw_n, st);
  if (e != hipSuccess) return e;
  return launch_fft_cols_inplace(data, volumes, n0, n1 * n2, inverse, tw, tw_n, st);
}

hipError_t launch3_real_to_complex(const float *x, float2 *out, long total, hipStream_t st) {
  if (total <= 0) return hipSuccess;
  LaunchScope obs("k3_real_to_complex", total * 12.0, 0.0, st);
  hipLaunchKernelGGL(k3_real_to_complex, dim3(blocks_for(total)), dim3(256), 0, st, x, out, total);
  return hipGetLastError();
}

hipError_t launch3_mul_table(const float2 *src, const float *filt, float2 *dst, long volumes, long n,
                             hipStream_t st) {
  const long total = volumes * n;
  if (total <= 0) return hipSuccess;
  LaunchScope obs("k3_mul_table", total * 16.0 + n * 4.0, total * 2.0, st);
  hipLaunchKernelGGL(k3_mul_table, dim3(blocks_for(total)), dim3(256), 0, st, src, filt, dst, total,
                     n);
  return hipGetLastError();
}

hipError_t launch3_accum_abs2(const float2 *y, float *acc, long total, bool first, hipStream_t st) {
  if (total <= 0) return hipSuccess;
  LaunchScope obs("k3_accum_abs2", total * (first ? 12.0 : 16.0), total * 4.0, st);
  hipLaunchKernelGGL(k3_accum_abs2, dim3(blocks_for(total)), dim3(256), 0, st, y, acc, total,
                     first ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch3_sqrt(const float *acc, float2 *out, long total, hipStream_t st) {
  if (total <= 0) return hipSuccess;
  LaunchScope obs("k3_sqrt", total * 12.0, total * 1.0, st);
  hipLaunchKernelGGL(k3_sqrt, dim3(blocks_for(total)), dim3(256), 0, st, acc, out, total);
  return hipGetLastError();
}

hipError_t launch3_sample(const float2 *src, float *out, long volumes, int K, int chan, int n0,
                          int n1, int n2, int J, hipStream_t st) {
  const long total = volumes * (n0 >> J) * (n1 >> J) * (n2 >> J);
  if (total <= 0) return hipSuccess;
  LaunchScope obs("k3_sample", total * 12.0, 0.0, st);
  hipLaunchKernelGGL(k3_sample, dim3(blocks_for(total)), dim3(256), 0, st, src, out, volumes, K, chan,
                     n0, n1, n2, J);
  return hipGetLastError();
}

}  // namespace scat
