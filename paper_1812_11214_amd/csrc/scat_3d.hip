// 3-D solid harmonic scattering (paper section 2: wavelets psi_{j,l,m}, non-linearity
// rho = sqrt(sum_m |x conv psi_{j,l,m}|^2)), evaluated as the definition states it: every
// convolution on the full periodic grid through 3-D FFTs, the lowpassed result read at
// the samples 2^J n.  A 3-D transform is three passes of the plain in-place transforms of
// the backward pass (last axis as rows, the other two as columns); the pointwise steps
// are the small kernels below.
#include <hip/hip_runtime.h>

#include <string>

#include "fft_regs.hpp"
#include "slab_fft.hpp"
#include "scat_kernels.hpp"

namespace scat {

namespace {

int ilog2h(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}

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

// dst[v][e] (+)= src[v][e] * filt[e * fstride]: one real table applied to every volume of the
// batch (fstride = 2 reads one member of a table pair stored as complex numbers)
__global__ __launch_bounds__(256) void k3_mul_table(const float2 *__restrict__ src,
                                                    const float *__restrict__ filt, int fstride,
                                                    float2 *__restrict__ dst, long total, long n,
                                                    int accumulate) {
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const float f = filt[(i % n) * fstride];
    const float2 v = src[i];
    float2 o = make_float2(v.x * f, v.y * f);
    if (accumulate) {
      const float2 d = dst[i];
      o.x += d.x;
      o.y += d.y;
    }
    dst[i] = o;
  }
}

// dst[v][k] (+)= phi[k] * Gs[v][chan][k mod m]: the spectrum of the zero-inserted output
// gradient is the small spectrum Gs tiled over the grid (adjoint of lowpass + subsampling)
__global__ __launch_bounds__(256) void k3_tile_phi(const float2 *__restrict__ Gs,
                                                   const float *__restrict__ phi,
                                                   float2 *__restrict__ dst, long volumes, int K,
                                                   int chan, int n0, int n1, int n2, int J,
                                                   int accumulate) {
  const long per = static_cast<long>(n0) * n1 * n2;
  const long total = volumes * per;
  const int m0 = n0 >> J, m1 = n1 >> J, m2 = n2 >> J;
  const long mper = static_cast<long>(m0) * m1 * m2;
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const long v = i / per;
    long e = i - v * per;
    const int c = static_cast<int>(e % n2);
    const long e1 = e / n2;
    const int b = static_cast<int>(e1 % n1);
    const int a = static_cast<int>(e1 / n1);
    const float2 gs = Gs[(static_cast<size_t>(v) * K + chan) * mper +
                         (static_cast<size_t>(a & (m0 - 1)) * m1 + (b & (m1 - 1))) * m2 + (c & (m2 - 1))];
    const float f = phi[e];
    float2 o = make_float2(gs.x * f, gs.y * f);
    if (accumulate) {
      const float2 d = dst[i];
      o.x += d.x;
      o.y += d.y;
    }
    dst[i] = o;
  }
}

// dst[v][e] (+)= src[v][e] * c[e] (or conj(c[e])): a pair of real tables stored as one complex
__global__ __launch_bounds__(256) void k3_mul_ctable(const float2 *__restrict__ src,
                                                     const float2 *__restrict__ ctab,
                                                     float2 *__restrict__ dst, long total, long n,
                                                     int conj_table, int accumulate) {
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    float2 c = ctab[i % n];
    if (conj_table) c.y = -c.y;
    float2 o = c_mul(src[i], c);
    if (accumulate) {
      const float2 d = dst[i];
      o.x += d.x;
      o.y += d.y;
    }
    dst[i] = o;
  }
}

// y[i] <- Re(gu[i]) * y[i] / sqrt(acc[i])  (0 where acc = sum_m |y_m|^2 vanishes): the
// gradient of rho = sqrt(sum_m |y_m|^2) with respect to y_m, given the gradient of rho
__global__ __launch_bounds__(256) void k3_rho_back(const float2 *__restrict__ gu,
                                                   const float *__restrict__ acc,
                                                   float2 *__restrict__ y, long total) {
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const float a = acc[i];
    const float s = over_sqrt(gu[i].x, a);
    const float2 v = y[i];
    y[i] = make_float2(v.x * s, v.y * s);
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


// ---- fused passes for volumes whose (axis 1, axis 2) slabs fit a workgroup's LDS --------
// (slabs of up to 4096 points: 256 threads and 1 to 16 slabs per workgroup; 8192 and 16384
// points: one slab per workgroup of 512 or 1024 threads and up to 152 KB of LDS)
//
// A 3-D transform is split into the two slab axes (one workgroup holds whole N1 x N2
// slabs: rows through registers, a transposition through LDS, columns through registers)
// and axis 0 (columns of stride N1*N2).  Around them:
//   k3_slab_mul_inv   W_p = inverse transform over the slab axes of F^ (g_2p + i g_2p+1), all
//                     pairs of one (j, l) in one launch (the slab of F^ is read once).  The
//                     signal F is real and the tables g_m are real with the parity of l, so
//                     F conv g_m is real (l even) or imaginary (l odd) and one complex
//                     transform carries two of them: |W_p|^2 = |F conv g_2p|^2 +
//                     |F conv g_2p+1|^2, which is all the non-linearity needs
//   k3_axis0_rho      inverse transform along axis 0 of every W_m, sum of squared moduli in
//                     registers, square root, forward transform along axis 0; the result T
//                     is the axis-0 spectrum of a real signal: rows 0 .. n0/2 are stored
//   k3_slab_fwd_low   forward transform over the slab axes of those rows (giving U^ for
//                     k0 <= n0/2 and, by conjugate symmetry, for n0 - k0), product with the
//                     lowpass and the sum over the aliases of the slab axes (periodic
//                     subsampling by 2^J seen from the Fourier side)
//   k3_fold0          the aliases of axis 0; the small inverse transforms then give S

template <int N1, int N2, bool SPLIT>
__global__ __launch_bounds__((Slab<N1, N2>::NT)) void k3_slab_mul_inv(const float2 *__restrict__ Fh,
                                                       const float2 *__restrict__ tab,
                                                       float2 *__restrict__ W, long slabs, int n0,
                                                       int M, size_t mstride,
                                                       const float2 *__restrict__ tw, int tw_n) {
  using S = Slab<N1, N2>;
  extern __shared__ float2 lds[];
  const int s = threadIdx.x / S::TS, q = threadIdx.x % S::TS;
  const long slab = static_cast<long>(blockIdx.x) * S::SPW + s;
  const bool live = slab < slabs;
  const long sl = live ? slab : slabs - 1;  // idle threads shadow the last slab, store nothing
  float2 *area = lds + s * N1 * S::RS;
  const int r = q / S::T2, t = q % S::T2;
  const int c = q % N2, t1 = q / N2;
  const int k0 = static_cast<int>(sl % n0);
  const size_t base = static_cast<size_t>(sl) * N1 * N2;
  const float2 *src = Fh + base + r * N2 + t;
  // the slab of F^ stays in registers across the filters; the 1024-thread variants (128
  // registers per thread) instead take one filter per workgroup and read it again
  constexpr bool KEEP = !SPLIT;
  float2 f[KEEP ? 16 : 1];
  if (KEEP) {
#pragma unroll
    for (int i = 0; i < 16; ++i) f[KEEP ? i : 0] = src[S::T2 * i];
  }
  // SPLIT: one filter per workgroup (blockIdx.y), no loop state to carry
  const int m_first = SPLIT ? static_cast<int>(blockIdx.y) : 0, m_last = SPLIT ? m_first + 1 : M;
  for (int m = m_first; m < m_last; ++m) {
    const float2 *tb = tab + (static_cast<size_t>(m) * n0 + k0) * N1 * N2 + r * N2 + t;
    float2 v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      v[i] = c_mul(KEEP ? f[KEEP ? i : 0] : src[S::T2 * i], tb[S::T2 * i]);
      // two batches of loads, so that the operands in flight fit
      if (!KEEP && i == 7) __builtin_amdgcn_sched_barrier(0);
    }
    S::template transform<true>(v, area, r, t, c, t1, tw, tw_n);
    if (live) {
      float2 *dst = W + static_cast<size_t>(m) * mstride + base + c;
#pragma unroll
      for (int i = 0; i < 16; ++i) dst[(t1 + S::T1 * i) * N2] = v[i];
    }
    if (!SPLIT) __syncthreads();  // the slab area is reused by the next filter
  }
}

// Tin holds slabs k0 = 0 .. n0/2 only (the axis-0 spectrum of a real signal); the slab
// n0 - k0 of U^ and of the folded lowpass product is the conjugate of slab k0 with both
// slab indices negated, and is written from the same registers.
template <int N1, int N2>
__global__ __launch_bounds__((Slab<N1, N2>::NT)) void k3_slab_fwd_low(const float2 *__restrict__ Tin,
                                                       float2 *__restrict__ Uout,
                                                       const float *__restrict__ phi,
                                                       float2 *__restrict__ P, long slabs, int n0,
                                                       int J, size_t p_vol_stride, size_t chan_off,
                                                       const float2 *__restrict__ tw, int tw_n) {
  using S = Slab<N1, N2>;
  extern __shared__ float2 lds[];
  const int s = threadIdx.x / S::TS, q = threadIdx.x % S::TS;
  const long slab = static_cast<long>(blockIdx.x) * S::SPW + s;
  const bool live = slab < slabs;
  const long sl = live ? slab : slabs - 1;
  float2 *area = lds + s * N1 * S::RS;
  const int r = q / S::T2, t = q % S::T2;
  const int c = q % N2, t1 = q / N2;
  const int H = n0 / 2 + 1;
  const int k0 = static_cast<int>(sl % H);
  const long vol = sl / H;
  const bool twin = k0 > 0 && k0 < n0 - k0;  // slab n0 - k0 is a different slab
  const float2 *src = Tin + static_cast<size_t>(sl) * N1 * N2 + r * N2 + t;
  float2 v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = src[S::T2 * i];
  S::template transform<false>(v, area, r, t, c, t1, tw, tw_n);
  if (Uout != nullptr && live) {
    float2 *dst = Uout + (static_cast<size_t>(vol) * n0 + k0) * N1 * N2 + c;
#pragma unroll
    for (int i = 0; i < 16; ++i) dst[(t1 + S::T1 * i) * N2] = v[i];
    if (twin) {
      float2 *dm = Uout + (static_cast<size_t>(vol) * n0 + (n0 - k0)) * N1 * N2 + ((N2 - c) & (N2 - 1));
#pragma unroll
      for (int i = 0; i < 16; ++i)
        dm[((N1 - (t1 + S::T1 * i)) & (N1 - 1)) * N2] = make_float2(v[i].x, -v[i].y);
    }
  }
  // lowpass product, then the sum over the 4^J aliases of the slab axes
  const float *ph = phi + static_cast<size_t>(k0) * N1 * N2 + c;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const float g = ph[(t1 + S::T1 * i) * N2];
    area[(t1 + S::T1 * i) * S::RS + c] = make_float2(v[i].x * g, v[i].y * g);
  }
  __syncthreads();
  const int m1 = N1 >> J, m2 = N2 >> J, al = 1 << J;
  if (!live) return;
  float2 *pv = P + static_cast<size_t>(vol) * p_vol_stride + chan_off;
  float2 *dst = pv + static_cast<size_t>(k0) * m1 * m2;
  float2 *dm = pv + static_cast<size_t>(n0 - k0) * m1 * m2;
  for (int o = q; o < m1 * m2; o += S::TS) {
    const int a = o / m2, b = o - a * m2;
    float2 acc = make_float2(0.f, 0.f);
    for (int p1 = 0; p1 < al; ++p1)
      for (int p2 = 0; p2 < al; ++p2) {
        const float2 e = area[(a + m1 * p1) * S::RS + b + m2 * p2];
        acc.x += e.x;
        acc.y += e.y;
      }
    dst[o] = acc;
    if (twin) dm[((m1 - a) & (m1 - 1)) * m2 + ((m2 - b) & (m2 - 1))] = make_float2(acc.x, -acc.y);
  }
}

// Axis 0 of [volumes][E*T][Mc]: a workgroup takes TC columns of one volume, thread (t, c)
// holds rows t + T i.  xreal != nullptr: forward transform of the real input.  Else: inverse
// transform of the M signals W_m, root of the sum of their squared moduli, forward transform.
// The transformed signal is real, so only rows 0 .. N0/2 of its spectrum are stored:
// dst [volumes][N0/2 + 1][Mc].
template <int E, int T>
__global__ __launch_bounds__(256) void k3_axis0_rho(const float2 *__restrict__ W,
                                                    const float *__restrict__ xreal,
                                                    float2 *__restrict__ dst, int Mc, int TC, int M,
                                                    size_t mstride, const float2 *__restrict__ tw,
                                                    int tw_n) {
  constexpr int N0 = E * T;
  extern __shared__ float2 lds[];
  const int KS = T * TC + (E == 32 ? 0 : 1);
  const int c = threadIdx.x % TC, t = threadIdx.x / TC;
  const int tiles = Mc / TC;
  const long vol = blockIdx.x / tiles;
  const int c0 = static_cast<int>(blockIdx.x % tiles) * TC;
  const size_t off = static_cast<size_t>(vol) * N0 * Mc + static_cast<size_t>(t) * Mc + c0 + c;
  const size_t step = static_cast<size_t>(T) * Mc;
  float2 wt[E];
  load_twiddles<E, T>(wt, t, tw, tw_n);
  float2 v[E];
  if (xreal != nullptr) {
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = make_float2(xreal[off + i * step], 0.f);
  } else {
    float acc[E];
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = 0.f;
    for (int m = 0; m < M; ++m) {
      const float2 *p = W + static_cast<size_t>(m) * mstride + off;
#pragma unroll
      for (int i = 0; i < E; ++i) v[i] = p[i * step];
      fft_core<E, T, true, false>(v, t, lds + c, KS, TC, wt);
#pragma unroll
      for (int i = 0; i < E; ++i) acc[i] += v[i].x * v[i].x + v[i].y * v[i].y;
    }
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = make_float2(__builtin_amdgcn_sqrtf(acc[i]), 0.f);
  }
  fft_core<E, T, false, false>(v, t, lds + c, KS, TC, wt);
  float2 *o = dst + static_cast<size_t>(vol) * (N0 / 2 + 1) * Mc + static_cast<size_t>(t) * Mc + c0 + c;
#pragma unroll
  for (int i = 0; i < E; ++i)
    if (t + T * i <= N0 / 2) o[i * step] = v[i];
}

// Backward pass, axis 0 of the P signals W_p [volumes][E*T][Mc] (in place).
// MODE 0: inverse transform of every W_p (the slab axes are already done), written back as
//         the filtered signals y_p, and acc = sum_p |y_p|^2.
// MODE 1: y_p <- Re(gu) y_p / sqrt(acc) (0 where acc = 0), then the forward transform.
template <int E, int T, int MODE>
__global__ __launch_bounds__(256) void k3_axis0_back(float2 *__restrict__ W, float *__restrict__ acc,
                                                     const float2 *__restrict__ gu, int Mc, int TC,
                                                     int P, size_t mstride,
                                                     const float2 *__restrict__ tw, int tw_n) {
  constexpr int N0 = E * T;
  extern __shared__ float2 lds[];
  const int KS = T * TC + (E == 32 ? 0 : 1);
  const int c = threadIdx.x % TC, t = threadIdx.x / TC;
  const int tiles = Mc / TC;
  const long vol = blockIdx.x / tiles;
  const int c0 = static_cast<int>(blockIdx.x % tiles) * TC;
  const size_t off = static_cast<size_t>(vol) * N0 * Mc + static_cast<size_t>(t) * Mc + c0 + c;
  const size_t step = static_cast<size_t>(T) * Mc;
  // The transforms' twiddles in an LDS table behind the exchange area (wtab[k T + t]); the
  // registers they would take hold the next signal's values, requested before the current
  // signal is transformed (otherwise they would queue behind its stores).
  constexpr bool TAB = T > 1;
  float2 *wtab = lds + E * KS;
  if (TAB) {
    for (int idx = threadIdx.x; idx < N0; idx += blockDim.x)
      wtab[idx] = tw[(idx / T) * (idx % T) * (tw_n / N0)];
    __syncthreads();
  }
  float a[E];
#pragma unroll
  for (int i = 0; i < E; ++i) {
    if (MODE == 0) {
      a[i] = 0.f;
    } else {
      const float s2 = acc[off + i * step];
      a[i] = over_sqrt(gu[off + i * step].x, s2);
    }
  }
  float2 vn[E];
  auto fetch = [&](int p) {
    const float2 *w = W + static_cast<size_t>(p) * mstride + off;
#pragma unroll
    for (int i = 0; i < E; ++i) vn[i] = w[i * step];
  };
  fetch(0);
  for (int p = 0; p < P; ++p) {
    float2 *w = W + static_cast<size_t>(p) * mstride + off;
    float2 v[E];
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = vn[i];
    if (p + 1 < P) fetch(p + 1);
    if (MODE == 0) {
      fft_core_tab<E, T, true, false>(v, t, lds + c, KS, TC, wtab + t, T);
#pragma unroll
      for (int i = 0; i < E; ++i) a[i] += v[i].x * v[i].x + v[i].y * v[i].y;
    } else {
#pragma unroll
      for (int i = 0; i < E; ++i) v[i] = make_float2(v[i].x * a[i], v[i].y * a[i]);
      fft_core_tab<E, T, false, false>(v, t, lds + c, KS, TC, wtab + t, T);
    }
#pragma unroll
    for (int i = 0; i < E; ++i) w[i * step] = v[i];
  }
  if (MODE == 0) {
#pragma unroll
    for (int i = 0; i < E; ++i) acc[off + i * step] = a[i];
  }
}

// Backward pass, slab axes: A[slab] += sum_p conj(c_p) * (forward slab transform of W_p), the
// adjoint of k3_slab_mul_inv (c_p = the pair tables of the node); A's slab is read and
// written once for all p.
template <int N1, int N2>
__global__ __launch_bounds__((Slab<N1, N2>::NT)) void k3_slab_fwd_mulacc(
    const float2 *__restrict__ W, const float2 *__restrict__ tab, float2 *__restrict__ A, long slabs,
    int n0, int P, size_t mstride, const float2 *__restrict__ tw, int tw_n) {
  using S = Slab<N1, N2>;
  extern __shared__ float2 lds[];
  const int s = threadIdx.x / S::TS, q = threadIdx.x % S::TS;
  const long slab = static_cast<long>(blockIdx.x) * S::SPW + s;
  const bool live = slab < slabs;
  const long sl = live ? slab : slabs - 1;
  float2 *area = lds + s * N1 * S::RS;
  const int r = q / S::T2, t = q % S::T2;
  const int c = q % N2, t1 = q / N2;
  const int k0 = static_cast<int>(sl % n0);
  const size_t base = static_cast<size_t>(sl) * N1 * N2;
  // the transforms' twiddles in LDS tables: their registers go to the table values, which
  // are requested before the transform they are used after
  float2 *wtab = lds + S::SPW * N1 * S::RS;
  S::fill_twiddles(wtab, tw, tw_n);
  float2 sum[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) sum[i] = make_float2(0.f, 0.f);
  for (int p = 0; p < P; ++p) {
    const float2 *src = W + static_cast<size_t>(p) * mstride + base + r * N2 + t;
    float2 v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = src[S::T2 * i];
    const float2 *tb = tab + (static_cast<size_t>(p) * n0 + k0) * N1 * N2 + c;
    float2 gt[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) gt[i] = tb[(t1 + S::T1 * i) * N2];
    S::template transform_tab<false>(v, area, r, t, c, t1, wtab);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      float2 g = gt[i];
      g.y = -g.y;
      const float2 o = c_mul(v[i], g);
      sum[i].x += o.x;
      sum[i].y += o.y;
    }
    __syncthreads();  // the slab area is reused by the next signal
  }
  if (!live) return;
  float2 *dst = A + base + c;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    float2 *d = dst + (t1 + S::T1 * i) * N2;
    const float2 old = *d;
    *d = make_float2(old.x + sum[i].x, old.y + sum[i].y);
  }
}

// Q[g][a0][e] = sum_p P[g][a0 + m0 p][e]: g over volumes x channels, e over the m1*m2
// folded slab points
__global__ __launch_bounds__(256) void k3_fold0(const float2 *__restrict__ P,
                                                float2 *__restrict__ Q, long groups, int n0, int m0,
                                                int slab) {
  const long per = static_cast<long>(m0) * slab;
  const long total = groups * per;
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const long g = i / per;
    const long e = i - g * per;  // a0 * slab + point
    const float2 *src = P + static_cast<size_t>(g) * n0 * slab + e;
    float2 acc = make_float2(0.f, 0.f);
    for (int a = 0; a < n0; a += m0) {
      const float2 u = src[static_cast<size_t>(a) * slab];
      acc.x += u.x;
      acc.y += u.y;
    }
    Q[i] = acc;
  }
}

__global__ __launch_bounds__(256) void k3_real_part(const float2 *__restrict__ src,
                                                    float *__restrict__ out, long total) {
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride)
    out[i] = src[i].x;
}

template <int N1, int N2>
hipError_t slab_mul_inv_t(const float2 *Fh, const float2 *tab, float2 *W, long volumes, int n0, int M,
                          const float2 *tw, int tw_n, hipStream_t st) {
  using S = Slab<N1, N2>;
  const long slabs = volumes * n0;
  const long blocks = (slabs + S::SPW - 1) / S::SPW;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const std::string name = "k3_slab_mul_inv<" + std::to_string(N1) + ", " + std::to_string(N2) +
                           (S::NT == 1024 ? ", true>" : ", false>");
  const double pts = static_cast<double>(slabs) * N1 * N2;
  LaunchScope obs(name.c_str(), pts * 8.0 * (1 + M) + 8.0 * M * n0 * N1 * N2,
                  pts * M * (5.0 * (ilog2h(N1) + ilog2h(N2)) + 6.0), st);
  constexpr bool SPLIT = S::NT == 1024;  // (measured: slower for the smaller slabs)
  if (SPLIT && M > 65535) return hipErrorInvalidValue;
  if (S::lds_bytes > 65536) {
    static unsigned long long lds_ok = 0;
    hipError_t e =
        allow_large_lds(reinterpret_cast<const void *>(k3_slab_mul_inv<N1, N2, SPLIT>), lds_ok);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((k3_slab_mul_inv<N1, N2, SPLIT>),
                     dim3(static_cast<unsigned>(blocks), SPLIT ? M : 1), dim3(S::NT),
                     S::lds_bytes, st, Fh, tab, W, slabs, n0, M,
                     static_cast<size_t>(slabs) * N1 * N2, tw, tw_n);
  return hipGetLastError();
}

template <int N1, int N2>
hipError_t slab_fwd_low_t(const float2 *Tin, float2 *Uout, const float *phi, float2 *P,
                          long volumes, int n0, int J, int K, int chan, const float2 *tw, int tw_n,
                          hipStream_t st) {
  using S = Slab<N1, N2>;
  const long slabs = volumes * (n0 / 2 + 1);
  const long blocks = (slabs + S::SPW - 1) / S::SPW;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const size_t folded = static_cast<size_t>(n0) * (N1 >> J) * (N2 >> J);
  const std::string name =
      "k3_slab_fwd_low<" + std::to_string(N1) + ", " + std::to_string(N2) + ">";
  const double pts = static_cast<double>(slabs) * N1 * N2;
  const double full = static_cast<double>(volumes) * n0 * N1 * N2;
  LaunchScope obs(name.c_str(),
                  pts * 8.0 + (Uout ? full * 8.0 : 0.0) + 4.0 * (n0 / 2 + 1) * N1 * N2 +
                      8.0 * volumes * folded,
                  pts * (5.0 * (ilog2h(N1) + ilog2h(N2)) + 4.0), st);
  if (S::lds_bytes > 65536) {
    static unsigned long long lds_ok = 0;
    hipError_t e = allow_large_lds(reinterpret_cast<const void *>(k3_slab_fwd_low<N1, N2>), lds_ok);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((k3_slab_fwd_low<N1, N2>), dim3(static_cast<unsigned>(blocks)), dim3(S::NT),
                     S::lds_bytes, st, Tin, Uout, phi, P, slabs, n0, J, folded * K, folded * chan,
                     tw, tw_n);
  return hipGetLastError();
}

template <int E, int T>
hipError_t axis0_t(const float2 *W, const float *xreal, float2 *dst, long volumes, int Mc, int M,
                   const float2 *tw, int tw_n, hipStream_t st) {
  int TC = 256 / T;
  if (TC > Mc) TC = Mc;
  const long blocks = volumes * (Mc / TC);
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const size_t lds =
      T == 1 ? 0 : static_cast<size_t>(E) * (T * TC + (E == 32 ? 0 : 1)) * sizeof(float2);
  const std::string name = "k3_axis0_rho<" + std::to_string(E) + ", " + std::to_string(T) + ">";
  const double pts = static_cast<double>(volumes) * E * T * Mc;
  const int passes = xreal ? 1 : M + 1;
  LaunchScope obs(name.c_str(), pts * (xreal ? 4.0 : 8.0 * M) + pts * 8.0 * (E * T / 2 + 1) / (E * T),
                  pts * (passes * 5.0 * ilog2h(E * T) + (xreal ? 0.0 : 4.0 * M)), st);
  hipLaunchKernelGGL((k3_axis0_rho<E, T>), dim3(static_cast<unsigned>(blocks)), dim3(T * TC), lds, st,
                     W, xreal, dst, Mc, TC, M, static_cast<size_t>(volumes) * E * T * Mc, tw, tw_n);
  return hipGetLastError();
}

template <int E, int T>
hipError_t axis0_back_t(int mode, float2 *W, float *acc, const float2 *gu, long volumes, int Mc, int P,
                        const float2 *tw, int tw_n, hipStream_t st) {
  int TC = 256 / T;
  if (TC > Mc) TC = Mc;
  const long blocks = volumes * (Mc / TC);
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  // exchange area of the transforms, then their twiddle table
  const size_t lds =
      T == 1 ? 0 : (static_cast<size_t>(E) * (T * TC + (E == 32 ? 0 : 1)) + E * T) * sizeof(float2);
  const std::string name = "k3_axis0_back<" + std::to_string(E) + ", " + std::to_string(T) + ", " +
                           (mode ? "1>" : "0>");
  const double pts = static_cast<double>(volumes) * E * T * Mc;
  LaunchScope obs(name.c_str(), pts * (16.0 * P + (mode ? 12.0 : 4.0)),
                  pts * P * (5.0 * ilog2h(E * T) + 4.0), st);
  const size_t mstride = static_cast<size_t>(volumes) * E * T * Mc;
  if (mode == 0)
    hipLaunchKernelGGL((k3_axis0_back<E, T, 0>), dim3(static_cast<unsigned>(blocks)), dim3(T * TC), lds,
                       st, W, acc, gu, Mc, TC, P, mstride, tw, tw_n);
  else
    hipLaunchKernelGGL((k3_axis0_back<E, T, 1>), dim3(static_cast<unsigned>(blocks)), dim3(T * TC), lds,
                       st, W, acc, gu, Mc, TC, P, mstride, tw, tw_n);
  return hipGetLastError();
}

template <int N1, int N2>
hipError_t slab_fwd_mulacc_t(const float2 *W, const float2 *tab, float2 *A, long volumes, int n0, int P,
                             const float2 *tw, int tw_n, hipStream_t st) {
  using S = Slab<N1, N2>;
  const long slabs = volumes * n0;
  const long blocks = (slabs + S::SPW - 1) / S::SPW;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const std::string name =
      "k3_slab_fwd_mulacc<" + std::to_string(N1) + ", " + std::to_string(N2) + ">";
  const double pts = static_cast<double>(slabs) * N1 * N2;
  LaunchScope obs(name.c_str(), pts * 8.0 * (P + 2) + 8.0 * P * n0 * N1 * N2,
                  pts * P * (5.0 * (ilog2h(N1) + ilog2h(N2)) + 8.0), st);
  const size_t lds = S::lds_bytes + S::tab_elems * sizeof(float2);
  if (lds > 65536) {
    static unsigned long long lds_ok = 0;
    hipError_t e =
        allow_large_lds(reinterpret_cast<const void *>(k3_slab_fwd_mulacc<N1, N2>), lds_ok);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((k3_slab_fwd_mulacc<N1, N2>), dim3(static_cast<unsigned>(blocks)), dim3(S::NT),
                     lds, st, W, tab, A, slabs, n0, P, static_cast<size_t>(slabs) * N1 * N2,
                     tw, tw_n);
  return hipGetLastError();
}

}  // namespace

bool fused3_supported(int n0, int n1, int n2, int J) {
  auto p2 = [](int v) { return v > 0 && (v & (v - 1)) == 0; };
  // slabs of up to 16384 points, except 256 x 64 whose padded rows exceed the LDS of a CU
  return p2(n0) && p2(n1) && p2(n2) && n0 >= 4 && n0 <= 256 && n1 >= 16 && n2 >= 16 &&
         n1 * n2 <= 16384 && !(n1 == 256 && n2 == 64) && J >= 0 && J <= 4 && (n1 >> J) >= 1 &&
         (n2 >> J) >= 1;
}

#define SCAT3_SLAB_DISPATCH(CALL)                  \
  switch ((n1 << 12) | n2) {                       \
    case (16 << 12) | 16: CALL(16, 16);            \
    case (16 << 12) | 32: CALL(16, 32);            \
    case (16 << 12) | 64: CALL(16, 64);            \
    case (16 << 12) | 128: CALL(16, 128);          \
    case (16 << 12) | 256: CALL(16, 256);          \
    case (32 << 12) | 16: CALL(32, 16);            \
    case (32 << 12) | 32: CALL(32, 32);            \
    case (32 << 12) | 64: CALL(32, 64);            \
    case (32 << 12) | 128: CALL(32, 128);          \
    case (64 << 12) | 16: CALL(64, 16);            \
    case (64 << 12) | 32: CALL(64, 32);            \
    case (64 << 12) | 64: CALL(64, 64);            \
    case (128 << 12) | 16: CALL(128, 16);          \
    case (128 << 12) | 32: CALL(128, 32);          \
    case (256 << 12) | 16: CALL(256, 16);          \
    case (32 << 12) | 256: CALL(32, 256);          \
    case (64 << 12) | 128: CALL(64, 128);          \
    case (128 << 12) | 64: CALL(128, 64);          \
    case (256 << 12) | 32: CALL(256, 32);          \
    case (64 << 12) | 256: CALL(64, 256);          \
    case (128 << 12) | 128: CALL(128, 128);        \
    default: return hipErrorInvalidValue;          \
  }

hipError_t launch3_slab_mul_inv(const float2 *Fh, const float2 *tab, float2 *W, long volumes, int n0,
                                int n1, int n2, int M, const float2 *tw, int tw_n, hipStream_t st) {
  if (volumes <= 0 || M <= 0) return hipSuccess;
  if (tw_n % n1 != 0 || tw_n % n2 != 0) return hipErrorInvalidValue;
#define SCAT3_A(A_, B_) return slab_mul_inv_t<A_, B_>(Fh, tab, W, volumes, n0, M, tw, tw_n, st)
  SCAT3_SLAB_DISPATCH(SCAT3_A)
#undef SCAT3_A
}

hipError_t launch3_slab_fwd_low(const float2 *Tin, float2 *Uout, const float *phi, float2 *P,
                                long volumes, int n0, int n1, int n2, int J, int K, int chan,
                                const float2 *tw, int tw_n, hipStream_t st) {
  if (volumes <= 0) return hipSuccess;
  if (tw_n % n1 != 0 || tw_n % n2 != 0 || J < 0 || J > 4 || (n1 >> J) < 1 || (n2 >> J) < 1)
    return hipErrorInvalidValue;
#define SCAT3_C(A_, B_) \
  return slab_fwd_low_t<A_, B_>(Tin, Uout, phi, P, volumes, n0, J, K, chan, tw, tw_n, st)
  SCAT3_SLAB_DISPATCH(SCAT3_C)
#undef SCAT3_C
}

hipError_t launch3_axis0_rho(const float2 *W, const float *xreal, float2 *dst, long volumes, int n0,
                             int Mc, int M, const float2 *tw, int tw_n, hipStream_t st) {
  if (volumes <= 0) return hipSuccess;
  if (tw_n % n0 != 0 || Mc < 256 || (Mc & (Mc - 1)) != 0 || (xreal == nullptr && M <= 0))
    return hipErrorInvalidValue;
#define SCAT3_B(E_, T_) return axis0_t<E_, T_>(W, xreal, dst, volumes, Mc, M, tw, tw_n, st)
  switch (n0) {
    case 4: SCAT3_B(4, 1);
    case 8: SCAT3_B(8, 1);
    case 16: SCAT3_B(16, 1);
    case 32: SCAT3_B(16, 2);
    case 64: SCAT3_B(16, 4);
    case 128: SCAT3_B(16, 8);
    case 256: SCAT3_B(16, 16);
    default: return hipErrorInvalidValue;
  }
#undef SCAT3_B
}

hipError_t launch3_axis0_back(int mode, float2 *W, float *acc, const float2 *gu, long volumes, int n0,
                              int Mc, int P, const float2 *tw, int tw_n, hipStream_t st) {
  if (volumes <= 0 || P <= 0) return hipSuccess;
  if (tw_n % n0 != 0 || Mc < 256 || (Mc & (Mc - 1)) != 0 || acc == nullptr ||
      (mode != 0 && gu == nullptr))
    return hipErrorInvalidValue;
#define SCAT3_AB(E_, T_) return axis0_back_t<E_, T_>(mode, W, acc, gu, volumes, Mc, P, tw, tw_n, st)
  switch (n0) {
    case 4: SCAT3_AB(4, 1);
    case 8: SCAT3_AB(8, 1);
    case 16: SCAT3_AB(16, 1);
    case 32: SCAT3_AB(16, 2);
    case 64: SCAT3_AB(16, 4);
    case 128: SCAT3_AB(16, 8);
    case 256: SCAT3_AB(16, 16);
    default: return hipErrorInvalidValue;
  }
#undef SCAT3_AB
}

hipError_t launch3_slab_fwd_mulacc(const float2 *W, const float2 *tab, float2 *A, long volumes, int n0,
                                   int n1, int n2, int P, const float2 *tw, int tw_n,
                                   hipStream_t st) {
  if (volumes <= 0 || P <= 0) return hipSuccess;
  if (tw_n % n1 != 0 || tw_n % n2 != 0) return hipErrorInvalidValue;
#define SCAT3_D(A_, B_) return slab_fwd_mulacc_t<A_, B_>(W, tab, A, volumes, n0, P, tw, tw_n, st)
  SCAT3_SLAB_DISPATCH(SCAT3_D)
#undef SCAT3_D
}

hipError_t launch3_fold0(const float2 *P, float2 *Q, long groups, int n0, int m0, int slab,
                         hipStream_t st) {
  const long total = groups * m0 * slab;
  if (total <= 0) return hipSuccess;
  LaunchScope obs("k3_fold0", groups * 8.0 * slab * (n0 + m0), groups * 2.0 * slab * n0, st);
  hipLaunchKernelGGL(k3_fold0, dim3(blocks_for(total)), dim3(256), 0, st, P, Q, groups, n0, m0, slab);
  return hipGetLastError();
}

hipError_t launch3_real_part(const float2 *src, float *out, long total, hipStream_t st) {
  if (total <= 0) return hipSuccess;
  LaunchScope obs("k3_real_part", total * 12.0, 0.0, st);
  hipLaunchKernelGGL(k3_real_part, dim3(blocks_for(total)), dim3(256), 0, st, src, out, total);
  return hipGetLastError();
}

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
                             hipStream_t st, int fstride, bool accumulate) {
  const long total = volumes * n;
  if (total <= 0) return hipSuccess;
  if (fstride < 1) return hipErrorInvalidValue;
  LaunchScope obs("k3_mul_table", total * (accumulate ? 24.0 : 16.0) + n * 4.0, total * 2.0, st);
  hipLaunchKernelGGL(k3_mul_table, dim3(blocks_for(total)), dim3(256), 0, st, src, filt, fstride, dst,
                     total, n, accumulate ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch3_tile_phi(const float2 *Gs, const float *phi, float2 *dst, long volumes, int K,
                            int chan, int n0, int n1, int n2, int J, bool accumulate, hipStream_t st) {
  const long total = volumes * n0 * n1 * n2;
  if (total <= 0) return hipSuccess;
  LaunchScope obs("k3_tile_phi", total * (accumulate ? 16.0 : 8.0) + 4.0 * n0 * n1 * n2, total * 2.0,
                  st);
  hipLaunchKernelGGL(k3_tile_phi, dim3(blocks_for(total)), dim3(256), 0, st, Gs, phi, dst, volumes, K,
                     chan, n0, n1, n2, J, accumulate ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch3_mul_ctable(const float2 *src, const float2 *ctab, float2 *dst, long volumes, long n,
                              bool conj_table, bool accumulate, hipStream_t st) {
  const long total = volumes * n;
  if (total <= 0) return hipSuccess;
  LaunchScope obs("k3_mul_ctable", total * (accumulate ? 24.0 : 16.0) + n * 8.0, total * 6.0, st);
  hipLaunchKernelGGL(k3_mul_ctable, dim3(blocks_for(total)), dim3(256), 0, st, src, ctab, dst, total, n,
                     conj_table ? 1 : 0, accumulate ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch3_rho_back(const float2 *gu, const float *acc, float2 *y, long total,
                            hipStream_t st) {
  if (total <= 0) return hipSuccess;
  LaunchScope obs("k3_rho_back", total * 28.0, total * 4.0, st);
  hipLaunchKernelGGL(k3_rho_back, dim3(blocks_for(total)), dim3(256), 0, st, gu, acc, y, total);
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
