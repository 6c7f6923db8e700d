// Kernels of the backward pass (gradient of <g, S(x)> with respect to x) of the 2-D
// cascade.  The paper lists differentiability as a feature of its package (section 3,
// "Relation to previous software") and gives no formulas; the forward cascade is a chain of
// real-linear maps and complex moduli, so its transpose is the chain of adjoints in
// reverse order:
//   S = Re IFFT_m(fold(Z^ phi))   ->  g_Z^ = tile(FFT_m(g_S)) phi        (k_small_fft2 / k_slab_fft2_real, then
//                                                                        the consumer tiles and multiplies)
//   Z^ = FFT(Z), Z real           ->  g_Z  = Re IFFT(g_Z^)               (k_fft_rows, k_cols_modback)
//   Z = |y|                       ->  g_y  = g_Z y / |y|  (0 at y = 0)   (k_cols_modback)
//   y = IFFT(fold(A^ psi))        ->  g_A^ += tile(FFT(g_y)) psi         (k_fft_* + k_tile_accum)
// with unnormalised transforms throughout: the filter tables already carry the 1/n of the
// forward pass, and the adjoint of a product with a real table is the same product.
#include <hip/hip_runtime.h>

#include <string>
#include <type_traits>

#include "fft_regs.hpp"
#include "slab_fft.hpp"
#include "scat_kernels.hpp"

namespace scat {

namespace {

__device__ __forceinline__ int chan(const ChanMap &cm, int g) {
  return cm.base + (g / cm.inner) * cm.outer_stride + (g % cm.inner);
}

// First half of the adjoint lowpass: Ghat [node][m_r][m_c] = FFT2 of the node's gradient
// plane (two dense stages in LDS; the planes are tiny).  A workgroup takes NPW = 256 / (m_r m_c)
// nodes when a plane has fewer than 256 points, one thread per point (else one node, several
// points per thread).
__global__ __launch_bounds__(256) void k_small_fft2(const float *__restrict__ gout, ChanMap cm,
                                                    int K, int m_r, int m_c, int NPW, long nodes,
                                                    float2 *__restrict__ ghat,
                                                    const float2 *__restrict__ tw, int tw_n) {
  extern __shared__ float2 lds[];
  const int mm = m_r * m_c;
  float2 *s1 = lds;                      // NPW planes
  float2 *twc = lds + NPW * mm, *twr = twc + m_c;
  float *a = reinterpret_cast<float *>(twr + m_r);  // NPW planes
  const int per = NPW > 1 ? mm : static_cast<int>(blockDim.x);  // threads of one node
  const int nl = threadIdx.x / per, t0 = threadIdx.x - nl * per;
  const long node_raw = static_cast<long>(blockIdx.x) * NPW + nl;
  const bool live = nl < NPW && node_raw < nodes;
  const long node = live ? node_raw : nodes - 1;  // idle threads shadow the last node, store nothing
  const long p = node / cm.G;
  const int g = static_cast<int>(node - p * cm.G);
  const float *gp = gout + (static_cast<size_t>(p) * K + chan(cm, g)) * mm;
  const int slot = nl < NPW ? nl : 0;
  float *an = a + slot * mm;
  float2 *sn = s1 + slot * mm;
  if (nl < NPW)
    for (int i = t0; i < mm; i += per) an[i] = gp[i];
  const int sc = tw_n / m_c, sr = tw_n / m_r;
  for (int i = threadIdx.x; i < m_c; i += blockDim.x) twc[i] = tw[i * sc];
  for (int i = threadIdx.x; i < m_r; i += blockDim.x) twr[i] = tw[i * sr];
  __syncthreads();
  if (nl < NPW)
    for (int i = t0; i < mm; i += per) {
      const int r = i / m_c, kc = i - r * m_c;
      float2 acc = make_float2(0.f, 0.f);
      for (int b = 0; b < m_c; ++b) {
        const float2 w = twc[(b * kc) & (m_c - 1)];
        const float x = an[r * m_c + b];
        acc.x += x * w.x;
        acc.y += x * w.y;
      }
      sn[i] = acc;
    }
  __syncthreads();
  if (!live) return;
  float2 *op = ghat + static_cast<size_t>(node) * mm;
  for (int i = t0; i < mm; i += per) {
    const int kr = i / m_c, kc = i - kr * m_c;
    float2 acc = make_float2(0.f, 0.f);
    for (int r = 0; r < m_r; ++r) acc = c_add(acc, c_mul(sn[r * m_c + kc], twr[(r * kr) & (m_r - 1)]));
    op[i] = acc;
  }
}

// k_small_fft2 for planes of 16 ... 128 points a side (square or 2 : 1) by the slab
// transform: 16 points per thread, a 32 x 32 plane per wavefront.
template <int N1, int N2>
__global__ __launch_bounds__((Slab<N1, N2>::NT)) void k_slab_fft2_real(const float *__restrict__ gout,
                                                                      ChanMap cm, int K,
                                                                      float2 *__restrict__ ghat,
                                                                      long nodes,
                                                                      const float2 *__restrict__ tw,
                                                                      int tw_n) {
  using S = Slab<N1, N2>;
  extern __shared__ float2 lds[];
  const int s = threadIdx.x / S::TS, q = threadIdx.x % S::TS;
  const long node_raw = static_cast<long>(blockIdx.x) * S::SPW + s;
  const bool live = node_raw < nodes;
  const long node = live ? node_raw : nodes - 1;  // idle threads shadow the last node, store nothing
  float2 *area = lds + s * N1 * S::RS;
  const int r = q / S::T2, t = q % S::T2;
  const int c = q % N2, t1 = q / N2;
  const long p = node / cm.G;
  const int g = static_cast<int>(node - p * cm.G);
  const float *gp = gout + (static_cast<size_t>(p) * K + chan(cm, g)) * (N1 * N2) + r * N2 + t;
  float2 v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = make_float2(gp[S::T2 * i], 0.f);
  S::template transform<false>(v, area, r, t, c, t1, tw, tw_n);
  if (live) {
    float2 *op = ghat + static_cast<size_t>(node) * (N1 * N2) + c;
#pragma unroll
    for (int i = 0; i < 16; ++i) op[(t1 + S::T1 * i) * N2] = v[i];
  }
}

// Second half fused with the inverse row transform that follows it: row (node, k_r) of the
// M x M gradient spectrum is Ghat[node][k_r mod m_r][k_c mod m_c] phi_rows[k_r] phi_cols[k_c];
// it is formed in registers, transformed along the row and written once.
template <int E, int T>
__global__ __launch_bounds__(E == 32 ? 128 : 256) void k_rows_lowpass_adj(
    const float2 *__restrict__ ghat, int m_r, int m_c, int lgMr, const float *__restrict__ phi_rows,
    const float *__restrict__ phi_cols, float2 *__restrict__ dst, long rows,
    const float2 *__restrict__ tw, int tw_n) {
  constexpr int NT = E == 32 ? 128 : 256;
  constexpr int RPB = NT / T, M = E * T;
  extern __shared__ float2 lds[];
  const int rl = threadIdx.x / T, t = threadIdx.x % T;
  const long row_raw = static_cast<long>(blockIdx.x) * RPB + rl;
  const bool valid = row_raw < rows;
  const long row = valid ? row_raw : rows - 1;
  const long node = row >> lgMr;
  const int kr = static_cast<int>(row & ((1 << lgMr) - 1));
  const float2 *gp = ghat + (static_cast<size_t>(node) * m_r + (kr & (m_r - 1))) * m_c;
  const float fr = phi_rows[kr];
  float2 v[E];
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const int kc = t + T * i;
    const float f = fr * phi_cols[kc];
    const float2 x = gp[kc & (m_c - 1)];
    v[i] = make_float2(x.x * f, x.y * f);
  }
  float2 wt[E];
  load_twiddles<E, T>(wt, t, tw, tw_n);
  fft_core<E, T, true, true>(v, t, lds + rl * (E * (T + 1)), T + 1, 1, wt);
  if (!valid) return;
  float2 *p = dst + static_cast<size_t>(row) * M + t;
#pragma unroll
  for (int i = 0; i < E; ++i) p[T * i] = v[i];
}

__global__ __launch_bounds__(256) void k_take_real(const float2 *__restrict__ a,
                                                   float *__restrict__ out, long count) {
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < count; i += stride)
    out[i] = a[i].x;
}

// dst [S][Sr][Sc] += sum_f filt[f][k_r][k_c] * G[s F + f][k_r mod Mr][k_c mod Mc]
// (adjoint of: multiply by the F filters, fold to Mr x Mc).  One thread per element
// (q_r, q_c) of the folded grid and group of SB sources: it reads its F values of G once per
// source (FB at a time) and updates every copy (q_r + a Mr, q_c + b Mc) of dst, loading
// each filter value once for the SB sources -- nothing is read twice, nothing is shared.
template <int FB, int SB>
__global__ __launch_bounds__(256) void k_tile_accum(float2 *__restrict__ dst,
                                                    const float *__restrict__ filt,
                                                    const float2 *__restrict__ G, long count,
                                                    long S, int F, int lgSr, int lgSc, int lgMr,
                                                    int lgMc) {
  const long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= count) return;
  const int lgM = lgMr + lgMc, lgS = lgSr + lgSc;
  const long s0 = (i >> lgM) * SB;
  const int e = static_cast<int>(i & ((1L << lgM) - 1));
  const int qr = e >> lgMc, qc = e & ((1 << lgMc) - 1);
  const int nr = 1 << (lgSr - lgMr), nc = 1 << (lgSc - lgMc);
  for (int f0 = 0; f0 < F; f0 += FB) {
    float2 g[SB][FB];
#pragma unroll
    for (int k = 0; k < SB; ++k) {
      const long s = s0 + k < S ? s0 + k : S - 1;  // sources past the end repeat the last, unstored
#pragma unroll
      for (int j = 0; j < FB; ++j)
        g[k][j] = f0 + j < F ? G[((static_cast<size_t>(s) * F + f0 + j) << lgM) + e]
                             : make_float2(0.f, 0.f);
    }
    for (int a = 0; a < nr; ++a)
      for (int b = 0; b < nc; ++b) {
        const int o = ((qr + (a << lgMr)) << lgSc) + qc + (b << lgMc);
        float w[FB];
#pragma unroll
        for (int j = 0; j < FB; ++j)
          w[j] = filt[(static_cast<size_t>(f0 + j < F ? f0 + j : F - 1) << lgS) + o];
#pragma unroll
        for (int k = 0; k < SB; ++k) {
          if (s0 + k >= S) break;
          float2 *dp = dst + (static_cast<size_t>(s0 + k) << lgS) + o;
          float2 acc = *dp;
#pragma unroll
          for (int j = 0; j < FB; ++j) {
            acc.x += g[k][j].x * w[j];
            acc.y += g[k][j].y * w[j];
          }
          *dp = acc;
        }
      }
  }
}

// In-place transform of every row of [rows][E*T] (T lanes per row, wave-level sync only).
template <int E, int T, bool INV>
__global__ __launch_bounds__(E == 32 ? 128 : 256) void k_fft_rows(float2 *__restrict__ data,
                                                                  long rows,
                                                                  const float2 *__restrict__ tw,
                                                                  int tw_n) {
  constexpr int NT = E == 32 ? 128 : 256;
  constexpr int RPB = NT / T, M = E * T;
  extern __shared__ float2 lds[];
  const int rl = threadIdx.x / T, t = threadIdx.x % T;
  const long row = static_cast<long>(blockIdx.x) * RPB + rl;
  const bool valid = row < rows;
  float2 *p = data + static_cast<size_t>(valid ? row : 0) * M + t;
  float2 v[E];
#pragma unroll
  for (int i = 0; i < E; ++i) v[i] = valid ? p[T * i] : make_float2(0.f, 0.f);
  float2 wt[E];
  load_twiddles<E, T>(wt, t, tw, tw_n);
  fft_core<E, T, INV, true>(v, t, lds + rl * (E * (T + 1)), T + 1, 1, wt);
  if (!valid) return;
#pragma unroll
  for (int i = 0; i < E; ++i) p[T * i] = v[i];
}

// In-place transform of every column of [nodes][E*T][Mc]: a workgroup takes TC columns of
// one node, thread (t, c) holds rows t + T i of column c.
template <int E, int T, bool INV>
__global__ __launch_bounds__(256) void k_fft_cols(float2 *__restrict__ data, int Mc, int TC,
                                                  const float2 *__restrict__ tw, int tw_n) {
  constexpr int M = E * T;
  extern __shared__ float2 lds[];
  const int KS = T * TC + (E == 32 ? 0 : 1);
  const int c = threadIdx.x % TC, t = threadIdx.x / TC;
  const int tiles = Mc / TC;
  const long node = blockIdx.x / tiles;
  const int c0 = static_cast<int>(blockIdx.x % tiles) * TC;
  float2 *p = data + static_cast<size_t>(node) * M * Mc + static_cast<size_t>(t) * Mc + c0 + c;
  const size_t step = static_cast<size_t>(T) * Mc;
  float2 v[E];
#pragma unroll
  for (int i = 0; i < E; ++i) v[i] = p[i * step];
  float2 wt[E];
  load_twiddles<E, T>(wt, t, tw, tw_n);
  fft_core<E, T, INV, false>(v, t, lds + c, KS, TC, wt);
#pragma unroll
  for (int i = 0; i < E; ++i) p[i * step] = v[i];
}

// Column pass of the modulus backward step: inverse transform of every column, then
// a = Re(a) y / |y| against the taped signal y (same layout), then forward transform.
// tw_m > 0 (1-D signals as an E*T x Mc matrix, tw_m = E*T*Mc): the data are multiplied by
// exp(+2 pi i k1 b / tw_m) before the inverse column transform and by its conjugate after
// the forward one (the twiddle step of the four-step transform; k1 = row, b = column).
template <int E, int T>
__global__ __launch_bounds__(256, (E <= 16 ? 3 : 1)) void k_cols_modback(float2 *__restrict__ data,
                                                      const float2 *__restrict__ y, int Mc, int TC,
                                                      int tw_m, int y_rows,
                                                      const float2 *__restrict__ tw, int tw_n) {
  constexpr int M = E * T;
  extern __shared__ float2 lds[];
  const int KS = T * TC + (E == 32 ? 0 : 1);
  const int c = threadIdx.x % TC, t = threadIdx.x / TC;
  const int tiles = Mc / TC;
  const long node = blockIdx.x / tiles;
  const int c0 = static_cast<int>(blockIdx.x % tiles) * TC;
  const size_t off = static_cast<size_t>(node) * M * Mc + static_cast<size_t>(t) * Mc + c0 + c;
  float2 *p = data + off;
  const float2 *yp = y + off;
  const size_t step = static_cast<size_t>(T) * Mc;
  float2 v[E];
#pragma unroll
  for (int i = 0; i < E; ++i) v[i] = p[i * step];
  // four-step twiddles exp(-2 pi i k1 b / tw_m) of this thread's elements.  FACT: k1 = t + T i,
  // b the column, tw_m = 16 T Mc, so the twiddle is exp(-2 pi i t b / tw_m) (`wa`, one table
  // read per thread) times exp(-2 pi i i b / (16 Mc)), fetched once for the workgroup's TC
  // columns into LDS (`ftab`, 16 TC entries behind the exchange area) instead of 16 scattered
  // reads per thread; they are rebuilt from there after the transforms rather than kept in
  // registers across them.
  const bool fact = tw_m > 0 && E == 16 && T > 1 && tw_m == M * Mc;
  float2 *ftab = lds + E * KS;
  float2 wa = make_float2(1.f, 0.f);
  if (fact) {
    const int bmask = 16 * Mc - 1, bstep = tw_n / (16 * Mc);
    for (int idx = threadIdx.x; idx < 16 * TC; idx += blockDim.x) {
      const int i = idx / TC, cc = idx - i * TC;
      ftab[idx] = tw[((i * (c0 + cc)) & bmask) * bstep];
    }
    __syncthreads();
    wa = tw[((t * (c0 + c)) & (tw_m - 1)) * (tw_n / tw_m)];
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const float2 f = c_mul(wa, ftab[(i & 15) * TC + c]);
      v[i] = c_mul(v[i], make_float2(f.x, -f.y));
    }
  } else if (tw_m > 0) {
    const int tstep = tw_n / tw_m;
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const int e = static_cast<int>((static_cast<long long>(t + T * i) * (c0 + c)) & (tw_m - 1));
      const float2 f = tw[e * tstep];
      v[i] = c_mul(v[i], make_float2(f.x, -f.y));
    }
  }
  // the transforms' own twiddles exp(-2 pi i t k / M), also through LDS (wtab[k T + t]);
  // 512-point columns (E = 32) fill the LDS with their exchange area and keep them in registers
  constexpr bool WTAB = E <= 16 && T > 1;
  float2 *wtab = ftab + 16 * TC;
  float2 wt[E];  // unused (and dropped by the compiler) with WTAB
  if constexpr (WTAB) {
    for (int idx = threadIdx.x; idx < M; idx += blockDim.x)
      wtab[idx] = tw[(idx / T) * (idx % T) * (tw_n / M)];
    __syncthreads();
  } else {
    load_twiddles<E, T>(wt, t, tw, tw_n);
  }
  auto transform_of = [&](float2 (&a)[E], auto inv) {
    if constexpr (WTAB)
      fft_core_tab<E, T, decltype(inv)::value, false>(a, t, lds + c, KS, TC, wtab + t, T);
    else
      fft_core<E, T, decltype(inv)::value, false>(a, t, lds + c, KS, TC, wt);
  };
  auto transform = [&](auto inv) { transform_of(v, inv); };
  // the tape values are requested before the inverse transform and used after it (3 waves
  // per SIMD with them in flight beat 4 without)
  float2 yv[E];
#pragma unroll
  for (int i = 0; i < E; ++i) yv[i] = yp[i * step];
  // y_rows: `y` holds the node before its inverse column transform (the forward row pass's
  // output, which spares the forward pass its column kernel): transformed here
  if (y_rows) transform_of(yv, std::true_type{});
  transform(std::true_type{});
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const float2 u = yv[i];
    const float m2 = u.x * u.x + u.y * u.y;
    const float sgn = over_sqrt(v[i].x, m2);
    v[i] = make_float2(u.x * sgn, u.y * sgn);
  }
  transform(std::false_type{});
  if (fact) {
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = c_mul(v[i], c_mul(wa, ftab[(i & 15) * TC + c]));
  } else if (tw_m > 0) {
    const int tstep = tw_n / tw_m;
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const int e = static_cast<int>((static_cast<long long>(t + T * i) * (c0 + c)) & (tw_m - 1));
      v[i] = c_mul(v[i], tw[e * tstep]);
    }
  }
#pragma unroll
  for (int i = 0; i < E; ++i) p[i * step] = v[i];
}

// ---- 1-D signals (four-step layout: an n1 x Mc matrix, sample a Mc + b, frequency
// k1 + n1 k2 stored at [k1][k2])

// data[node][k1][b] *= exp(-+ 2 pi i k1 b / m): the twiddle step between the column and
// the row pass of a four-step transform (conj = inverse direction)
__global__ __launch_bounds__(256) void k_twiddle(float2 *__restrict__ data, long count, int lgMc,
                                                 int lgN1, int m, int conj,
                                                 const float2 *__restrict__ tw, int tw_n) {
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  const int tstep = tw_n / m;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < count; i += stride) {
    const int b = static_cast<int>(i & ((1 << lgMc) - 1));
    const int k1 = static_cast<int>((i >> lgMc) & ((1 << lgN1) - 1));
    float2 w = tw[static_cast<int>((static_cast<long long>(k1) * b) & (m - 1)) * tstep];
    if (conj) w.y = -w.y;
    data[i] = c_mul(data[i], w);
  }
}

// dst[node][i] = (g_out[plane][chan(cm, g)][i], 0), i < m: one gradient signal per node
__global__ __launch_bounds__(256) void k_gather_real(const float *__restrict__ gout, ChanMap cm,
                                                     int K, int m, float2 *__restrict__ dst,
                                                     long count) {
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < count; i += stride) {
    const long node = i / m;
    const int e = static_cast<int>(i - node * m);
    const long p = node / cm.G;
    const int g = static_cast<int>(node - p * cm.G);
    dst[i] = make_float2(gout[(static_cast<size_t>(p) * K + chan(cm, g)) * m + e], 0.f);
  }
}

// dst[node][k1][k2] = ghat[node][k1][k2 mod mc] * filt[k1][k2]   (tile along k2, one table)
__global__ __launch_bounds__(256) void k_tile_filter(const float2 *__restrict__ ghat,
                                                     const float *__restrict__ filt,
                                                     float2 *__restrict__ dst, long count, int lgN1,
                                                     int lgMc, int lgmc) {
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < count; i += stride) {
    const int k2 = static_cast<int>(i & ((1 << lgMc) - 1));
    const long r = i >> lgMc;  // node * n1 + k1
    const int k1 = static_cast<int>(r & ((1 << lgN1) - 1));
    const float f = filt[(static_cast<size_t>(k1) << lgMc) + k2];
    const float2 v = ghat[(static_cast<size_t>(r) << lgmc) + (k2 & ((1 << lgmc) - 1))];
    dst[i] = make_float2(v.x * f, v.y * f);
  }
}

int ilog2h(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}

bool pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

template <int E, int T>
hipError_t rows_t(float2 *data, long rows, bool inverse, const float2 *tw, int tw_n,
                  hipStream_t st) {
  constexpr int NT = E == 32 ? 128 : 256, RPB = NT / T;
  const long blocks = (rows + RPB - 1) / RPB;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const size_t lds = T == 1 ? 0 : static_cast<size_t>(RPB) * E * (T + 1) * sizeof(float2);
  const std::string name = std::string("k_fft_rows<") + std::to_string(E) + ", " +
                           std::to_string(T) + (inverse ? ", true>" : ", false>");
  const double n = static_cast<double>(E) * T;
  LaunchScope obs(name.c_str(), rows * n * 16, rows * 5.0 * n * ilog2h(E * T), st);
  if (inverse)
    hipLaunchKernelGGL((k_fft_rows<E, T, true>), dim3(static_cast<unsigned>(blocks)), dim3(NT), lds,
                       st, data, rows, tw, tw_n);
  else
    hipLaunchKernelGGL((k_fft_rows<E, T, false>), dim3(static_cast<unsigned>(blocks)), dim3(NT), lds,
                       st, data, rows, tw, tw_n);
  return hipGetLastError();
}

template <int E, int T>
hipError_t cols_t(float2 *data, long nodes, int Mc, bool inverse, const float2 *tw, int tw_n,
                  hipStream_t st) {
  int TC = 256 / T;
  if (TC > Mc) TC = Mc;
  const long blocks = nodes * (Mc / TC);
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const size_t lds = T == 1 ? 0 : static_cast<size_t>(E) * (T * TC + (E == 32 ? 0 : 1)) * sizeof(float2);
  if (lds > 65536) return hipErrorInvalidValue;
  const std::string name = std::string("k_fft_cols<") + std::to_string(E) + ", " +
                           std::to_string(T) + (inverse ? ", true>" : ", false>");
  const double n = static_cast<double>(E) * T;
  LaunchScope obs(name.c_str(), nodes * n * Mc * 16, nodes * Mc * 5.0 * n * ilog2h(E * T), st);
  if (inverse)
    hipLaunchKernelGGL((k_fft_cols<E, T, true>), dim3(static_cast<unsigned>(blocks)), dim3(T * TC),
                       lds, st, data, Mc, TC, tw, tw_n);
  else
    hipLaunchKernelGGL((k_fft_cols<E, T, false>), dim3(static_cast<unsigned>(blocks)),
                       dim3(T * TC), lds, st, data, Mc, TC, tw, tw_n);
  return hipGetLastError();
}

template <int E, int T>
hipError_t cols_modback_t(float2 *data, const float2 *y, long nodes, int Mc, int tw_m, bool y_rows,
                          const float2 *tw, int tw_n, hipStream_t st) {
  int TC = 256 / T;
  if (TC > Mc) TC = Mc;
  const long blocks = nodes * (Mc / TC);
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  // exchange area of the transforms, the table of row twiddles, the transforms' twiddles
  const size_t lds = T == 1 ? 0
                            : (static_cast<size_t>(E) * (T * TC + (E == 32 ? 0 : 1)) +
                               (E <= 16 ? 16 * TC + E * T : 0)) * sizeof(float2);
  if (lds > 65536) return hipErrorInvalidValue;
  const std::string name = std::string("k_cols_modback<") + std::to_string(E) + ", " +
                           std::to_string(T) + ">";
  const double n = static_cast<double>(E) * T;
  LaunchScope obs(name.c_str(), nodes * n * Mc * 24,
                  nodes * Mc * ((y_rows ? 15.0 : 10.0) * n * ilog2h(E * T) + 8.0 * n), st);
  hipLaunchKernelGGL((k_cols_modback<E, T>), dim3(static_cast<unsigned>(blocks)), dim3(T * TC), lds,
                     st, data, y, Mc, TC, tw_m, static_cast<int>(y_rows), tw, tw_n);
  return hipGetLastError();
}

template <int E, int T>
hipError_t rows_lowpass_adj_t(const float2 *ghat, long nodes, int m_r, int m_c, int Mr,
                              const float *phi_rows, const float *phi_cols, float2 *dst,
                              const float2 *tw, int tw_n, hipStream_t st) {
  constexpr int NT = E == 32 ? 128 : 256, RPB = NT / T;
  const long rows = nodes * Mr;
  const long blocks = (rows + RPB - 1) / RPB;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const size_t lds = T == 1 ? 0 : static_cast<size_t>(RPB) * E * (T + 1) * sizeof(float2);
  const std::string name = std::string("k_rows_lowpass_adj<") + std::to_string(E) + ", " +
                           std::to_string(T) + ">";
  const double n = static_cast<double>(E) * T;
  LaunchScope obs(name.c_str(), nodes * 8.0 * m_r * m_c + rows * n * 8,
                  rows * (5.0 * n * ilog2h(E * T) + 3.0 * n), st);
  hipLaunchKernelGGL((k_rows_lowpass_adj<E, T>), dim3(static_cast<unsigned>(blocks)), dim3(NT), lds,
                     st, ghat, m_r, m_c, ilog2h(Mr), phi_rows, phi_cols, dst, rows, tw, tw_n);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// 1-D cascade, adjoint of the forward row kernel (k_rows1d_reg): the gradient of a parent's
// column spectra, dst [nodes][Sr][Sc], from the gradients of its children.  Per row:
//   dst = IFFT_Sc( sum_c  filt_c * tile_{Sc / m_c}( FFT_{m_c}(src_c row) ) )
// where child c's row has m_c = Sc >> lg_fold points (tile = adjoint of the fold) and filt_c
// is the real table [Sr][Sc] of the forward pass; both transforms unnormalised, no twiddles
// (the four-step twiddles belong to the column kernels on either side).  Which node of src_c
// belongs to a node of dst is the child's (cm, K) (see Rows1dAdjChild): the children may be
// separate arrays, the nodes of one array (first order: the wavelets of one octave) or
// channels of the channel-major array of output gradients.  The parent's
// spectrum stays in registers over the whole child list (lane t holds k = t + T i), every
// child is read once, and nothing but dst is written: the unfused form writes each child's
// spectrum and re-reads and re-writes the parent once per child.
// Same thread layout as the forward kernel: T lanes per row, 256 / T rows per workgroup,
// wave-level synchronisation only; the child's transform runs on its m_c / 16 lanes.
template <int E2, int T2>
__device__ __forceinline__ void rows1d_child_fwd(float2 *slot, int t, int tw_step,
                                                 const float2 *twl, const float2 *sp) {
  if (t >= T2) return;
  float2 v[E2], wt[E2];
#pragma unroll
  for (int i = 0; i < E2; ++i) v[i] = sp[t + T2 * i];
#pragma unroll
  for (int k = 0; k < E2; ++k) wt[k] = twl[t * k * tw_step];
  fft_core<E2, T2, false, true>(v, t, slot, T2 + 1, 1, wt);
  // the exchange area becomes the child's spectrum in natural order
#pragma unroll
  for (int i = 0; i < E2; ++i) slot[t + T2 * i] = v[i];
}

template <int E, int T>
__global__ __launch_bounds__(256, 4) void k_rows1d_adj(float2 *__restrict__ dst, long rows, int Sr,
                                                    Rows1dAdjArgs a,
                                                    const float2 *__restrict__ tw, int tw_n) {
  static_assert(E == 16 || T == 1, "short rows are held by one lane");
  constexpr int Sc = E * T, RPB = 256 / T;
  constexpr int XS = T == 1 ? E : E * (T + 1);
  constexpr int lgSc = (E == 4 ? 2 : E == 8 ? 3 : 4) + (T == 1 ? 0 : T == 2 ? 1 : T == 4 ? 2 : T == 8 ? 3 : 4);
  extern __shared__ float2 lds[];
  float2 *twl = lds;
  for (int j = threadIdx.x; j < Sc; j += blockDim.x) twl[j] = tw[j * (tw_n / Sc)];
  __syncthreads();
  const int rl = threadIdx.x / T, t = threadIdx.x % T;
  const long row_raw = static_cast<long>(blockIdx.x) * RPB + rl;
  const bool valid = row_raw < rows;
  const long row = valid ? row_raw : rows - 1;  // idle groups redo the last row, unstored
  const long node = row / Sr;
  const int k1 = static_cast<int>(row - node * Sr);
  float2 *slot = lds + Sc + rl * XS;
  float2 acc[E];
#pragma unroll
  for (int i = 0; i < E; ++i) acc[i] = make_float2(0.f, 0.f);
  for (int ci = 0; ci < a.n; ++ci) {
    const Rows1dAdjChild &ch = a.c[ci];
    const int lgm = lgSc - ch.lg_fold, m = 1 << lgm;
    const long cnode = ch.K > 0 ? (node / ch.cm.G) * ch.K + chan(ch.cm, static_cast<int>(node % ch.cm.G))
                                : node * ch.cm.G + ch.cm.base;
    const float2 *sp = ch.src + (static_cast<size_t>(cnode) * Sr + k1) * m;
    const int tws = Sc >> lgm;
    switch (lgm) {
      case 0:
        if (t == 0) slot[0] = sp[0];
        break;
      case 1: rows1d_child_fwd<2, 1>(slot, t, tws, twl, sp); break;
      case 2: rows1d_child_fwd<4, 1>(slot, t, tws, twl, sp); break;
      case 3: if (E >= 8) rows1d_child_fwd<(E >= 8 ? 8 : 4), 1>(slot, t, tws, twl, sp); break;
      case 4: if (E >= 16) rows1d_child_fwd<(E >= 16 ? 16 : 4), 1>(slot, t, tws, twl, sp); break;
      case 5: if (T >= 2) rows1d_child_fwd<16, (T >= 2 ? 2 : 1)>(slot, t, tws, twl, sp); break;
      case 6: if (T >= 4) rows1d_child_fwd<16, (T >= 4 ? 4 : 1)>(slot, t, tws, twl, sp); break;
      case 7: if (T >= 8) rows1d_child_fwd<16, (T >= 8 ? 8 : 1)>(slot, t, tws, twl, sp); break;
      case 8: if (T >= 16) rows1d_child_fwd<16, (T >= 16 ? 16 : 1)>(slot, t, tws, twl, sp); break;
      default: break;
    }
    wave_sync();
    // tile: lane t needs the spectrum at (t + T i) mod m.  For m >= T those are its first
    // m / T registers' worth, repeated; below, the single entry t mod m.
    float2 s[E];
#pragma unroll
    for (int i = 0; i < E; ++i) s[i] = slot[(t + T * i) & (m - 1)];
    const float *fp = ch.filt + static_cast<size_t>(k1) * Sc + t;
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const float f = fp[T * i];
      acc[i].x += s[i].x * f;
      acc[i].y += s[i].y * f;
    }
    wave_sync();  // the slot is reused by the next child
  }
  float2 wt[E];
#pragma unroll
  for (int k = 0; k < E; ++k) wt[k] = twl[t * k];
  fft_core<E, T, true, true>(acc, t, slot, T + 1, 1, wt);
  if (!valid) return;
  float2 *dp = dst + static_cast<size_t>(row) * Sc + t;
  if (a.accumulate) {
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const float2 o = dp[T * i];
      acc[i].x += o.x;
      acc[i].y += o.y;
    }
  }
#pragma unroll
  for (int i = 0; i < E; ++i) dp[T * i] = acc[i];
}

// acc[i] += f[i] * s[i mod EP]: the child's EP distinct values of this lane (sp[T j], j < EP)
// against the filter values fp[T i] (times fr)
template <int E, int T, int EP>
__device__ __forceinline__ void rows2d_accumulate(float2 (&acc)[E], const float2 *__restrict__ sp,
                                                  const float *__restrict__ fp, float fr) {
  constexpr int NP = EP < E ? EP : E;
  float2 sv[NP];
#pragma unroll
  for (int j = 0; j < NP; ++j) sv[j] = sp[T * j];
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const float f = fr * fp[T * i];
    acc[i].x += sv[i % NP].x * f;
    acc[i].y += sv[i % NP].y * f;
  }
}

// The same for a child of full row length given BEFORE its forward row transform (pre_rows):
// the lane's 16 values are transformed in registers first, which spares the child a row pass
// of its own.
template <int E, int T>
__device__ __forceinline__ void rows2d_accumulate_fft(float2 (&acc)[E], const float2 *__restrict__ sp,
                                                      const float *__restrict__ fp, float fr, int t,
                                                      float2 *xch, const float2 *wtab) {
  float2 sv[E];
#pragma unroll
  for (int j = 0; j < E; ++j) sv[j] = sp[T * j];
  fft_core_tab<E, T, false, true>(sv, t, xch, T + 1, 1, wtab + t, T);
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const float f = fr * fp[T * i];
    acc[i].x += sv[i].x * f;
    acc[i].y += sv[i].y * f;
  }
}

// ------------------------------------------------------------------------------------
// 2-D cascade: the gradient spectrum of a parent, dst [nodes][Sr][Sc], from the gradient
// spectra of all its children in one pass,
//   dst[kr][kc] (+)= sum_c filt_c[kr][kc] * src_c[kr mod (Sr >> fr_c)][kc mod (Sc >> fc_c)]
// (the adjoint of filter product + fold, for every child at once), optionally followed by
// the inverse row transform that the modulus backward step of the parent starts with.
// filt_c is a table [Sr][Sc], or with filt_row != nullptr the separable filt_row[kr] filt[kc]
// (lowpass; its src is the small transform of the parent's own output gradient).  Nodes of
// the children as in Rows1dAdjChild.  T lanes per row hold the parent's row in registers
// over the child list; dst is written once (the one-child-level-per-launch form re-reads
// and re-writes it for every level, and once more for the row transform).
template <int E, int T>
__global__ __launch_bounds__(256, 4) void k_rows2d_adj(float2 *__restrict__ dst, long nodes, int Sr,
                                                    Rows2dAdjArgs a,
                                                    const float2 *__restrict__ tw, int tw_n) {
  static_assert(E == 16 || T == 1, "short rows are held by one lane");
  constexpr int Sc = E * T, RPB = 256 / T;
  constexpr int XS = T == 1 ? E : E * (T + 1);
  constexpr int lgT = T == 1 ? 0 : T == 2 ? 1 : T == 4 ? 2 : T == 8 ? 3 : T == 16 ? 4 : 5;
  constexpr int lgSc = (E == 4 ? 2 : E == 8 ? 3 : 4) + lgT;
  extern __shared__ float2 lds[];
  // twiddles of the children's forward row transforms (pre_rows), wtab[k T + t], behind the
  // rows' exchange areas
  float2 *wtab = lds + RPB * XS;
  if (T > 1 && T <= E && a.any_pre_rows) {
    for (int idx = threadIdx.x; idx < Sc; idx += blockDim.x)
      wtab[idx] = tw[(idx / T) * (idx % T) * (tw_n / Sc)];
    __syncthreads();
  }
  // A workgroup takes 2^lgR rows kr0 + a (Sr >> lgR) of each of its nodes: the rows that
  // read the same rows of the folded children (2^lgR = the largest fold of the list, at most
  // 256 / T), so that those are fetched from memory once; its nodes share the filters' rows.
  const int rl = threadIdx.x / T, t = threadIdx.x % T;
  const int lgR = a.lg_rows, span = Sr >> lgR;
  const int kr = static_cast<int>(blockIdx.x % span) + (rl & ((1 << lgR) - 1)) * span;
  const long node_raw = static_cast<long>(blockIdx.x / span) * (RPB >> lgR) + (rl >> lgR);
  const bool valid = node_raw < nodes;
  const long node = valid ? node_raw : nodes - 1;  // idle groups redo the last node, unstored
  const long row = node * Sr + kr;
  float2 acc[E];
#pragma unroll
  for (int i = 0; i < E; ++i) acc[i] = make_float2(0.f, 0.f);
  for (int ci = 0; ci < a.n; ++ci) {
    const Rows2dAdjChild &ch = a.c[ci];
    const int Mr = Sr >> ch.lg_fr, m = Sc >> ch.lg_fc;
    const long cnode = ch.K > 0 ? (node / ch.cm.G) * ch.K + chan(ch.cm, static_cast<int>(node % ch.cm.G))
                                : node * ch.cm.G + ch.cm.base;
    const float2 *sp = ch.src + (static_cast<size_t>(cnode) * Mr + (kr & (Mr - 1))) * m;
    // lane t needs the child's row at (t + T i) mod m: its first EP = m / T values, repeated
    // (below T points: the single value at t mod m).  EP is the same for the whole launch's
    // lanes, so the accumulate is specialised on it: EP loads at fixed offsets, no masks.
    const float fr = ch.filt_row != nullptr ? ch.filt_row[kr] : 1.f;
    const float *fp = ch.filt_row != nullptr ? ch.filt + t : ch.filt + static_cast<size_t>(kr) * Sc + t;
    const int lgEP = (lgSc - ch.lg_fc) - lgT;
    if constexpr (T <= E) {
      if (ch.pre_rows) {  // (full-length rows only, checked by the launcher)
        rows2d_accumulate_fft<E, T>(acc, sp + t, fp, fr, t, lds + rl * XS, wtab);
        continue;
      }
    }
    switch (lgEP) {
      case 0: rows2d_accumulate<E, T, 1>(acc, sp + t, fp, fr); break;
      case 1: rows2d_accumulate<E, T, 2>(acc, sp + t, fp, fr); break;
      case 2: rows2d_accumulate<E, T, 4>(acc, sp + t, fp, fr); break;
      case 3: rows2d_accumulate<E, T, 8>(acc, sp + t, fp, fr); break;
      case 4: rows2d_accumulate<E, T, 16>(acc, sp + t, fp, fr); break;
      default: rows2d_accumulate<E, T, 1>(acc, sp + (t & (m - 1)), fp, fr); break;  // m < T
    }
  }
  if constexpr (T <= E) {  // (512-point rows, T = 32: no transform here, see the launcher)
    if (a.inverse) {
      float2 wt[E];
      load_twiddles<E, T>(wt, t, tw, tw_n);
      fft_core<E, T, true, true>(acc, t, lds + rl * XS, T + 1, 1, wt);
    }
  }
  if (!valid) return;
  float2 *dp = dst + static_cast<size_t>(row) * Sc + t;
  if (a.accumulate) {
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const float2 o = dp[T * i];
      acc[i].x += o.x;
      acc[i].y += o.y;
    }
  }
#pragma unroll
  for (int i = 0; i < E; ++i) dp[T * i] = acc[i];
}

// ------------------------------------------------------------------------------------
// Modulus backward step of whole nodes of N1 x N2 points (at most 16384) in one pass, the
// node held by one workgroup (slab_fft.hpp): gradient spectrum -> inverse 2-D transform ->
// a = Re(a) y / |y| against the taped y -> forward 2-D transform -> gradient spectrum of y.
// LOW: the incoming spectrum is the node's adjoint lowpass, built on the fly from the small
// transform ghat [node][m_r][m_c] of its output gradient: ghat tiled over the node times
// phi_rows[k_r] phi_cols[k_c]; otherwise it is read from `data` (and replaced).
// Per point: the tape read and the spectrum written (plus the spectrum read without LOW),
// where the separate row and column passes read and write the node three times.
template <int N1, int N2, bool LOW, bool YROWS>
__global__ __launch_bounds__((Slab<N1, N2>::NT)) void k_node_modback(
    const float2 *__restrict__ ghat, int m_r, int m_c, const float *__restrict__ phi_rows,
    const float *__restrict__ phi_cols, const float2 *__restrict__ y, float2 *__restrict__ data,
    long nodes, const float2 *__restrict__ tw, int tw_n) {
  using S = Slab<N1, N2>;
  extern __shared__ float2 lds[];
  const int s = threadIdx.x / S::TS, q = threadIdx.x % S::TS;
  const long node_raw = static_cast<long>(blockIdx.x) * S::SPW + s;
  const bool live = node_raw < nodes;
  const long node = live ? node_raw : nodes - 1;  // idle threads shadow the last node, store nothing
  float2 *area = lds + s * N1 * S::RS;
  float2 *wtab = lds + S::SPW * N1 * S::RS;  // the transforms' twiddles, shared by the slabs
  S::fill_twiddles(wtab, tw, tw_n);
  const int r = q / S::T2, t = q % S::T2;
  const int c = q % N2, t1 = q / N2;
  const size_t base = static_cast<size_t>(node) * N1 * N2;
  float2 *row = data + base + r * N2 + t;
  float2 v[16];
  if (LOW) {
    const float2 *gp = ghat + static_cast<size_t>(node) * m_r * m_c + (r & (m_r - 1)) * m_c;
    const float fr = phi_rows[r];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int kc = t + S::T2 * i;
      const float2 g = gp[kc & (m_c - 1)];
      const float f = fr * phi_cols[kc];
      v[i] = make_float2(g.x * f, g.y * f);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = row[S::T2 * i];
  }
  // the tape values are requested before the inverse transform and used after it (loads do
  // not move across its barriers by themselves)
  float2 yv[16];
  {
    const float2 *yp = y + base + c;
#pragma unroll
    for (int i = 0; i < 16; ++i) yv[i] = yp[(t1 + S::T1 * i) * N2];
  }
  S::template transform_tab<true>(v, area, r, t, c, t1, wtab);
  // YROWS: `y` holds the forward row pass's output (the node before its inverse column
  // transform); the columns are transformed here, which spares the forward pass that kernel
  // and the tape one write and one read of the node
  if (YROWS) fft_core_tab<16, S::T1, true, false>(yv, t1, area + c, S::T1 * S::RS, S::RS, wtab + N2 + t1, S::T1);
  {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float2 u = yv[i];
      const float m2 = u.x * u.x + u.y * u.y;
      const float sgn = over_sqrt(v[i].x, m2);
      v[i] = make_float2(u.x * sgn, u.y * sgn);
    }
  }
  S::template transform_back_tab<false>(v, area, r, t, c, t1, wtab);
  if (live) {
#pragma unroll
    for (int i = 0; i < 16; ++i) row[S::T2 * i] = v[i];
  }
}

}  // namespace

bool backward_side_supported(int m) { return pow2(m) && m >= 4 && m <= 512; }

hipError_t launch_fft_rows_inplace(float2 *data, long rows, int Mc, bool inverse, const float2 *tw,
                                   int tw_n, hipStream_t st) {
  if (rows <= 0 || Mc == 1) return hipSuccess;
  if (!pow2(Mc) || Mc > 512 || tw_n % Mc != 0) return hipErrorInvalidValue;
#define SCAT_ROWS(E_, T_) return rows_t<E_, T_>(data, rows, inverse, tw, tw_n, st)
  switch (Mc) {
    case 2: SCAT_ROWS(2, 1);
    case 4: SCAT_ROWS(4, 1);
    case 8: SCAT_ROWS(8, 1);
    case 16: SCAT_ROWS(16, 1);
    case 32: SCAT_ROWS(16, 2);
    case 64: SCAT_ROWS(16, 4);
    case 128: SCAT_ROWS(16, 8);
    case 256: SCAT_ROWS(16, 16);
    default: SCAT_ROWS(32, 16);
  }
#undef SCAT_ROWS
}

hipError_t launch_cols_modback(float2 *data, const float2 *y, long nodes, int Mr, int Mc,
                               const float2 *tw, int tw_n, hipStream_t st, int tw_m, bool y_rows) {
  if (nodes <= 0) return hipSuccess;
  if (!backward_side_supported(Mr) || !pow2(Mc) || Mc > 512 || tw_n % Mr != 0 ||
      (tw_m > 0 && (!pow2(tw_m) || tw_n % tw_m != 0)))
    return hipErrorInvalidValue;
#define SCAT_CM(E_, T_) return cols_modback_t<E_, T_>(data, y, nodes, Mc, tw_m, y_rows, tw, tw_n, st)
  switch (Mr) {
    case 4: SCAT_CM(4, 1);
    case 8: SCAT_CM(8, 1);
    case 16: SCAT_CM(16, 1);
    case 32: SCAT_CM(16, 2);
    case 64: SCAT_CM(16, 4);
    case 128: SCAT_CM(16, 8);
    case 256: SCAT_CM(16, 16);
    default: SCAT_CM(32, 16);
  }
#undef SCAT_CM
}

hipError_t launch_fft_cols_inplace(float2 *data, long nodes, int Mr, int Mc, bool inverse,
                                   const float2 *tw, int tw_n, hipStream_t st) {
  if (nodes <= 0 || Mr == 1) return hipSuccess;
  if (!pow2(Mr) || Mr > 512 || !pow2(Mc) || tw_n % Mr != 0) return hipErrorInvalidValue;
#define SCAT_COLS1(E_, T_) return cols_t<E_, T_>(data, nodes, Mc, inverse, tw, tw_n, st)
  switch (Mr) {
    case 2: SCAT_COLS1(2, 1);
    case 4: SCAT_COLS1(4, 1);
    case 8: SCAT_COLS1(8, 1);
    case 16: SCAT_COLS1(16, 1);
    case 32: SCAT_COLS1(16, 2);
    case 64: SCAT_COLS1(16, 4);
    case 128: SCAT_COLS1(16, 8);
    case 256: SCAT_COLS1(16, 16);
    default: SCAT_COLS1(32, 16);
  }
#undef SCAT_COLS1
}

unsigned grid_for(long count) {
  long b = (count + 255) / 256;
  if (b > 65536 * 16) b = 65536 * 16;
  return static_cast<unsigned>(b < 1 ? 1 : b);
}

hipError_t launch_twiddle(float2 *data, long nodes, int n1, int Mc, bool conj, const float2 *tw,
                          int tw_n, hipStream_t st) {
  const long count = nodes * n1 * Mc;
  const long m = static_cast<long>(n1) * Mc;
  if (count <= 0 || Mc == 1) return hipSuccess;  // k1 * 0 = 0: no twiddle with one column
  if (!pow2(n1) || !pow2(Mc) || m > tw_n || tw_n % m != 0) return hipErrorInvalidValue;
  LaunchScope obs("k_twiddle", count * 16.0, count * 6.0, st);
  hipLaunchKernelGGL(k_twiddle, dim3(grid_for(count)), dim3(256), 0, st, data, count, ilog2h(Mc),
                     ilog2h(n1), static_cast<int>(m), conj ? 1 : 0, tw, tw_n);
  return hipGetLastError();
}

hipError_t launch_gather_real(const float *gout, long nodes, ChanMap cm, int K, int m, float2 *dst,
                              hipStream_t st) {
  const long count = nodes * m;
  if (count <= 0) return hipSuccess;
  LaunchScope obs("k_gather_real", count * 12.0, 0.0, st);
  hipLaunchKernelGGL(k_gather_real, dim3(grid_for(count)), dim3(256), 0, st, gout, cm, K, m, dst,
                     count);
  return hipGetLastError();
}

hipError_t launch_tile_filter(const float2 *ghat, const float *filt, float2 *dst, long nodes, int n1,
                              int Mc, int mc, hipStream_t st) {
  const long count = nodes * n1 * Mc;
  if (count <= 0) return hipSuccess;
  if (!pow2(n1) || !pow2(Mc) || !pow2(mc) || mc > Mc) return hipErrorInvalidValue;
  LaunchScope obs("k_tile_filter", count * 8.0 + nodes * 8.0 * n1 * mc + 4.0 * n1 * Mc, count * 2.0,
                  st);
  hipLaunchKernelGGL(k_tile_filter, dim3(grid_for(count)), dim3(256), 0, st, ghat, filt, dst, count,
                     ilog2h(n1), ilog2h(Mc), ilog2h(mc));
  return hipGetLastError();
}

// node shapes of k_node_modback: sides 16 ... 128, square or 2 : 1
bool node_modback_supported(int Mr, int Mc) {
  return pow2(Mr) && pow2(Mc) && Mr >= 16 && Mc >= 16 && Mr <= 128 && Mc <= 128 &&
         (Mr == Mc || Mr == 2 * Mc || Mc == 2 * Mr);
}

// output grids whose gradient planes launch_small_fft2 transforms: up to 1024 points by the
// dense kernel, or a slab shape
bool small_fft2_supported(int m_r, int m_c) {
  return pow2(m_r) && pow2(m_c) && (m_r * m_c <= 1024 || node_modback_supported(m_r, m_c));
}

#define SCAT_NODE_DISPATCH(CALL)            \
  switch ((Mr << 12) | Mc) {                \
    case (16 << 12) | 16: CALL(16, 16);     \
    case (16 << 12) | 32: CALL(16, 32);     \
    case (32 << 12) | 16: CALL(32, 16);     \
    case (32 << 12) | 32: CALL(32, 32);     \
    case (32 << 12) | 64: CALL(32, 64);     \
    case (64 << 12) | 32: CALL(64, 32);     \
    case (64 << 12) | 64: CALL(64, 64);     \
    case (64 << 12) | 128: CALL(64, 128);   \
    case (128 << 12) | 64: CALL(128, 64);   \
    case (128 << 12) | 128: CALL(128, 128); \
    default: return hipErrorInvalidValue;   \
  }

template <int N1, int N2>
hipError_t slab_fft2_real_t(const float *gout, long nodes, ChanMap cm, int K, float2 *ghat,
                            const float2 *tw, int tw_n, hipStream_t st) {
  using S = Slab<N1, N2>;
  const long blocks = (nodes + S::SPW - 1) / S::SPW;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const std::string name = "k_slab_fft2_real<" + std::to_string(N1) + ", " + std::to_string(N2) + ">";
  const double pts = static_cast<double>(nodes) * N1 * N2;
  LaunchScope obs(name.c_str(), pts * 12.0, pts * 5.0 * (ilog2h(N1) + ilog2h(N2)), st);
  if (S::lds_bytes > 65536) {
    static unsigned long long lds_ok = 0;
    hipError_t e = allow_large_lds(reinterpret_cast<const void *>(k_slab_fft2_real<N1, N2>), lds_ok);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((k_slab_fft2_real<N1, N2>), dim3(static_cast<unsigned>(blocks)), dim3(S::NT),
                     S::lds_bytes, st, gout, cm, K, ghat, nodes, tw, tw_n);
  return hipGetLastError();
}

// ghat [node][m_r][m_c] = FFT2 of the nodes' output gradient planes
hipError_t launch_small_fft2(const float *gout, long nodes, ChanMap cm, int K, int m_r, int m_c,
                             float2 *ghat, const float2 *tw, int tw_n, hipStream_t st) {
  if (nodes <= 0) return hipSuccess;
  if (!small_fft2_supported(m_r, m_c) || tw_n % m_r != 0 || tw_n % m_c != 0 ||
      nodes > 0x7fffffffL || cm.G < 1 || cm.inner < 1 || nodes % cm.G != 0)
    return hipErrorInvalidValue;
  if (node_modback_supported(m_r, m_c)) {
    const int Mr = m_r, Mc = m_c;
#define SCAT_SF(A_, B_) return slab_fft2_real_t<A_, B_>(gout, nodes, cm, K, ghat, tw, tw_n, st)
    SCAT_NODE_DISPATCH(SCAT_SF)
#undef SCAT_SF
  }
  const int mm = m_r * m_c;
  const int npw = mm < 256 ? 256 / mm : 1;  // nodes per workgroup
  const long blocks = (nodes + npw - 1) / npw;
  const size_t lds = static_cast<size_t>(npw) * mm * (sizeof(float2) + sizeof(float)) +
                     static_cast<size_t>(m_r + m_c) * sizeof(float2);
  LaunchScope obs("k_small_fft2", nodes * 12.0 * m_r * m_c, nodes * 8.0 * m_r * m_c * (m_r + m_c), st);
  hipLaunchKernelGGL(k_small_fft2, dim3(static_cast<unsigned>(blocks)), dim3(256), lds, st, gout, cm, K,
                     m_r, m_c, npw, nodes, ghat, tw, tw_n);
  return hipGetLastError();
}

// Adjoint lowpass fused with the inverse row transform: dst [nodes][Mr][Mc] = inverse row
// FFT of ( FFT2(g_out node)[k mod m] phi_rows[k_r] phi_cols[k_c] ); `ghat` is scratch for
// the small transforms, nodes * m_r * m_c elements.
hipError_t launch_lowpass_adj_rows(const float *gout, long nodes, ChanMap cm, int K, int m_r,
                                   int m_c, int Mr, int Mc, const float *phi_rows,
                                   const float *phi_cols, float2 *ghat, float2 *dst,
                                   const float2 *tw, int tw_n, hipStream_t st) {
  if (nodes <= 0) return hipSuccess;
  if (!pow2(m_r) || !pow2(m_c) || !backward_side_supported(Mr) || !backward_side_supported(Mc) ||
      m_r > Mr || m_c > Mc || !small_fft2_supported(m_r, m_c) || tw_n % Mc != 0 || tw_n % m_r != 0 ||
      tw_n % m_c != 0 || nodes > 0x7fffffffL)
    return hipErrorInvalidValue;
  {
    hipError_t e = launch_small_fft2(gout, nodes, cm, K, m_r, m_c, ghat, tw, tw_n, st);
    if (e != hipSuccess) return e;
  }
#define SCAT_RLA(E_, T_) \
  return rows_lowpass_adj_t<E_, T_>(ghat, nodes, m_r, m_c, Mr, phi_rows, phi_cols, dst, tw, tw_n, st)
  switch (Mc) {
    case 4: SCAT_RLA(4, 1);
    case 8: SCAT_RLA(8, 1);
    case 16: SCAT_RLA(16, 1);
    case 32: SCAT_RLA(16, 2);
    case 64: SCAT_RLA(16, 4);
    case 128: SCAT_RLA(16, 8);
    case 256: SCAT_RLA(16, 16);
    default: SCAT_RLA(32, 16);
  }
#undef SCAT_RLA
}

hipError_t launch_take_real(const float2 *a, float *out, long count, hipStream_t st) {
  if (count <= 0) return hipSuccess;
  long blocks = (count + 255) / 256;
  if (blocks > 65536 * 16) blocks = 65536 * 16;
  LaunchScope obs("k_take_real", count * 12.0, 0.0, st);
  hipLaunchKernelGGL(k_take_real, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, a, out,
                     count);
  return hipGetLastError();
}

hipError_t launch_tile_accum(float2 *dst, const float *filt, const float2 *G, long S, int F, int Sr,
                             int Sc, int Mr, int Mc, hipStream_t st) {
  if (S <= 0 || F <= 0) return hipSuccess;
  if (!pow2(Sr) || !pow2(Sc) || !pow2(Mr) || !pow2(Mc) || Mr > Sr || Mc > Sc)
    return hipErrorInvalidValue;
  constexpr int SB = 4;
  const long count = ((S + SB - 1) / SB) * Mr * Mc;
  const long blocks = (count + 255) / 256;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  LaunchScope obs("k_tile_accum<8, 4>",
                  S * 16.0 * Sr * Sc + static_cast<double>(F) * Sr * Sc * 4 + S * F * 8.0 * Mr * Mc,
                  S * 4.0 * F * Sr * Sc, st);
  hipLaunchKernelGGL((k_tile_accum<8, SB>), dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st,
                     dst, filt, G, count, S, F, ilog2h(Sr), ilog2h(Sc), ilog2h(Mr), ilog2h(Mc));
  return hipGetLastError();
}

template <int E, int T>
hipError_t launch_rows1d_adj_t(float2 *dst, long rows, int Sr, const Rows1dAdjArgs &a, double bytes,
                               double flops, const float2 *tw, int tw_n, hipStream_t st) {
  constexpr int Sc = E * T, RPB = 256 / T;
  constexpr int XS = T == 1 ? E : E * (T + 1);  // as in the kernel
  const long blocks = (rows + RPB - 1) / RPB;
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const size_t lds = (static_cast<size_t>(Sc) + static_cast<size_t>(RPB) * XS) * sizeof(float2);
  const std::string name = "k_rows1d_adj<" + std::to_string(E) + ", " + std::to_string(T) + ">";
  LaunchScope obs(name.c_str(), bytes, flops, st);
  hipLaunchKernelGGL((k_rows1d_adj<E, T>), dim3(static_cast<unsigned>(blocks)), dim3(256), lds, st, dst,
                     rows, Sr, a, tw, tw_n);
  return hipGetLastError();
}

bool rows1d_adj_supported(int Sc) { return Sc >= 4 && Sc <= 256 && pow2(Sc); }

hipError_t launch_rows1d_adj(float2 *dst, long nodes, int Sr, int Sc, const Rows1dAdjArgs &a,
                             const float2 *tw, int tw_n, hipStream_t st) {
  if (nodes <= 0) return hipSuccess;
  if (a.n < 0 || a.n > kRows1dMaxChildren || !pow2(Sr) || !rows1d_adj_supported(Sc) || tw_n % Sc != 0)
    return hipErrorInvalidValue;
  const int lgSc = ilog2h(Sc);
  double bytes = static_cast<double>(nodes) * Sr * Sc * (a.accumulate ? 16 : 8), flops = 5.0 * Sc * lgSc;
  for (int i = 0; i < a.n; ++i) {
    const Rows1dAdjChild &c = a.c[i];
    if (c.src == nullptr || c.filt == nullptr || c.lg_fold < 0 || c.lg_fold > lgSc ||
        c.cm.G < 1 || (c.K == 0 && (c.cm.base < 0 || c.cm.base >= c.cm.G)) ||
        (c.K > 0 && (c.cm.inner < 1 || nodes % c.cm.G != 0)))
      return hipErrorInvalidValue;
    const double m = static_cast<double>(Sc >> c.lg_fold);
    bytes += static_cast<double>(Sr) * Sc * 4 + static_cast<double>(nodes) * Sr * m * 8;
    flops += 4.0 * Sc + 5.0 * m * (lgSc - c.lg_fold);
  }
  const double all_flops = static_cast<double>(nodes) * Sr * flops;
  const long rows = nodes * Sr;
  switch (Sc) {
    case 4: return launch_rows1d_adj_t<4, 1>(dst, rows, Sr, a, bytes, all_flops, tw, tw_n, st);
    case 8: return launch_rows1d_adj_t<8, 1>(dst, rows, Sr, a, bytes, all_flops, tw, tw_n, st);
    case 16: return launch_rows1d_adj_t<16, 1>(dst, rows, Sr, a, bytes, all_flops, tw, tw_n, st);
    case 32: return launch_rows1d_adj_t<16, 2>(dst, rows, Sr, a, bytes, all_flops, tw, tw_n, st);
    case 64: return launch_rows1d_adj_t<16, 4>(dst, rows, Sr, a, bytes, all_flops, tw, tw_n, st);
    case 128: return launch_rows1d_adj_t<16, 8>(dst, rows, Sr, a, bytes, all_flops, tw, tw_n, st);
    default: return launch_rows1d_adj_t<16, 16>(dst, rows, Sr, a, bytes, all_flops, tw, tw_n, st);
  }
}

template <int N1, int N2, bool LOW, bool YROWS>
hipError_t node_modback_t(const float2 *ghat, int m_r, int m_c, const float *phi_rows,
                          const float *phi_cols, const float2 *y, float2 *data, long nodes,
                          const float2 *tw, int tw_n, hipStream_t st) {
  using S = Slab<N1, N2>;
  const long blocks = (nodes + S::SPW - 1) / S::SPW;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const std::string name = "k_node_modback<" + std::to_string(N1) + ", " + std::to_string(N2) +
                           (LOW ? ", true" : ", false") + (YROWS ? ", true>" : ", false>");
  const double pts = static_cast<double>(nodes) * N1 * N2;
  LaunchScope obs(name.c_str(), pts * (LOW ? 16.0 : 24.0) + (LOW ? nodes * 8.0 * m_r * m_c : 0.0),
                  pts * (10.0 * (ilog2h(N1) + ilog2h(N2)) + 8.0 + (YROWS ? 5.0 * ilog2h(N1) : 0.0)), st);
  const size_t lds = S::lds_bytes + S::tab_elems * sizeof(float2);
  if (lds > 65536) {
    static unsigned long long lds_ok = 0;
    hipError_t e = allow_large_lds(reinterpret_cast<const void *>(k_node_modback<N1, N2, LOW, YROWS>), lds_ok);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((k_node_modback<N1, N2, LOW, YROWS>), dim3(static_cast<unsigned>(blocks)), dim3(S::NT),
                     lds, st, ghat, m_r, m_c, phi_rows, phi_cols, y, data, nodes, tw, tw_n);
  return hipGetLastError();
}

hipError_t launch_node_modback(float2 *data, const float2 *y, long nodes, int Mr, int Mc,
                               const float2 *tw, int tw_n, hipStream_t st, bool y_rows) {
  if (nodes <= 0) return hipSuccess;
  if (!node_modback_supported(Mr, Mc) || tw_n % Mr != 0 || tw_n % Mc != 0 || data == nullptr ||
      y == nullptr)
    return hipErrorInvalidValue;
#define SCAT_NM(A_, B_)                                                                          \
  return y_rows ? node_modback_t<A_, B_, false, true>(nullptr, 1, 1, nullptr, nullptr, y, data,  \
                                                      nodes, tw, tw_n, st)                       \
                : node_modback_t<A_, B_, false, false>(nullptr, 1, 1, nullptr, nullptr, y, data, \
                                                       nodes, tw, tw_n, st)
  SCAT_NODE_DISPATCH(SCAT_NM)
#undef SCAT_NM
}

hipError_t launch_node_modback_low(const float *gout, long nodes, ChanMap cm, int K, int m_r, int m_c,
                                   int Mr, int Mc, const float *phi_rows, const float *phi_cols,
                                   float2 *ghat, const float2 *y, float2 *dst, const float2 *tw,
                                   int tw_n, hipStream_t st, bool y_rows) {
  if (nodes <= 0) return hipSuccess;
  if (!node_modback_supported(Mr, Mc) || !small_fft2_supported(m_r, m_c) || m_r > Mr || m_c > Mc ||
      tw_n % Mr != 0 || tw_n % Mc != 0 || tw_n % m_r != 0 || tw_n % m_c != 0 ||
      nodes > 0x7fffffffL || cm.G < 1 || cm.inner < 1 || nodes % cm.G != 0)
    return hipErrorInvalidValue;
  {
    hipError_t e = launch_small_fft2(gout, nodes, cm, K, m_r, m_c, ghat, tw, tw_n, st);
    if (e != hipSuccess) return e;
  }
#define SCAT_NL(A_, B_)                                                                           \
  return y_rows ? node_modback_t<A_, B_, true, true>(ghat, m_r, m_c, phi_rows, phi_cols, y, dst, \
                                                     nodes, tw, tw_n, st)                        \
                : node_modback_t<A_, B_, true, false>(ghat, m_r, m_c, phi_rows, phi_cols, y, dst, \
                                                      nodes, tw, tw_n, st)
  SCAT_NODE_DISPATCH(SCAT_NL)
#undef SCAT_NL
}

template <int E, int T>
hipError_t launch_rows2d_adj_t(float2 *dst, long nodes, int Sr, Rows2dAdjArgs a, double bytes,
                               double flops, const float2 *tw, int tw_n, hipStream_t st) {
  constexpr int RPB = 256 / T;
  constexpr int XS = T == 1 ? E : E * (T + 1);  // as in the kernel
  // rows per node and workgroup: the largest row fold of the list (see the kernel)
  a.lg_rows = 0;
  for (int i = 0; i < a.n; ++i)
    if (a.c[i].lg_fr > a.lg_rows) a.lg_rows = a.c[i].lg_fr;
  while ((1 << a.lg_rows) > RPB || (1 << a.lg_rows) > Sr) --a.lg_rows;
  const int npb = RPB >> a.lg_rows;
  const long blocks = ((nodes + npb - 1) / npb) * (Sr >> a.lg_rows);
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  a.any_pre_rows = 0;
  for (int i = 0; i < a.n; ++i)
    if (a.c[i].pre_rows) a.any_pre_rows = 1;
  const size_t lds = T > E ? 0 : (static_cast<size_t>(RPB) * XS + E * T) * sizeof(float2);
  const std::string name = "k_rows2d_adj<" + std::to_string(E) + ", " + std::to_string(T) + ">";
  LaunchScope obs(name.c_str(), bytes, flops, st);
  hipLaunchKernelGGL((k_rows2d_adj<E, T>), dim3(static_cast<unsigned>(blocks)), dim3(256), lds, st, dst,
                     nodes, Sr, a, tw, tw_n);
  return hipGetLastError();
}

// row lengths of k_rows2d_adj: 4 ... 512, the inverse row transform up to 256
bool rows2d_adj_supported(int Sc, bool inverse) {
  return pow2(Sc) && Sc >= 4 && Sc <= (inverse ? 256 : 512);
}

hipError_t launch_rows2d_adj(float2 *dst, long nodes, int Sr, int Sc, const Rows2dAdjArgs &a,
                             const float2 *tw, int tw_n, hipStream_t st) {
  if (nodes <= 0) return hipSuccess;
  if (a.n < 0 || a.n > kRows1dMaxChildren || !pow2(Sr) || !rows2d_adj_supported(Sc, a.inverse != 0) ||
      tw_n % Sc != 0)
    return hipErrorInvalidValue;
  const int lgSc = ilog2h(Sc), lgSr = ilog2h(Sr);
  double bytes = static_cast<double>(nodes) * Sr * Sc * (a.accumulate ? 16 : 8);
  double flops = a.inverse ? 5.0 * Sc * lgSc : 0.0;
  for (int i = 0; i < a.n; ++i) {
    const Rows2dAdjChild &c = a.c[i];
    if (c.src == nullptr || c.filt == nullptr || c.lg_fr < 0 || c.lg_fr > lgSr || c.lg_fc < 0 ||
        c.lg_fc > lgSc || c.cm.G < 1 || (c.K == 0 && (c.cm.base < 0 || c.cm.base >= c.cm.G)) ||
        (c.K > 0 && (c.cm.inner < 1 || nodes % c.cm.G != 0)) ||
        (c.pre_rows != 0 && (c.lg_fc != 0 || Sc > 256)))
      return hipErrorInvalidValue;
    if (c.pre_rows) flops += 5.0 * Sc * lgSc;
    bytes += (c.filt_row != nullptr ? 0.0 : static_cast<double>(Sr) * Sc * 4) +
             static_cast<double>(nodes) * (Sr >> c.lg_fr) * (Sc >> c.lg_fc) * 8;
    flops += 4.0 * Sc;
  }
  const double all_flops = static_cast<double>(nodes) * Sr * flops;
  switch (Sc) {
    case 4: return launch_rows2d_adj_t<4, 1>(dst, nodes, Sr, a, bytes, all_flops, tw, tw_n, st);
    case 8: return launch_rows2d_adj_t<8, 1>(dst, nodes, Sr, a, bytes, all_flops, tw, tw_n, st);
    case 16: return launch_rows2d_adj_t<16, 1>(dst, nodes, Sr, a, bytes, all_flops, tw, tw_n, st);
    case 32: return launch_rows2d_adj_t<16, 2>(dst, nodes, Sr, a, bytes, all_flops, tw, tw_n, st);
    case 64: return launch_rows2d_adj_t<16, 4>(dst, nodes, Sr, a, bytes, all_flops, tw, tw_n, st);
    case 128: return launch_rows2d_adj_t<16, 8>(dst, nodes, Sr, a, bytes, all_flops, tw, tw_n, st);
    case 256: return launch_rows2d_adj_t<16, 16>(dst, nodes, Sr, a, bytes, all_flops, tw, tw_n, st);
    default: return launch_rows2d_adj_t<16, 32>(dst, nodes, Sr, a, bytes, all_flops, tw, tw_n, st);
  }
}

}  // namespace scat
