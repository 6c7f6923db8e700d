// HIP kernels (gfx950) for the Fourier-domain scattering cascade, generic path.
//
// Every transform is a batched power-of-two FFT done entirely in LDS by one workgroup;
// a 2-D transform (and the four-step form of a long 1-D transform) is a row pass and a
// column pass.  The cascade's pointwise work is fused into the passes:
//   * k_mulfold_invrow : filter multiply + periodisation (sum of Fourier blocks, i.e.
//                        subsampling) on load, inverse row FFT, store
//   * k_col            : inverse column FFT, complex modulus, forward column FFT of the
//                        modulus, and (2-D) the column half of the separable lowpass with
//                        its subsampling, all on one tile of columns held in LDS
//   * k_row_fwd        : forward row FFT in place
//   * k_row_lowpass    : row half of the separable lowpass + subsampling, writes S
// Paper section 2 ("Implementation"): periodic convolutions via FFT, downsampled
// intermediates, modulus non-linearity.
#include <hip/hip_runtime.h>

#include "scat_kernels.hpp"

namespace scat {

namespace {

__device__ __forceinline__ float2 cmul(float2 a, float2 b) {
  return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }

__device__ __forceinline__ int bitrev(int i, int log2n) {
  return log2n == 0 ? 0 : static_cast<int>(__brev(static_cast<unsigned>(i)) >> (32 - log2n));
}

// Twiddle exp(-+ 2 pi i e / m) from the table tw[j] = exp(-2 pi i j / tw_n), m | tw_n.
template <bool INV>
__device__ __forceinline__ float2 twiddle(const float2 *__restrict__ tw, int tw_n, int e, int m) {
  float2 w = tw[e * (tw_n / m)];
  if (INV) w.y = -w.y;
  return w;
}

// In-place decimation-in-time FFT of `nseq` sequences of length n = 2^log2n living in
// LDS at buf[seq * seq_stride + i * elem_stride].  Input must be stored in bit-reversed
// order; output is in natural order.  Stages are taken two at a time (radix-2^2).
// SEQ_FAST: consecutive threads work on consecutive sequences (column tiles) rather
// than on consecutive butterflies of one sequence (row tiles).
// Starts and ends with a workgroup barrier.  Unnormalised in both directions.
template <bool INV, bool SEQ_FAST>
__device__ void lds_fft(float2 *buf, int log2n, int nseq, int seq_stride, int elem_stride,
                        const float2 *__restrict__ tw, int tw_n) {
  const int n = 1 << log2n;
  __syncthreads();
  int s = 0;
  if (log2n & 1) {
    const int nb = n >> 1;
    const int total = nseq * nb;
    for (int t = threadIdx.x; t < total; t += blockDim.x) {
      int seq = SEQ_FAST ? t % nseq : t / nb;
      int b = SEQ_FAST ? t / nseq : t % nb;
      float2 *p = buf + seq * seq_stride + (2 * b) * elem_stride;
      float2 x0 = p[0], x1 = p[elem_stride];
      p[0] = cadd(x0, x1);
      p[elem_stride] = csub(x0, x1);
    }
    s = 1;
    __syncthreads();
  }
  for (; s < log2n; s += 2) {
    const int h = 1 << s;
    const int nb = n >> 2;
    const int total = nseq * nb;
    for (int t = threadIdx.x; t < total; t += blockDim.x) {
      int seq = SEQ_FAST ? t % nseq : t / nb;
      int b = SEQ_FAST ? t / nseq : t % nb;
      int grp = b >> s;
      int j = b & (h - 1);
      float2 *p = buf + seq * seq_stride + ((grp << (s + 2)) + j) * elem_stride;
      const int hs = h * elem_stride;
      float2 x0 = p[0], x1 = p[hs], x2 = p[2 * hs], x3 = p[3 * hs];
      float2 w1 = twiddle<INV>(tw, tw_n, j, 2 * h);
      float2 w2 = twiddle<INV>(tw, tw_n, j, 4 * h);
      float2 t1 = cmul(w1, x1), t3 = cmul(w1, x3);
      float2 a0 = cadd(x0, t1), a1 = csub(x0, t1);
      float2 a2 = cadd(x2, t3), a3 = csub(x2, t3);
      float2 u2 = cmul(w2, a2);
      float2 u3 = cmul(w2, a3);
      // second stage twiddle of the odd pair is w2 * exp(-+ i pi / 2)
      u3 = INV ? make_float2(-u3.y, u3.x) : make_float2(u3.y, -u3.x);
      p[0] = cadd(a0, u2);
      p[2 * hs] = csub(a0, u2);
      p[hs] = cadd(a1, u3);
      p[3 * hs] = csub(a1, u3);
    }
    __syncthreads();
  }
}

__device__ __forceinline__ int ilog2(int v) { return 31 - __clz(v); }

// Output channel of node g (see ChanMap).
__device__ __forceinline__ int chan_of(const ChanMap &cm, int g) {
  return cm.base + (g / cm.inner) * cm.outer_stride + (g % cm.inner);
}

// ------------------------------------------------------------------------------------
// Filter multiply + fold + inverse row FFT.
// src  : [S][Sr][Sc] complex spectra; filt: [F][Sr][Sc] real (already carries 1/(Sr*Sc))
// dst  : [S*F][Mr][Mc] complex, Mr = Sr >> fr, Mc = Sc >> fc:
//        dst[q_r][.] = IFFT_cols-index( sum_{a,b} src[q_r + a Mr][q_c + b Mc] * filt[same] )
// post_tw_m > 0 (1-D four-step inverse): multiply dst[q_r][b] by exp(+2 pi i q_r b / post_tw_m).
// One workgroup handles RB consecutive output rows of one (source, filter) pair.
__global__ void k_mulfold_invrow(const float2 *__restrict__ src, const float *__restrict__ filt,
                                 float2 *__restrict__ dst, int F, int Sr, int Sc, int fr, int fc,
                                 int RB, int post_tw_m, const float2 *__restrict__ tw, int tw_n) {
  extern __shared__ float2 lds[];
  const int Mr = Sr >> fr, Mc = Sc >> fc;
  const int log2mc = ilog2(Mc);
  const int blocks_per_pair = Mr / RB;
  const int pair = blockIdx.x / blocks_per_pair;
  const int r0 = (blockIdx.x % blocks_per_pair) * RB;
  const int s_idx = pair / F, f_idx = pair % F;
  const float2 *sp = src + static_cast<size_t>(s_idx) * Sr * Sc;
  const float *fp = filt + static_cast<size_t>(f_idx) * Sr * Sc;
  const int nfr = 1 << fr, nfc = 1 << fc;
  for (int t = threadIdx.x; t < RB * Mc; t += blockDim.x) {
    int row = t / Mc, qc = t % Mc;
    int qr = r0 + row;
    float2 acc = make_float2(0.f, 0.f);
    for (int a = 0; a < nfr; ++a) {
      size_t ro = static_cast<size_t>(qr + a * Mr) * Sc;
      for (int b = 0; b < nfc; ++b) {
        size_t o = ro + qc + b * Mc;
        float2 v = sp[o];
        float f = fp[o];
        acc.x += v.x * f;
        acc.y += v.y * f;
      }
    }
    lds[row * Mc + bitrev(qc, log2mc)] = acc;
  }
  lds_fft<true, false>(lds, log2mc, RB, Mc, 1, tw, tw_n);
  float2 *dp = dst + (static_cast<size_t>(pair) * Mr + r0) * Mc;
  for (int t = threadIdx.x; t < RB * Mc; t += blockDim.x) {
    float2 v = lds[t];
    if (post_tw_m > 0) {
      int row = t / Mc, b = t % Mc;
      int e = static_cast<int>((static_cast<long long>(r0 + row) * b) % post_tw_m);
      v = cmul(v, twiddle<true>(tw, tw_n, e, post_tw_m));
    }
    dp[t] = v;
  }
}

// ------------------------------------------------------------------------------------
// Column pass on a tile of TC columns of one node ([Mr][Mc] plane).
// MODE 0: src real; forward column FFT.
// MODE 1: src complex; inverse column FFT, modulus, forward column FFT.
// MODE 2: src complex; inverse column FFT, real part written to `out` (1-D final stage).
// MODE 0/1 outputs: `uc` (nullable) receives the forward column spectrum [node][k_r][c],
//   multiplied by exp(-2 pi i k_r c / post_tw_m) if post_tw_m > 0 (1-D four-step forward);
//   `w_out` (nullable, 2-D) receives the column half of the lowpass: for every column,
//   IFFT_{m_r}( fold_{Mr -> m_r}( spectrum[k_r] * phi_rows[k_r] ) ), real, [node][m_r][Mc].
template <int MODE>
__global__ void k_col(const void *__restrict__ src_v, int Mr, int Mc, int TC,
                      float2 *__restrict__ uc, int post_tw_m, const float *__restrict__ phi_rows,
                      int m_r, float *__restrict__ w_out, float *__restrict__ out, ChanMap cm,
                      int K, const float2 *__restrict__ tw, int tw_n) {
  extern __shared__ float2 lds[];
  const int log2mr = ilog2(Mr);
  const int tiles = Mc / TC;
  const int node = blockIdx.x / tiles;
  const int c0 = (blockIdx.x % tiles) * TC;
  const size_t plane = static_cast<size_t>(node) * Mr * Mc;
  const int total = Mr * TC;
  // load (bit-reversed along the column)
  for (int t = threadIdx.x; t < total; t += blockDim.x) {
    int i = t / TC, c = t % TC;
    float2 v;
    if (MODE == 0) {
      v = make_float2(static_cast<const float *>(src_v)[plane + static_cast<size_t>(i) * Mc + c0 + c], 0.f);
    } else {
      v = static_cast<const float2 *>(src_v)[plane + static_cast<size_t>(i) * Mc + c0 + c];
    }
    lds[bitrev(i, log2mr) * TC + c] = v;
  }
  if (MODE != 0) {
    lds_fft<true, true>(lds, log2mr, TC, 1, TC, tw, tw_n);
  }
  if (MODE == 2) {
    const int p = node / cm.G, g = node % cm.G;
    float *op = out + (static_cast<size_t>(p) * K + chan_of(cm, g)) * Mr * Mc;
    for (int t = threadIdx.x; t < total; t += blockDim.x) {
      int i = t / TC, c = t % TC;
      op[static_cast<size_t>(i) * Mc + c0 + c] = lds[t].x;
    }
    return;
  }
  if (MODE == 1) {
    // modulus, and put the result in bit-reversed order for the forward transform:
    // rows i and rev(i) swap places; the thread owning the smaller index does both.
    for (int t = threadIdx.x; t < total; t += blockDim.x) {
      int i = t / TC, c = t % TC;
      int ri = bitrev(i, log2mr);
      if (ri < i) continue;
      float2 a = lds[i * TC + c];
      float2 b = lds[ri * TC + c];
      float ma = sqrtf(a.x * a.x + a.y * a.y);
      float mb = sqrtf(b.x * b.x + b.y * b.y);
      lds[ri * TC + c] = make_float2(ma, 0.f);
      lds[i * TC + c] = make_float2(mb, 0.f);
    }
  }
  lds_fft<false, true>(lds, log2mr, TC, 1, TC, tw, tw_n);
  if (uc != nullptr) {
    for (int t = threadIdx.x; t < total; t += blockDim.x) {
      int i = t / TC, c = t % TC;
      float2 v = lds[t];
      if (post_tw_m > 0) {
        int e = static_cast<int>((static_cast<long long>(i) * (c0 + c)) % post_tw_m);
        v = cmul(v, twiddle<false>(tw, tw_n, e, post_tw_m));
      }
      uc[plane + static_cast<size_t>(i) * Mc + c0 + c] = v;
    }
  }
  if (w_out != nullptr) {
    float2 *low = lds + total;
    const int log2m = ilog2(m_r);
    const int nf = Mr / m_r;
    for (int t = threadIdx.x; t < m_r * TC; t += blockDim.x) {
      int m = t / TC, c = t % TC;
      float2 acc = make_float2(0.f, 0.f);
      for (int a = 0; a < nf; ++a) {
        int k = m + a * m_r;
        float2 v = lds[k * TC + c];
        float f = phi_rows[k];
        acc.x += v.x * f;
        acc.y += v.y * f;
      }
      low[bitrev(m, log2m) * TC + c] = acc;
    }
    lds_fft<true, true>(low, log2m, TC, 1, TC, tw, tw_n);
    float *wp = w_out + static_cast<size_t>(node) * m_r * Mc;
    for (int t = threadIdx.x; t < m_r * TC; t += blockDim.x) {
      int m = t / TC, c = t % TC;
      wp[static_cast<size_t>(m) * Mc + c0 + c] = low[t].x;
    }
  }
}

// ------------------------------------------------------------------------------------
// Forward row FFT in place: data [rows][Mc] complex, RB rows per workgroup.
__global__ void k_row_fwd(float2 *__restrict__ data, int Mc, int RB,
                          const float2 *__restrict__ tw, int tw_n) {
  extern __shared__ float2 lds[];
  const int log2mc = ilog2(Mc);
  float2 *dp = data + static_cast<size_t>(blockIdx.x) * RB * Mc;
  for (int t = threadIdx.x; t < RB * Mc; t += blockDim.x) {
    int row = t / Mc, c = t % Mc;
    lds[row * Mc + bitrev(c, log2mc)] = dp[t];
  }
  lds_fft<false, false>(lds, log2mc, RB, Mc, 1, tw, tw_n);
  for (int t = threadIdx.x; t < RB * Mc; t += blockDim.x) dp[t] = lds[t];
}

// ------------------------------------------------------------------------------------
// Row half of the separable lowpass (2-D): w [node][m_r][Mc] real ->
// out[p][chan][m_r][m_c] = IFFT_{m_c}( fold_{Mc -> m_c}( FFT_{Mc}(row) * phi_cols ) ).
// RB rows per workgroup (RB divides m_r).
__global__ void k_row_lowpass(const float *__restrict__ w, int m_r, int Mc, int m_c, int RB,
                              const float *__restrict__ phi_cols, float *__restrict__ out,
                              ChanMap cm, int K, const float2 *__restrict__ tw, int tw_n) {
  extern __shared__ float2 lds[];
  const int log2mc = ilog2(Mc), log2m = ilog2(m_c);
  const int blocks_per_node = m_r / RB;
  const int node = blockIdx.x / blocks_per_node;
  const int r0 = (blockIdx.x % blocks_per_node) * RB;
  const float *wp = w + (static_cast<size_t>(node) * m_r + r0) * Mc;
  for (int t = threadIdx.x; t < RB * Mc; t += blockDim.x) {
    int row = t / Mc, c = t % Mc;
    lds[row * Mc + bitrev(c, log2mc)] = make_float2(wp[t], 0.f);
  }
  lds_fft<false, false>(lds, log2mc, RB, Mc, 1, tw, tw_n);
  float2 *low = lds + RB * Mc;
  const int nf = Mc / m_c;
  for (int t = threadIdx.x; t < RB * m_c; t += blockDim.x) {
    int row = t / m_c, m = t % m_c;
    float2 acc = make_float2(0.f, 0.f);
    for (int b = 0; b < nf; ++b) {
      int k = m + b * m_c;
      float2 v = lds[row * Mc + k];
      float f = phi_cols[k];
      acc.x += v.x * f;
      acc.y += v.y * f;
    }
    low[row * m_c + bitrev(m, log2m)] = acc;
  }
  lds_fft<true, false>(low, log2m, RB, m_c, 1, tw, tw_n);
  const int p = node / cm.G, g = node % cm.G;
  float *op = out + ((static_cast<size_t>(p) * K + chan_of(cm, g)) * m_r + r0) * m_c;
  for (int t = threadIdx.x; t < RB * m_c; t += blockDim.x) op[t] = low[t].x;
}

constexpr int kThreads = 256;
constexpr int kTileElems = 4096;  // complex elements of one workgroup's LDS tile (32 KB)

int pow2_floor(int v) {
  int p = 1;
  while (2 * p <= v) p *= 2;
  return p;
}

}  // namespace

// ----------------------------------------------------------------------------- launchers

hipError_t launch_mulfold_invrow(const float2 *src, const float *filt, float2 *dst, long S, int F,
                                 int Sr, int Sc, int fr, int fc, int post_tw_m, const float2 *tw,
                                 int tw_n, hipStream_t st) {
  const int Mr = Sr >> fr, Mc = Sc >> fc;
  int RB = pow2_floor(kTileElems / Mc);
  if (RB > Mr) RB = Mr;
  if (RB < 1) return hipErrorInvalidValue;
  long blocks = S * F * (Mr / RB);
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  size_t lds = static_cast<size_t>(RB) * Mc * sizeof(float2);
  hipLaunchKernelGGL(k_mulfold_invrow, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), lds, st,
                     src, filt, dst, F, Sr, Sc, fr, fc, RB, post_tw_m, tw, tw_n);
  return hipGetLastError();
}

hipError_t launch_col(int mode, const void *src, long nodes, int Mr, int Mc, float2 *uc,
                      int post_tw_m, const float *phi_rows, int m_r, float *w_out, float *out,
                      ChanMap cm, int K, const float2 *tw, int tw_n, hipStream_t st) {
  int TC = pow2_floor(kTileElems / Mr);
  if (TC > 16) TC = 16;
  if (TC > Mc) TC = Mc;
  if (TC < 1) return hipErrorInvalidValue;
  long blocks = nodes * (Mc / TC);
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  size_t lds = (static_cast<size_t>(Mr) + (w_out ? m_r : 0)) * TC * sizeof(float2);
  dim3 g(static_cast<unsigned>(blocks)), b(kThreads);
  switch (mode) {
    case 0:
      hipLaunchKernelGGL(k_col<0>, g, b, lds, st, src, Mr, Mc, TC, uc, post_tw_m, phi_rows, m_r,
                         w_out, out, cm, K, tw, tw_n);
      break;
    case 1:
      hipLaunchKernelGGL(k_col<1>, g, b, lds, st, src, Mr, Mc, TC, uc, post_tw_m, phi_rows, m_r,
                         w_out, out, cm, K, tw, tw_n);
      break;
    case 2:
      hipLaunchKernelGGL(k_col<2>, g, b, lds, st, src, Mr, Mc, TC, uc, post_tw_m, phi_rows, m_r,
                         w_out, out, cm, K, tw, tw_n);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_row_fwd(float2 *data, long rows, int Mc, const float2 *tw, int tw_n,
                          hipStream_t st) {
  int RB = pow2_floor(kTileElems / Mc);
  while (RB > 1 && rows % RB != 0) RB >>= 1;
  if (RB < 1) return hipErrorInvalidValue;
  long blocks = rows / RB;
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  size_t lds = static_cast<size_t>(RB) * Mc * sizeof(float2);
  hipLaunchKernelGGL(k_row_fwd, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), lds, st, data,
                     Mc, RB, tw, tw_n);
  return hipGetLastError();
}

hipError_t launch_row_lowpass(const float *w, long nodes, int m_r, int Mc, int m_c,
                              const float *phi_cols, float *out, ChanMap cm, int K,
                              const float2 *tw, int tw_n, hipStream_t st) {
  int RB = pow2_floor(kTileElems / Mc);
  if (RB > m_r) RB = m_r;
  if (RB < 1) return hipErrorInvalidValue;
  long blocks = nodes * (m_r / RB);
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  size_t lds = static_cast<size_t>(RB) * (Mc + m_c) * sizeof(float2);
  hipLaunchKernelGGL(k_row_lowpass, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), lds, st, w,
                     m_r, Mc, m_c, RB, phi_cols, out, cm, K, tw, tw_n);
  return hipGetLastError();
}

}  // namespace scat
