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

#include <cmath>
#include <string>
#include <type_traits>

#include "fft_regs.hpp"
#include "slab_fft.hpp"
#include "scat_kernels.hpp"

namespace scat {

namespace {

thread_local LaunchObserver *g_observer = nullptr;

// 5 n log2 n, the usual flop model of one complex transform of n points
double fft_flops(double n) { return n > 1 ? 5.0 * n * std::log2(n) : 0.0; }

struct Observe {
  hipStream_t st;
  bool on;
  Observe(const char *name, double bytes, double flops, hipStream_t s) : st(s), on(g_observer != nullptr) {
    if (on) g_observer->before(name, bytes, flops, st);
  }
  ~Observe() {
    if (on) g_observer->after(st);
  }
};


}  // namespace

LaunchScope::LaunchScope(const char *name, double bytes, double flops, hipStream_t st)
    : st_(st), on_(g_observer != nullptr) {
  if (on_) g_observer->before(name, bytes, flops, st_);
}
LaunchScope::~LaunchScope() {
  if (on_) g_observer->after(st_);
}

namespace {

__device__ __forceinline__ float2 cmul(float2 a, float2 b) {
  return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }

// Streaming store: the value is written once and read much later by another kernel.
__device__ __forceinline__ void nt_store(float2 *p, float2 v) {
  __builtin_nontemporal_store(v.x, &p->x);
  __builtin_nontemporal_store(v.y, &p->y);
}

// The same for two adjacent complex values (16 bytes)
typedef float scat_v4f __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void nt_store4(float2 *p, float4 v) {
  scat_v4f x = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(x, reinterpret_cast<scat_v4f *>(p));
}
__device__ __forceinline__ float4 nt_load4(const float2 *p) {
  const scat_v4f x = __builtin_nontemporal_load(reinterpret_cast<const scat_v4f *>(p));
  return make_float4(x.x, x.y, x.z, x.w);
}

// Streaming load: the value is read exactly once.
__device__ __forceinline__ float2 nt_load(const float2 *p) {
  return make_float2(__builtin_nontemporal_load(&p->x), __builtin_nontemporal_load(&p->y));
}

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
// Forward row FFT in place, transform in registers (rows of E*T points, T lanes per row).
template <int E, int T>
__global__ __launch_bounds__(E == 32 ? 128 : 256) void k_row_fwd_reg(float2 *__restrict__ data,
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
  fft_core<E, T, false, true>(v, t, lds + rl * (E * (T + 1)), T + 1, 1, wt);
  if (!valid) return;
#pragma unroll
  for (int i = 0; i < E; ++i) p[T * i] = v[i];
}

// ------------------------------------------------------------------------------------
// k_mulfold_invrow with the transform in registers (output rows of E*T points, T lanes per
// row, only wave-level synchronisation).  Same contract; `rows` is the number of output rows
// per XCD (see below), lgMr = log2(Mr).
template <int E, int T, bool MULTI>
__global__ __launch_bounds__(E == 32 ? 128 : 256) void k_mulfold_reg(
    const float2 *__restrict__ src, const float *__restrict__ filt, float2 *__restrict__ dst,
    long rows, int F, int Sr, int Sc, int fr, int fc, int lgMr, int post_tw_m,
    const float2 *__restrict__ tw, int tw_n, const unsigned long long *__restrict__ mask) {
  constexpr int NT = E == 32 ? 128 : 256;
  constexpr int RPB = NT / T, M = E * T;
  extern __shared__ float2 lds[];
  const int rl = threadIdx.x / T, t = threadIdx.x % T;
  // Workgroups go round-robin to the 8 XCDs, each with its own L2.  XCD x takes the output
  // rows qr in [x Mr/8, (x+1) Mr/8) of every source, so it only ever reads its own eighth of
  // the filter tables (which then stays in its L2) and of every source.  Within an XCD rows
  // are numbered filter-fastest: the lane groups of a wave that work on the same output row
  // of different filters load the same source addresses (one fetch per wave).
  // `rows` = rows per XCD = S * (Mr/8) * F when lgMr >= 3, else all rows (no split).
  const bool split = lgMr >= 3;
  const int xcd = split ? static_cast<int>(blockIdx.x & 7) : 0;
  const long blk = split ? static_cast<long>(blockIdx.x >> 3) : static_cast<long>(blockIdx.x);
  const int lgQ = split ? lgMr - 3 : lgMr;
  const long row_raw = blk * RPB + rl;
  const bool valid = row_raw < rows;
  const long row = valid ? row_raw : rows - 1;  // idle groups redo the last row, unstored
  const int Mr = 1 << lgMr;
  const long sq = row / F;  // source * (rows of this XCD) + output row within the XCD's range
  const int f_idx = static_cast<int>(row - sq * F);
  const long s_idx = sq >> lgQ;
  const int qr = (xcd << lgQ) + static_cast<int>(sq & ((1 << lgQ) - 1));
  float2 v[E];
  const int nfr = 1 << fr, nfc = 1 << fc;
  if (M >= 64 || (M >= 32 && Sc >= 64)) {
    // The whole wave accumulates one row at a time, reading the source row W = max(M, 64)
    // contiguous columns per step (a lane owns M/64 consecutive columns, or one column when
    // M < 64; then the 64/M lanes that hold the same output column are summed by lane
    // exchange).  So source and filter reads are contiguous across the wave.  The row is
    // parked in its exchange area, where the T lanes of the row pick it up.
    constexpr int CPL = M >= 64 ? M / 64 : 1;
    constexpr int W = M >= 64 ? M : 64;
    constexpr int RW = 64 / T;  // rows per wave
    constexpr int XS = T == 1 ? E : E * (T + 1);
    const int nsteps = Sc / W;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
    float2 *xw = lds + wv * RW * XS;
    const long row0 = blk * RPB + wv * RW;
    // Rows are numbered filter-fastest, so a run of consecutive rows shares its source
    // row: with MULTI up to FB filters are accumulated at once from one read of the source
    // values (pays off for rows of 128 points and more and several filters; measured).
    constexpr int FB = !MULTI ? 1 : CPL == 1 ? 4 : CPL == 2 ? 8 : CPL == 4 ? 4 : 2;
    for (int r = 0; r < RW;) {
      long rr = row0 + r;
      if (rr >= rows) rr = rows - 1;
      const long sq_r = rr / F;
      const int f_r = static_cast<int>(rr - sq_r * F);
      int n = F - f_r;
      if (n > RW - r) n = RW - r;
      if (n > FB) n = FB;
      const long s_r = sq_r >> lgQ;
      const int q_r = (xcd << lgQ) + static_cast<int>(sq_r & ((1 << lgQ) - 1));
      const float2 *sp = src + static_cast<size_t>(s_r) * Sr * Sc + lane * CPL;
      const size_t fstride = static_cast<size_t>(Sr) * Sc;
      const float *fp = filt + static_cast<size_t>(f_r) * fstride + lane * CPL;
      float2 acc[FB][CPL];
#pragma unroll
      for (int j = 0; j < FB; ++j)
#pragma unroll
        for (int e = 0; e < CPL; ++e) acc[j][e] = make_float2(0.f, 0.f);
      // alias blocks (a, b) on which every filter of the run is negligible are left out (mask:
      // per filter, bit a * 2^fc + b set = block in use).  A test per filter inside the block measured slower: its branches
      // serialise the loads.
      unsigned long long used = ~0ull;
      if (mask != nullptr) {
        used = 0ull;
        for (int j = 0; j < n; ++j) used |= mask[f_r + j];
      }
      for (int a = 0; a < nfr; ++a) {
        const size_t ro = static_cast<size_t>(q_r + a * Mr) * Sc;
#pragma unroll 2
        for (int b = 0; b < nsteps; ++b) {
          // (a step covers W / M alias blocks: one for rows of 64 points and more)
          if (!((used >> ((a * nsteps + b) * (W / M))) & ((1ull << (W / M)) - 1ull))) continue;
          const size_t o = ro + static_cast<size_t>(b) * W;
          float2 x[CPL];
#pragma unroll
          for (int e = 0; e < CPL; ++e) x[e] = sp[o + e];
#pragma unroll
          for (int j = 0; j < FB; ++j) {
            // filters past the run repeat its last one (loaded, not stored)
            const float *fj = fp + static_cast<size_t>(j < n ? j : n - 1) * fstride;
#pragma unroll
            for (int e = 0; e < CPL; ++e) {
              const float f = fj[o + e];
              acc[j][e].x += x[e].x * f;
              acc[j][e].y += x[e].y * f;
            }
          }
        }
      }
      if (M < 64) {
#pragma unroll
        for (int j = 0; j < FB; ++j)
#pragma unroll
          for (int d = M; d < 64; d <<= 1) {
            acc[j][0].x += __shfl_xor(acc[j][0].x, d);
            acc[j][0].y += __shfl_xor(acc[j][0].y, d);
          }
      }
      if (lane * CPL < M) {
#pragma unroll
        for (int j = 0; j < FB; ++j)
          if (j < n) {
#pragma unroll
            for (int e = 0; e < CPL; ++e) xw[(r + j) * XS + lane * CPL + e] = acc[j][e];
          }
      }
      r += n;
    }
    wave_sync();
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = xw[(lane / T) * XS + t + T * i];
    wave_sync();
  } else {
    // short rows (the per-row cost of the wave-wide scheme outweighs its coalescing;
    // measured) or sources narrower than a wave: the T lanes of a row gather directly
    const float2 *sp = src + static_cast<size_t>(s_idx) * Sr * Sc + t;
    const float *fp = filt + static_cast<size_t>(f_idx) * Sr * Sc + t;
    const unsigned long long used = mask != nullptr ? mask[f_idx] : ~0ull;  // per row (its filter)
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = make_float2(0.f, 0.f);
    for (int a = 0; a < nfr; ++a) {
      const size_t ro = static_cast<size_t>(qr + a * Mr) * Sc;
      for (int b = 0; b < nfc; ++b) {
        if (!((used >> (a * nfc + b)) & 1ull)) continue;
        const size_t o = ro + static_cast<size_t>(b) * M;
#pragma unroll
        for (int i = 0; i < E; ++i) {
          const float2 x = sp[o + T * i];
          const float f = fp[o + T * i];
          v[i].x += x.x * f;
          v[i].y += x.y * f;
        }
      }
    }
  }
  float2 wt[E];
  load_twiddles<E, T>(wt, t, tw, tw_n);
  fft_core<E, T, true, true>(v, t, lds + rl * (T == 1 ? E : E * (T + 1)), T + 1, 1, wt);
  if (!valid) return;
  float2 *dp = dst + ((static_cast<size_t>(s_idx) * F + f_idx) * Mr + qr) * M + t;
  // (non-temporal where a row's T lanes write whole cache lines: the output is read much later,
  // by another kernel; for partial lines it measured slower)
  auto put = [](float2 *q, float2 val) {
    if constexpr (T >= 16) nt_store(q, val);
    else *q = val;
  };
  if (post_tw_m > 0 && E == 16 && T >= 4 && post_tw_m == Mr * M) {
    // exp(+2 pi i qr b / (Mr M)), b = t + T i, factors into exp(2 pi i qr t / (Mr M)) (one
    // table read per lane) and exp(2 pi i qr i / (16 Mr)): 16 values per row, fetched by the
    // row's T lanes into its exchange slot instead of 16 scattered reads per lane
    float2 *slot = lds + rl * (E * (T + 1));
    const int bstep = tw_n / (16 * Mr);
    for (int i = t; i < 16; i += T) slot[i] = tw[((qr * i) & (16 * Mr - 1)) * bstep];
    wave_sync();
    float2 wa = tw[((qr * t) & (post_tw_m - 1)) * (tw_n / post_tw_m)];
    wa.y = -wa.y;
    if (valid) {
#pragma unroll
      for (int i = 0; i < E; ++i) {
        float2 wb = slot[i];
        wb.y = -wb.y;
        put(dp + T * i, cmul(v[i], cmul(wa, wb)));
      }
    }
  } else if (post_tw_m > 0) {
    const int step = tw_n / post_tw_m;
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const int e = static_cast<int>((static_cast<long long>(qr) * (t + T * i)) & (post_tw_m - 1));
      float2 w = tw[e * step];
      w.y = -w.y;
      put(dp + T * i, cmul(v[i], w));
    }
  } else {
#pragma unroll
    for (int i = 0; i < E; ++i) put(dp + T * i, v[i]);
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
                      float2 *__restrict__ uc, int uc_half, int post_tw_m,
                      const float *__restrict__ phi_rows,
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
    // uc_half: the input was real, so rows Mr/2+1.. are conjugates of rows Mr/2-1..1 and
    // only rows 0..Mr/2 are stored, compactly
    const int rows_kept = uc_half ? Mr / 2 + 1 : Mr;
    float2 *ucp = uc + static_cast<size_t>(node) * rows_kept * Mc;
    for (int t = threadIdx.x; t < rows_kept * TC; t += blockDim.x) {
      int i = t / TC, c = t % TC;
      float2 v = lds[t];
      if (post_tw_m > 0) {
        int e = static_cast<int>((static_cast<long long>(i) * (c0 + c)) % post_tw_m);
        v = cmul(v, twiddle<false>(tw, tw_n, e, post_tw_m));
      }
      ucp[static_cast<size_t>(i) * Mc + c0 + c] = v;
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
// 1-D cascade, row half of everything that follows a modulus: forward row FFT of the
// column spectra src [nodes][Sr][Sc] (never written back), then for every child c of the
// list: product with the real table c.filt [Sr][Sc], sum over the 2^c.lg_fold blocks of the
// row (second digit of the four-step order), inverse row FFT of Sc >> c.lg_fold points, the
// four-step twiddle exp(+2 pi i k1 b / c.post_tw_m), store to c.dst [nodes][Sr][Sc >> lg_fold].
// The children are the wavelets of all coarser octaves and / or the lowpass, so the signal
// is read once for all of them.  RB rows per workgroup, all transforms through lds_fft.
__global__ __launch_bounds__(256) void k_rows1d(const float2 *__restrict__ src, int Sr, int Sc,
                                                int RB, Rows1dArgs a,
                                                const float2 *__restrict__ tw, int tw_n) {
  extern __shared__ float2 lds[];
  float2 *spec = lds, *low = lds + RB * Sc;
  // the Sc-point twiddle table in LDS: the transforms' strided reads of the global table
  // (one cache line per twiddle) would otherwise sit on every butterfly's critical path
  float2 *twl = low + RB * Sc;
  for (int j = threadIdx.x; j < Sc; j += blockDim.x) twl[j] = tw[j * (tw_n / Sc)];
  const int lgSc = ilog2(Sc);
  const long row0 = static_cast<long>(blockIdx.x) * RB;
  const float2 *sp = src + static_cast<size_t>(row0) * Sc;
  for (int t = threadIdx.x; t < RB * Sc; t += blockDim.x) {
    const int row = t >> lgSc, c = t & (Sc - 1);
    spec[row * Sc + bitrev(c, lgSc)] = sp[t];
  }
  lds_fft<false, false>(spec, lgSc, RB, Sc, 1, twl, Sc);
  const int k1_0 = static_cast<int>(row0 % Sr);  // RB divides Sr: the rows share one node
  for (int ci = 0; ci < a.n; ++ci) {
    const Rows1dChild &ch = a.c[ci];
    const int lgm = lgSc - ch.lg_fold, m = 1 << lgm;
    // products of the whole rows (every thread busy, filter reads contiguous), each block of
    // m columns stored bit-reversed within itself; the blocks are then added pairwise, which
    // leaves the folded row, bit-reversed, in the first m columns of its Sc-column slot
    const float *fp = ch.filt + static_cast<size_t>(k1_0) * Sc;
    for (int t = threadIdx.x; t < RB * Sc; t += blockDim.x) {
      const int c = t & (Sc - 1);
      const float2 v = spec[t];
      const float f = fp[t];
      low[(t - c) + (c & ~(m - 1)) + bitrev(c & (m - 1), lgm)] = make_float2(v.x * f, v.y * f);
    }
    for (int half = Sc >> 1; half >= m; half >>= 1) {
      __syncthreads();
      const int lgh = ilog2(half);
      for (int t = threadIdx.x; t < RB * half; t += blockDim.x) {
        const int row = t >> lgh, i = t & (half - 1);
        float2 *q = low + row * Sc + i;
        const float2 u = q[half];
        q[0].x += u.x;
        q[0].y += u.y;
      }
    }
    lds_fft<true, false>(low, lgm, RB, Sc, 1, twl, Sc);
    long drow0 = row0;
    if (ch.K > 0) {
      const long node = row0 / Sr;
      const int g = static_cast<int>(node % ch.cm.G);
      drow0 = ((node / ch.cm.G) * ch.K + (ch.chan_tab != nullptr ? ch.chan_tab[g] : chan_of(ch.cm, g))) * Sr + k1_0;
    }
    float2 *dp = ch.dst + static_cast<size_t>(drow0) * m;
    for (int t = threadIdx.x; t < RB * m; t += blockDim.x) {
      const int row = t >> lgm, b = t & (m - 1);
      float2 v = low[row * Sc + b];
      if (ch.post_tw_m > 0) {
        const int e = static_cast<int>((static_cast<long long>(k1_0 + row) * b) % ch.post_tw_m);
        v = cmul(v, twiddle<true>(tw, tw_n, e, ch.post_tw_m));
      }
      dp[t] = v;
    }
    __syncthreads();  // `low` is reused by the next child
  }
}

// ------------------------------------------------------------------------------------
// k_rows1d with the transforms in registers, for rows of Sc = 16 T points (T lanes per row,
// 256 / T rows per workgroup, wave-level synchronisation only).  The forward transform
// leaves lane t with X[t + T i]; a child's fold by 2^d halves that register array
// min(d, 4) times, the remaining halvings add lanes t and t ^ s; the folded row is parked
// in the row's LDS slot in natural order, picked up by the m / 16 lanes that share its
// inverse transform (one lane below 16 points), transformed and stored.
// Four-step twiddle of output b = t + T2 i of row k1: exp(+2 pi i k1 b / M), M = Sr m (so
// k1 b < M).  With m = 16 T2 it factors into exp(2 pi i k1 t / M) (one table read per lane)
// times exp(2 pi i k1 i / (16 Sr)), which depends on the row only: `rowtw`, read once per row
// and kept behind the row's LDS slot.
// (ROWTW = false: rows too short for that to pay; every twiddle is read from the table.)
template <int E2, int T2, bool ROWTW>
__device__ __forceinline__ void rows1d_child_inv(float2 *slot, int t, int tw_step,
                                                 const float2 *twl, float2 *dp, int k1,
                                                 int post_tw_m, const float2 *__restrict__ tw,
                                                 int tw_n, bool store, const float2 *rowtw) {
  if (t >= T2) return;
  float2 v[E2], wt[E2];
#pragma unroll
  for (int i = 0; i < E2; ++i) v[i] = slot[t + T2 * i];
#pragma unroll
  for (int k = 0; k < E2; ++k) wt[k] = twl[t * k * tw_step];
  wave_sync();  // the slot becomes the exchange area
  fft_core<E2, T2, true, true>(v, t, slot, T2 + 1, 1, wt);
  if (!store) return;
  const int step = post_tw_m > 0 ? tw_n / post_tw_m : 0;
  float2 wl = make_float2(1.f, 0.f);
  if (ROWTW && E2 == 16 && post_tw_m > 0) {
    wl = tw[k1 * t * step];
    wl.y = -wl.y;
  }
#pragma unroll
  for (int i = 0; i < E2; ++i) {
    const int b = t + T2 * i;
    float2 o = v[i];
    if (post_tw_m > 0) {
      float2 w;
      if (ROWTW && E2 == 16) {
        w = cmul(wl, rowtw[i]);
      } else {
        w = tw[k1 * b * step];
        w.y = -w.y;
      }
      o = cmul(o, w);
    }
    dp[b] = o;
  }
}

// (E = 16 points per lane; rows of 4 and 8 points: E = row length, T = 1.)
// HALF: src holds rows 0 .. Sr/2 of every node only ([nodes][Sr/2+1][Sc], as the column pass
// writes them for real columns).  Row Sr - k1 of the twiddled column spectra is the conjugate
// of row k1 times exp(-2 pi i b / Sc), so its row transform is the stored row's, conjugated and
// read backwards: X'[k2] = conj(X[Sc - 1 - k2]).  A row group therefore serves two rows of the
// node from one load and one forward transform (rows 0 and Sr/2 have no partner).
template <int E, int T, bool HALF>
__global__ __launch_bounds__(256, 4) void k_rows1d_reg(const float2 *__restrict__ src, long rows,
                                                    int Sr, Rows1dArgs a,
                                                    const float2 *__restrict__ tw, int tw_n) {
  static_assert(E == 16 || T == 1, "short rows are held by one lane");
  constexpr bool ROWTW = T >= 4;
  constexpr int Sc = E * T, RPB = 256 / T;
  // (an odd number of elements per row slot: the rows of a quarter wave start in different banks)
  constexpr int XS = ((T == 1 ? E : E * (T + 1)) + (ROWTW ? 16 : 0)) | 1;
  constexpr int lgSc = (E == 4 ? 2 : E == 8 ? 3 : 4) + (T == 1 ? 0 : T == 2 ? 1 : T == 4 ? 2 : T == 8 ? 3 : 4);
  extern __shared__ float2 lds[];
  float2 *twl = lds;
  for (int j = threadIdx.x; j < Sc; j += blockDim.x) twl[j] = tw[j * (tw_n / Sc)];
  __syncthreads();
  const int rl = threadIdx.x / T, t = threadIdx.x % T;
  const long row_raw = static_cast<long>(blockIdx.x) * RPB + rl;
  const bool valid = row_raw < rows;
  const long row = valid ? row_raw : rows - 1;  // idle groups redo the last row, unstored
  const int SrS = HALF ? Sr / 2 + 1 : Sr;        // stored rows of a node
  const long node = row / SrS;
  int k1 = static_cast<int>(row - node * SrS);
  bool live = valid;
  float2 *slot = lds + Sc + rl * XS;
  float2 v[E];
  {
    const float2 *sp = src + static_cast<size_t>(row) * Sc + t;
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = a.spec_out != nullptr ? sp[T * i] : nt_load(sp + T * i);
    float2 wt[E];
#pragma unroll
    for (int k = 0; k < E; ++k) wt[k] = twl[t * k];
    fft_core<E, T, false, true>(v, t, slot, T + 1, 1, wt);
    if (!HALF && a.spec_out != nullptr && valid) {
      float2 *op = a.spec_out + static_cast<size_t>(row) * Sc + t;
#pragma unroll
      for (int i = 0; i < E; ++i) op[T * i] = v[i];
    }
  }
  float2 *rowtw = ROWTW ? slot + XS - 16 : slot;
#pragma unroll 1
  for (int pass = 0; pass < (HALF ? 2 : 1); ++pass) {
  if (HALF && pass == 1) {
    // the partner row Sr - k1: spectrum conj(X[Sc - 1 - k2]); element t + T i comes from lane
    // T - 1 - t of the row group, register E - 1 - i
    live = live && k1 != 0 && 2 * k1 != Sr;
    k1 = (Sr - k1) & (Sr - 1);  // (rows without a partner: unstored)
    float2 u[E];
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const float2 x = v[E - 1 - i];
      if (T > 1) {
        const int from = (static_cast<int>(threadIdx.x) & 63 & ~(T - 1)) | (T - 1 - t);
        u[i] = make_float2(__shfl(x.x, from), -__shfl(x.y, from));
      } else {
        u[i] = make_float2(x.x, -x.y);
      }
    }
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = u[i];
    wave_sync();  // the first pass's reads of the row's twiddles are done
  }
  // exp(+2 pi i k1 i / (16 Sr)): the row's share of every child's four-step twiddle
  if (ROWTW) {
    // lane t fetches entries t, t + T, ... (T >= 4 lanes share the 16 entries)
    const int rstep = tw_n / (16 * Sr);
    for (int i = t; i < 16; i += T) {
      float2 w = rstep > 0 ? tw[k1 * i * rstep] : make_float2(1.f, 0.f);
      w.y = -w.y;
      rowtw[i] = w;
    }
  }
  for (int ci = 0; ci < a.n; ++ci) {
    const Rows1dChild &ch = a.c[ci];
    const int lgm = lgSc - ch.lg_fold, m = 1 << lgm;
    const float *fp = ch.filt + static_cast<size_t>(k1) * Sc + t;
    float2 p[E];
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const float f = fp[T * i];
      p[i] = make_float2(v[i].x * f, v[i].y * f);
    }
    int dd = ch.lg_fold;
#pragma unroll
    for (int h = E / 2; h >= 1; h >>= 1) {
      if (dd > 0) {
#pragma unroll
        for (int i = 0; i < h; ++i) {
          p[i].x += p[i + h].x;
          p[i].y += p[i + h].y;
        }
        --dd;
      }
    }
#pragma unroll
    for (int s = T / 2; s >= 1; s >>= 1) {
      if (dd > 0) {
        p[0].x += __shfl_xor(p[0].x, s);
        p[0].y += __shfl_xor(p[0].y, s);
        --dd;
      }
    }
#pragma unroll
    for (int i = 0; i < E; ++i)
      if (t + T * i < m) slot[t + T * i] = p[i];
    wave_sync();
    long drow = node * Sr + k1;
    if (ch.K > 0) {
      const int g = static_cast<int>(node % ch.cm.G);
      drow = ((node / ch.cm.G) * ch.K + (ch.chan_tab != nullptr ? ch.chan_tab[g] : chan_of(ch.cm, g))) * Sr + k1;
    }
    float2 *dp = ch.dst + static_cast<size_t>(drow) * m;
    const int tws = Sc >> lgm;
    switch (lgm) {
      case 0:
        if (t == 0 && live) dp[0] = slot[0];
        break;
      case 1: rows1d_child_inv<2, 1, ROWTW>(slot, t, tws, twl, dp, k1, ch.post_tw_m, tw, tw_n, live, rowtw); break;
      case 2: rows1d_child_inv<4, 1, ROWTW>(slot, t, tws, twl, dp, k1, ch.post_tw_m, tw, tw_n, live, rowtw); break;
      case 3: if (E >= 8) rows1d_child_inv<(E >= 8 ? 8 : 4), 1, ROWTW>(slot, t, tws, twl, dp, k1, ch.post_tw_m, tw, tw_n, live, rowtw); break;
      case 4: if (E >= 16) rows1d_child_inv<(E >= 16 ? 16 : 4), 1, ROWTW>(slot, t, tws, twl, dp, k1, ch.post_tw_m, tw, tw_n, live, rowtw); break;
      case 5: if (T >= 2) rows1d_child_inv<16, (T >= 2 ? 2 : 1), ROWTW>(slot, t, tws, twl, dp, k1, ch.post_tw_m, tw, tw_n, live, rowtw); break;
      case 6: if (T >= 4) rows1d_child_inv<16, (T >= 4 ? 4 : 1), ROWTW>(slot, t, tws, twl, dp, k1, ch.post_tw_m, tw, tw_n, live, rowtw); break;
      case 7: if (T >= 8) rows1d_child_inv<16, (T >= 8 ? 8 : 1), ROWTW>(slot, t, tws, twl, dp, k1, ch.post_tw_m, tw, tw_n, live, rowtw); break;
      case 8: if (T >= 16) rows1d_child_inv<16, (T >= 16 ? 16 : 1), ROWTW>(slot, t, tws, twl, dp, k1, ch.post_tw_m, tw, tw_n, live, rowtw); break;
      default: break;
    }
    wave_sync();  // the slot is reused by the next child
  }
  }  // pass
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


// ------------------------------------------------------------------------------------
// Column pass with register-resident transforms (column length MR = 16 * T, compile
// time).  Same contract as k_col<0> / k_col<1>; T threads share one column, TC columns
// per workgroup (blockDim = T * TC, thread = c + TC * t so that global accesses run
// along rows).  LM_R = compile-time lowpass length (8 or 32: the fold is done in registers
// and the small inverse transform by 1 or 2 lanes per column) or 0 = any length (generic
// tail through lds_fft).
// (blk: the workgroup's number among those that work on this array of nodes)
template <int MR, int MODE, int LM_R>
__device__ __forceinline__ void col_fast_body(unsigned blk, const void *__restrict__ src_v, int Mc, int TC,
                                              float2 *__restrict__ uc, int uc_half, int post_tw_m,
                                              const float *__restrict__ phi_rows, int m_r,
                                              float *__restrict__ w_out,
                                              const float2 *__restrict__ tw, int tw_n) {
  constexpr int E = MR > 256 ? 32 : 16, T = MR / E;
  extern __shared__ float2 lds[];
  const int KS = T * TC + 16;
  const int c = threadIdx.x % TC, t = threadIdx.x / TC;
  const int tiles = Mc / TC;
  const int node = blk / tiles;
  const int c0 = (blk % tiles) * TC;
  const size_t plane = static_cast<size_t>(node) * MR * Mc;
  const int off0 = t * Mc + c0 + c;  // offset of this thread's first element in the plane
  const int step = T * Mc;
  float2 wt[E];
  load_twiddles<E, T>(wt, t, tw, tw_n);
  float2 v[E];
  if (MODE == 0) {
    const float *sp = static_cast<const float *>(src_v) + plane + off0;
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = make_float2(sp[i * step], 0.f);
  } else {
    const float2 *sp = static_cast<const float2 *>(src_v) + plane + off0;
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = nt_load(sp + i * step);
    fft_core<E, T, true>(v, t, lds + c, KS, TC, wt);
#pragma unroll
    for (int i = 0; i < E; ++i)
      v[i] = make_float2(__builtin_amdgcn_sqrtf(v[i].x * v[i].x + v[i].y * v[i].y), 0.f);
  }
  fft_core<E, T, false>(v, t, lds + c, KS, TC, wt);
  if (uc != nullptr) {
    if (uc_half && post_tw_m == 0) {
      // real input: rows above MR/2 are conjugates of stored ones; keep rows 0..MR/2 compactly
      float2 *up = uc + static_cast<size_t>(node) * (MR / 2 + 1) * Mc + off0;
#pragma unroll
      for (int i = 0; i < E; ++i)
        if (t + T * i <= MR / 2) nt_store(up + i * step, v[i]);
    } else if (post_tw_m > 0 && E == 16 && post_tw_m == MR * Mc) {
      // four-step forward: times exp(-2 pi i k_r b / M), k_r = t + T i, b the column,
      // M = MR Mc = 16 T Mc.  It factors into exp(-2 pi i t b / M) (one table read per
      // thread) and exp(-2 pi i i b / (16 Mc)), which the workgroup's threads fetch once for
      // its TC columns into LDS (16 TC entries) instead of 16 scattered reads per thread.
      __syncthreads();
      const int bmask = 16 * Mc - 1, bstep = tw_n / (16 * Mc);
      for (int idx = threadIdx.x; idx < 16 * TC; idx += blockDim.x) {
        const int i = idx / TC, cc = idx - i * TC;
        lds[idx] = tw[((i * (c0 + cc)) & bmask) * bstep];
      }
      __syncthreads();
      // (uc_half: the column was real, so row MR - k of the twiddled result is the conjugate of
      // row k times exp(-2 pi i b / Mc); rows 0 .. MR/2 are kept, compactly, and the row pass
      // derives the others from them)
      float2 *up = uc_half ? uc + static_cast<size_t>(node) * (MR / 2 + 1) * Mc + off0 : uc + plane + off0;
      const float2 wa = tw[((t * (c0 + c)) & (post_tw_m - 1)) * (tw_n / post_tw_m)];
#pragma unroll
      for (int i = 0; i < E; ++i)
        if (!uc_half || t + T * i <= MR / 2) up[i * step] = cmul(v[i], cmul(wa, lds[i * TC + c]));
    } else if (post_tw_m > 0) {
      // four-step forward: times exp(-2 pi i k_r c / post_tw_m), k_r = t + T i, c the column
      float2 *up = uc + plane + off0;
      const int tstep = tw_n / post_tw_m;
#pragma unroll
      for (int i = 0; i < E; ++i) {
        const int e = static_cast<int>((static_cast<long long>(t + T * i) * (c0 + c)) & (post_tw_m - 1));
        up[i * step] = cmul(v[i], tw[e * tstep]);
      }
    } else {
      float2 *up = uc + plane + off0;
#pragma unroll
      for (int i = 0; i < E; ++i) up[i * step] = v[i];
    }
  }
  if (w_out == nullptr) return;
  float *wp = w_out + static_cast<size_t>(node) * m_r * Mc + c0;
  if (LM_R > 0) {
    // fold in registers: row t + T*i lands on lowpass frequency t + T*(i mod JT)
    constexpr int JT = LM_R / T > 0 ? LM_R / T : 1;
    float2 fm[JT];
#pragma unroll
    for (int j = 0; j < JT; ++j) fm[j] = make_float2(0.f, 0.f);
    const float *ph = phi_rows + t;
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const float f = ph[T * i];
      fm[i % JT].x += v[i].x * f;
      fm[i % JT].y += v[i].y * f;
    }
#pragma unroll
    for (int j = 0; j < JT; ++j) lds[(t + T * j) * TC + c] = fm[j];
    __syncthreads();
    if (LM_R == 32 && T >= 4) {
      // 4 lanes per column, 8 points each
      if (static_cast<int>(threadIdx.x) < 4 * TC) {
        const int tp = threadIdx.x & 3, cc = threadIdx.x >> 2;
        float2 y[8], w2[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = lds[(tp + 4 * i) * TC + cc];
        load_twiddles<8, 4>(w2, tp, tw, tw_n);
        fft_core<8, 4, true, true>(y, tp, lds + LM_R * TC + cc * 48, 5, 1, w2);
#pragma unroll
        for (int i = 0; i < 8; ++i) wp[(tp + 4 * i) * Mc + cc] = y[i].x;
      }
    } else if (LM_R == 32) {
      if (static_cast<int>(threadIdx.x) < 2 * TC) {
        const int tp = threadIdx.x & 1, cc = threadIdx.x >> 1;
        float2 y[16], w2[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) y[i] = lds[(tp + 2 * i) * TC + cc];
        load_twiddles<16, 2>(w2, tp, tw, tw_n);
        fft_core<16, 2, true, true>(y, tp, lds + LM_R * TC + cc * 48, 3, 1, w2);
#pragma unroll
        for (int i = 0; i < 16; ++i) wp[(tp + 2 * i) * Mc + cc] = y[i].x;
      }
    } else {
      if (static_cast<int>(threadIdx.x) < TC) {
        const int cc = threadIdx.x;
        float2 y[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = lds[i * TC + cc];
        DftRegs<8, true>::run(y);
#pragma unroll
        for (int i = 0; i < 8; ++i) wp[i * Mc + cc] = y[i].x;
      }
    }
  } else {
    // spectrum * phi in natural row order, then fold and a small inverse transform
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const int r = t + T * i;
      const float f = phi_rows[r];
      lds[r * TC + c] = make_float2(v[i].x * f, v[i].y * f);
    }
    __syncthreads();
    float2 *low = lds + E * KS;
    const int log2m = ilog2(m_r);
    const int nf = MR / m_r;
    for (int idx = threadIdx.x; idx < m_r * TC; idx += blockDim.x) {
      int m = idx / TC, cc = idx % TC;
      float2 acc = make_float2(0.f, 0.f);
      for (int a = 0; a < nf; ++a) acc = cadd(acc, lds[(m + a * m_r) * TC + cc]);
      low[bitrev(m, log2m) * TC + cc] = acc;
    }
    lds_fft<true, true>(low, log2m, TC, 1, TC, tw, tw_n);
    for (int idx = threadIdx.x; idx < m_r * TC; idx += blockDim.x) {
      int m = idx / TC, cc = idx % TC;
      wp[static_cast<size_t>(m) * Mc + cc] = low[idx].x;
    }
  }
}

template <int MR, int MODE, int LM_R>
__global__ __launch_bounds__(256) void k_col_fast(const void *__restrict__ src_v, int Mc, int TC,
                                                  float2 *__restrict__ uc, int uc_half,
                                                  int post_tw_m,
                                                  const float *__restrict__ phi_rows, int m_r,
                                                  float *__restrict__ w_out,
                                                  const float2 *__restrict__ tw, int tw_n) {
  col_fast_body<MR, MODE, LM_R>(blockIdx.x, src_v, Mc, TC, uc, uc_half, post_tw_m, phi_rows, m_r, w_out, tw,
                                tw_n);
}

// Mode 1 (inverse transform, modulus, forward transform, four-step twiddle: the 1-D cascade's
// column pass) over several arrays of nodes that differ in their number of columns, in one
// launch: workgroups first[s] .. first[s + 1] - 1 take segment s.
struct ColSegsDev {
  int n;
  unsigned first[kColMaxSegs];
  int Mc[kColMaxSegs];
  long long src_off[kColMaxSegs], uc_off[kColMaxSegs];  // in elements from the common bases
  long long nodes[kColMaxSegs];                          // (read by k_col_pair_segs only)
};
template <int MR>
__global__ __launch_bounds__(256) void k_col_fast_segs(const float2 *__restrict__ src,
                                                       float2 *__restrict__ uc, ColSegsDev sg, int TC,
                                                       int uc_half, const float2 *__restrict__ tw, int tw_n) {
  int s = 0;
#pragma unroll
  for (int i = 1; i < kColMaxSegs; ++i)
    if (i < sg.n && blockIdx.x >= sg.first[i]) s = i;
  s = __builtin_amdgcn_readfirstlane(s);
  const int Mc = sg.Mc[s];
  col_fast_body<MR, 1, 0>(blockIdx.x - sg.first[s], src + sg.src_off[s], Mc, TC, uc + sg.uc_off[s], uc_half,
                          MR * Mc, nullptr, 0, nullptr, tw, tw_n);
}

// The same pass for half spectra with TWO adjacent columns per thread (16-byte loads and
// stores): both are inverse-transformed, and since their moduli are real they go through ONE
// forward transform as z = |a| + i |b|; the two spectra are taken apart again with the help of
// row MR - k (through LDS): A[k] = (Z[k] + conj(Z[-k])) / 2, B[k] = -i (Z[k] - conj(Z[-k])) / 2.
// Rows 0 .. MR/2 are written, with the four-step twiddle.  A tile is TCp = min(16, Mc / 2)
// column pairs of one node, held by 16 TCp threads; narrow nodes (Mc < 32) are one tile each and
// 16 / TCp of them share a workgroup, each with an LDS area of its own.
template <int MR>
__global__ __launch_bounds__(256, 4) void k_col_pair_segs(const float2 *__restrict__ src,
                                                       float2 *__restrict__ uc, ColSegsDev sg,
                                                       const float2 *__restrict__ tw, int tw_n) {
  constexpr int E = 16, T = MR / E;
  static_assert(T == 16, "256 threads = 16 row lanes x up to 16 column pairs");
  extern __shared__ float2 lds[];
  int sgi = 0;
#pragma unroll
  for (int i = 1; i < kColMaxSegs; ++i)
    if (i < sg.n && blockIdx.x >= sg.first[i]) sgi = i;
  sgi = __builtin_amdgcn_readfirstlane(sgi);
  const int Mc = sg.Mc[sgi];
  const unsigned blk = blockIdx.x - sg.first[sgi];
  const int TCp = Mc >= 32 ? 16 : Mc / 2;  // column pairs per tile
  const int per = T * TCp;                 // threads per tile
  const int slot = threadIdx.x / per, l = threadIdx.x % per;
  const int cp = l % TCp, t = l / TCp;
  long node;
  int c0;
  bool valid = true;
  if (Mc >= 32) {
    const int tiles = Mc / 32;
    node = blk / tiles;
    c0 = (blk % tiles) * 32;
  } else {
    const long node_raw = static_cast<long>(blk) * (256 / per) + slot;
    valid = node_raw < sg.nodes[sgi];
    node = valid ? node_raw : sg.nodes[sgi] - 1;  // idle tiles redo the last node, unstored
    c0 = 0;
  }
  const int KS = per + 16;
  // a tile's LDS area: the transforms' exchange (16 KS elements), later Z by rows (MR TCp) and the
  // twiddle factors (32 TCp)
  const int SA = 288 * TCp > 256 * TCp + 256 ? 288 * TCp : 256 * TCp + 256;
  float2 *area = lds + slot * SA;
  // the transforms' twiddles exp(-2 pi i t k / MR) as a table in LDS, [k T + t], behind the tiles'
  // areas (three transforms would otherwise hold sixteen of them in registers throughout)
  float2 *wtab = lds + (256 / per) * SA;
  for (int idx = threadIdx.x; idx < MR; idx += 256) wtab[idx] = tw[(idx / T) * (idx % T) * (tw_n / MR)];
  __syncthreads();
  const float2 *sp = src + sg.src_off[sgi] + static_cast<size_t>(node) * MR * Mc + t * Mc + c0 + 2 * cp;
  const int step = T * Mc;
  float2 va[E], vb[E];
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const float4 x = nt_load4(sp + i * step);
    va[i] = make_float2(x.x, x.y);
    vb[i] = make_float2(x.z, x.w);
  }
  fft_core_tab<E, T, true>(va, t, area + cp, KS, TCp, wtab + t, T);
  fft_core_tab<E, T, true>(vb, t, area + cp, KS, TCp, wtab + t, T);
#pragma unroll
  for (int i = 0; i < E; ++i)
    va[i] = make_float2(__builtin_amdgcn_sqrtf(va[i].x * va[i].x + va[i].y * va[i].y),
                        __builtin_amdgcn_sqrtf(vb[i].x * vb[i].x + vb[i].y * vb[i].y));
  fft_core_tab<E, T, false>(va, t, area + cp, KS, TCp, wtab + t, T);  // ends with a barrier: the area is free
  // Z by rows for the partners, and behind it the column-dependent factors of the twiddle
  // exp(-2 pi i i b / (16 Mc)), i < 16, for the tile's 2 TCp columns
  float2 *zt = area, *ctw = area + MR * TCp;
#pragma unroll
  for (int i = 0; i < E; ++i) zt[(t + T * i) * TCp + cp] = va[i];
  const int M = MR * Mc;
  const int bmask = 16 * Mc - 1, bstep = tw_n / (16 * Mc);
  for (int idx = l; idx < 16 * 2 * TCp; idx += per) {
    const int i = idx / (2 * TCp), cc = idx - i * (2 * TCp);
    ctw[idx] = tw[((i * (c0 + cc)) & bmask) * bstep];
  }
  __syncthreads();
  if (!valid) return;
  const int b0 = c0 + 2 * cp;
  const int tstep = tw_n / M;
  const float2 wa0 = tw[((t * b0) & (M - 1)) * tstep], wa1 = tw[((t * (b0 + 1)) & (M - 1)) * tstep];
  float2 *up = uc + sg.uc_off[sgi] + static_cast<size_t>(node) * (MR / 2 + 1) * Mc + t * Mc + b0;
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const int r = t + T * i;
    if (r > MR / 2) continue;
    const float2 zk = va[i], zn = zt[((MR - r) & (MR - 1)) * TCp + cp];
    const float2 a = make_float2(0.5f * (zk.x + zn.x), 0.5f * (zk.y - zn.y));
    const float2 b = make_float2(0.5f * (zk.y + zn.y), 0.5f * (zn.x - zk.x));
    const float2 oa = cmul(a, cmul(wa0, ctw[i * (2 * TCp) + 2 * cp]));
    const float2 ob = cmul(b, cmul(wa1, ctw[i * (2 * TCp) + 2 * cp + 1]));
    nt_store4(up + i * step, make_float4(oa.x, oa.y, ob.x, ob.y));
  }
}

hipError_t launch_col_segs_impl(const float2 *src, float2 *uc, int Mr, const ColSeg *segs, int n, bool uc_half,
                                const float2 *tw, int tw_n, hipStream_t st) {
  if (Mr != 256 || n < 1 || n > kColMaxSegs || tw_n % Mr != 0) return hipErrorInvalidValue;
  constexpr int MR = 256, E = 16, T = MR / E, TC = 16;
  ColSegsDev sg{};
  sg.n = n;
  long blocks = 0;
  double pts = 0.0, cols = 0.0;
  bool pairs = uc_half;
  for (int i = 0; i < n; ++i)
    pairs = pairs && segs[i].Mc >= 4 && (segs[i].Mc & (segs[i].Mc - 1)) == 0 && segs[i].src_off % 2 == 0 &&
            segs[i].uc_off % 2 == 0;
  if (pairs) {
    // two adjacent columns per thread; narrow nodes share a workgroup
    size_t lds_p = 0;
    for (int i = 0; i < n; ++i) {
      const long long m = static_cast<long long>(MR) * segs[i].Mc;
      if (segs[i].nodes < 1 || tw_n % m != 0) return hipErrorInvalidValue;
      const int TCp = segs[i].Mc >= 32 ? 16 : segs[i].Mc / 2, NS = 16 / TCp;
      const size_t SA = static_cast<size_t>(std::max(288 * TCp, 256 * TCp + 256));
      lds_p = std::max(lds_p, (NS * SA + MR) * sizeof(float2));
      sg.first[i] = static_cast<unsigned>(blocks);
      sg.Mc[i] = segs[i].Mc;
      sg.src_off[i] = segs[i].src_off;
      sg.uc_off[i] = segs[i].uc_off;
      sg.nodes[i] = segs[i].nodes;
      blocks += segs[i].Mc >= 32 ? segs[i].nodes * (segs[i].Mc / 32) : (segs[i].nodes + NS - 1) / NS;
      if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
      pts += static_cast<double>(segs[i].nodes) * m;
      cols += static_cast<double>(segs[i].nodes) * segs[i].Mc;
    }
    Observe ob("k_col_pair_segs<256>", pts * 12, cols * 1.5 * fft_flops(MR) + 4.0 * pts, st);
    hipLaunchKernelGGL((k_col_pair_segs<MR>), dim3(static_cast<unsigned>(blocks)), dim3(256), lds_p, st, src, uc, sg,
                       tw, tw_n);
    return hipGetLastError();
  }
  for (int i = 0; i < n; ++i) {
    const long long m = static_cast<long long>(MR) * segs[i].Mc;
    if (segs[i].nodes < 1 || segs[i].Mc < TC || segs[i].Mc % TC != 0 || tw_n % m != 0 || (m & (m - 1)) != 0)
      return hipErrorInvalidValue;
    sg.first[i] = static_cast<unsigned>(blocks);
    sg.Mc[i] = segs[i].Mc;
    sg.src_off[i] = segs[i].src_off;
    sg.uc_off[i] = segs[i].uc_off;
    blocks += segs[i].nodes * (segs[i].Mc / TC);
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    pts += static_cast<double>(segs[i].nodes) * m;
    cols += static_cast<double>(segs[i].nodes) * segs[i].Mc;
  }
  const size_t lds = static_cast<size_t>(E) * (T * TC + 16) * sizeof(float2);
  Observe ob("k_col_fast_segs<256>", pts * (uc_half ? 12 : 16), cols * 2 * fft_flops(MR) + 4.0 * pts, st);
  hipLaunchKernelGGL((k_col_fast_segs<MR>), dim3(static_cast<unsigned>(blocks)), dim3(T * TC), lds, st, src, uc, sg,
                     TC, static_cast<int>(uc_half), tw, tw_n);
  return hipGetLastError();
}

// Mode 2 (the last step of the 1-D cascade: inverse column transform of the lowpassed rows,
// real part to the output channel) with the transform in registers: nodes of MR = 256 rows
// and TC <= 16 columns, 16 TC threads per node (thread = column c, rows t + 16 i), 16 / TC
// nodes per workgroup.  src [nodes][MR][TC] complex; out[(p K + channel(g)) MR TC + row TC + c].
template <int MR>
// Nodes from `tail_from` on are channel 0 of signal node - tail_from (the order-0 coefficient,
// whose rows are stored behind the others').
__global__ __launch_bounds__(256) void k_col_out(const float2 *__restrict__ src, long nodes, int TC,
                                                 float *__restrict__ out, ChanMap cm, int K, long tail_from,
                                                 const float2 *__restrict__ tw, int tw_n) {
  constexpr int E = 16, T = MR / E;
  extern __shared__ float2 lds[];
  const int per = T * TC;                      // threads per node
  const int slot = threadIdx.x / per, l = threadIdx.x % per;
  const int c = l % TC, t = l / TC;
  const int KS = per + 16;
  const long node_raw = static_cast<long>(blockIdx.x) * (256 / per) + slot;
  const bool valid = node_raw < nodes;
  const long node = valid ? node_raw : nodes - 1;  // idle slots redo the last node, unstored
  float2 wt[E], v[E];
  load_twiddles<E, T>(wt, t, tw, tw_n);
  const float2 *sp = src + static_cast<size_t>(node) * MR * TC + t * TC + c;
#pragma unroll
  for (int i = 0; i < E; ++i) v[i] = nt_load(sp + i * per);
  fft_core<E, T, true>(v, t, lds + slot * E * KS + c, KS, TC, wt);
  if (!valid) return;
  long p = node / cm.G;
  int chan = chan_of(cm, static_cast<int>(node - p * cm.G));
  if (node >= tail_from) {
    p = node - tail_from;
    chan = 0;
  }
  float *op = out + (static_cast<size_t>(p) * K + chan) * MR * TC + t * TC + c;
#pragma unroll
  for (int i = 0; i < E; ++i) op[i * per] = v[i].x;
}

hipError_t launch_col_out(const float2 *src, long nodes, int Mc, float *out, ChanMap cm, int K,
                          const float2 *tw, int tw_n, hipStream_t st, long tail_from = -1) {
  if (tail_from < 0) tail_from = nodes;
  constexpr int MR = 256, E = 16, T = MR / E;
  const int per = T * Mc;
  const long blocks = (nodes + 256 / per - 1) / (256 / per);
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const size_t lds = static_cast<size_t>(256 / per) * E * (per + 16) * sizeof(float2);
  const double pts = static_cast<double>(nodes) * MR * Mc;
  Observe ob("k_col_out<256>", pts * 12, static_cast<double>(nodes) * Mc * fft_flops(MR), st);
  hipLaunchKernelGGL((k_col_out<MR>), dim3(static_cast<unsigned>(blocks)), dim3(256), lds, st, src, nodes, Mc, out,
                     cm, K, tail_from, tw, tw_n);
  return hipGetLastError();
}

// Mode 1 for nodes without children (no spectrum output, lowpass length 32) with TWO adjacent
// columns per thread: 16-byte loads, both columns inverse-transformed, and their two real
// moduli sent through the forward transform and the whole (linear, real-filter) lowpass tail as
// ONE complex signal z = |a| + i |b|: the real part of the result is column a's lowpassed
// column, the imaginary part column b's.  Tiles of 2 TC columns, TC = 256 / T.
template <int MR>
__global__ __launch_bounds__(256, 4) void k_col_pair_low(const float2 *__restrict__ src, int Mc, int TC,
                                                      int wtab_off, const float *__restrict__ phi_rows,
                                                      float *__restrict__ w_out,
                                                      const float2 *__restrict__ tw, int tw_n) {
  constexpr int E = 16, T = MR / E, LM = 32;
  static_assert(T >= 4 && T <= 16, "64 to 256 rows");
  extern __shared__ float2 lds[];
  const int KS = T * TC + 16;
  const int cp = threadIdx.x % TC, t = threadIdx.x / TC;
  const int tiles = Mc / (2 * TC);
  const int node = blockIdx.x / tiles;
  const int c0 = (blockIdx.x % tiles) * (2 * TC);
  const float2 *sp = src + static_cast<size_t>(node) * MR * Mc + t * Mc + c0 + 2 * cp;
  const int step = T * Mc;
  // (the transforms' twiddles as a table in LDS behind the exchange area, [k T + t])
  float2 *wtab = lds + wtab_off;
  for (int idx = threadIdx.x; idx < MR; idx += 256) wtab[idx] = tw[(idx / T) * (idx % T) * (tw_n / MR)];
  __syncthreads();
  float2 va[E], vb[E];
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const float4 x = nt_load4(sp + i * step);  // (read once)
    va[i] = make_float2(x.x, x.y);
    vb[i] = make_float2(x.z, x.w);
  }
  fft_core_tab<E, T, true>(va, t, lds + cp, KS, TC, wtab + t, T);
  fft_core_tab<E, T, true>(vb, t, lds + cp, KS, TC, wtab + t, T);
#pragma unroll
  for (int i = 0; i < E; ++i)
    va[i] = make_float2(__builtin_amdgcn_sqrtf(va[i].x * va[i].x + va[i].y * va[i].y),
                        __builtin_amdgcn_sqrtf(vb[i].x * vb[i].x + vb[i].y * vb[i].y));
  fft_core_tab<E, T, false>(va, t, lds + cp, KS, TC, wtab + t, T);
  // fold in registers: row t + T i lands on lowpass frequency t + T (i mod JT)
  constexpr int JT = LM / T;
  float2 fm[JT];
#pragma unroll
  for (int j = 0; j < JT; ++j) fm[j] = make_float2(0.f, 0.f);
  const float *ph = phi_rows + t;
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const float f = ph[T * i];
    fm[i % JT].x += va[i].x * f;
    fm[i % JT].y += va[i].y * f;
  }
#pragma unroll
  for (int j = 0; j < JT; ++j) lds[(t + T * j) * TC + cp] = fm[j];
  __syncthreads();
  if (static_cast<int>(threadIdx.x) < 4 * TC) {
    // 4 lanes per column pair, 8 points each
    const int tp = threadIdx.x & 3, cc = threadIdx.x >> 2;
    float2 y[8], w2[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) y[i] = lds[(tp + 4 * i) * TC + cc];
    load_twiddles<8, 4>(w2, tp, tw, tw_n);
    fft_core<8, 4, true, true>(y, tp, lds + LM * TC + cc * 48, 5, 1, w2);
    float *wp = w_out + static_cast<size_t>(node) * LM * Mc + c0 + 2 * cc;
#pragma unroll
    for (int i = 0; i < 8; ++i) *reinterpret_cast<float2 *>(wp + (tp + 4 * i) * Mc) = y[i];
  }
}

template <int MR>
hipError_t launch_col_fast_t(int mode, const void *src, long nodes, int Mc, float2 *uc, bool uc_half,
                             int post_tw_m, const float *phi_rows, int m_r, float *w_out,
                             const float2 *tw, int tw_n, hipStream_t st) {
  constexpr int E = MR > 256 ? 32 : 16, T = MR / E;
  if (post_tw_m > 0 && (tw_n % post_tw_m != 0 || (post_tw_m & (post_tw_m - 1)) != 0)) return hipErrorInvalidValue;
  // half spectra with the four-step twiddle: the factored-twiddle path only (16 points per thread)
  if (post_tw_m > 0 && uc_half && (E != 16 || post_tw_m != MR * Mc || mode != 1)) return hipErrorInvalidValue;
  int TC = 256 / T;
  if (TC < 16) TC = 16;
  if (TC > Mc) TC = Mc;
  long blocks = nodes * (Mc / TC);
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  // lowpass tail variant: registers when the lowpass length is 32 or 8 and a multiple of T
  const int lm = (w_out && m_r == 32 && T <= 32 && tw_n >= 32) ? 32 : (w_out && m_r == 8 && T <= 8) ? 8 : 0;
  const int lm_t = (lm == 8 && MR > 128) ? 0 : lm;  // the template argument actually used
  if constexpr (E == 16 && T >= 4) {
    if (mode == 1 && uc == nullptr && lm == 32 && post_tw_m == 0 && Mc % (2 * TC) == 0 && T * TC == 256) {
      // leaves: two columns per thread (see k_col_pair_low)
      const long blocks2 = nodes * (Mc / (2 * TC));
      if (blocks2 <= 0 || blocks2 > 0x7fffffffL) return hipErrorInvalidValue;
      size_t words2 = static_cast<size_t>(E) * (T * TC + 16);
      if (static_cast<size_t>(80) * TC > words2) words2 = static_cast<size_t>(80) * TC;
      const size_t lds2 = (words2 + MR) * sizeof(float2);  // + the twiddle table
      const std::string name2 = "k_col_pair_low<" + std::to_string(MR) + ">";
      const double pts2 = static_cast<double>(nodes) * MR * Mc, cols2 = static_cast<double>(nodes) * Mc;
      Observe ob(name2.c_str(), pts2 * 8 + cols2 * m_r * 4 + MR * 4.0,
                 cols2 * (1.5 * fft_flops(MR) + fft_flops(m_r) + 2.0 * MR) + 4.0 * pts2, st);
      static unsigned long long lds_ok2 = 0;
      if (lds2 > 65536) {
        hipError_t e = allow_large_lds(reinterpret_cast<const void *>(k_col_pair_low<MR>), lds_ok2);
        if (e != hipSuccess) return e;
      }
      hipLaunchKernelGGL((k_col_pair_low<MR>), dim3(static_cast<unsigned>(blocks2)), dim3(256), lds2, st,
                         static_cast<const float2 *>(src), Mc, TC, static_cast<int>(words2), phi_rows, w_out, tw,
                         tw_n);
      return hipGetLastError();
    }
  }
  size_t words = static_cast<size_t>(E) * (T * TC + 16);
  if (lm_t == 0 && w_out) words += static_cast<size_t>(m_r) * TC;  // the generic tail's own area
  if (lm_t == 32 && static_cast<size_t>(80) * TC > words) words = static_cast<size_t>(80) * TC;
  size_t lds = words * sizeof(float2);
  if (lds > 160 * 1024) return hipErrorInvalidValue;
  dim3 g(static_cast<unsigned>(blocks)), b(T * TC);
  const std::string name = "k_col_fast<" + std::to_string(MR) + ", " + (mode ? "1" : "0") + ", " +
                           std::to_string(lm_t) + ">";
  const double pts = static_cast<double>(nodes) * MR * Mc;
  const double cols = static_cast<double>(nodes) * Mc;
  Observe ob(name.c_str(),
             pts * (mode == 0 ? 4 : 8) + (uc ? (uc_half ? cols * (MR / 2 + 1) : pts) * 8 : 0) +
                 (w_out ? cols * m_r * 4 + MR * 4.0 : 0),
             cols * ((mode ? 2 : 1) * fft_flops(MR) + (w_out ? fft_flops(m_r) + 2.0 * MR : 0)) +
                 (mode ? 4.0 * pts : 0),
             st);
#define SCAT_COL_LAUNCH(MODE_, LM_)                                                               \
  {                                                                                               \
    static unsigned long long lds_ok = 0;                                        \
    if (lds > 65536) {                                                            \
      hipError_t e = allow_large_lds(reinterpret_cast<const void *>(k_col_fast<MR, MODE_, LM_>), lds_ok); \
      if (e != hipSuccess) return e;                                        \
    }                                                                      \
    hipLaunchKernelGGL((k_col_fast<MR, MODE_, LM_>), g, b, lds, st, src, Mc, TC, uc,              \
                       static_cast<int>(uc_half), post_tw_m, phi_rows, m_r, w_out, tw, tw_n);     \
  }
  if (mode == 0) {
    if (lm == 32) SCAT_COL_LAUNCH(0, 32)
    else if (lm == 8) SCAT_COL_LAUNCH(0, (MR <= 128 ? 8 : 0))
    else SCAT_COL_LAUNCH(0, 0)
  } else {
    if (lm == 32) SCAT_COL_LAUNCH(1, 32)
    else if (lm == 8) SCAT_COL_LAUNCH(1, (MR <= 128 ? 8 : 0))
    else SCAT_COL_LAUNCH(1, 0)
  }
#undef SCAT_COL_LAUNCH
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// Column pass of a whole square node with the row half of the lowpass fused in: one
// workgroup walks the node's column tiles (each tile as in k_col_fast), keeps the
// column-lowpassed rows W (LM rows of MR reals) in LDS, and finishes with the row half
// (k_row_lowpass_fast's arithmetic) so that S goes straight to `out` and W never to memory.
// LM = lowpass length on both axes: 32 (needs MR >= 64) or 8 (MR <= 128); instantiated for
// MR >= 128 only.
template <int MR, int MODE, int LM, bool PF>
__global__ __launch_bounds__(256) void k_col_node(const void *__restrict__ src_v,
                                                  float2 *__restrict__ uc, int uc_half,
                                                  const float *__restrict__ phi_rows,
                                                  const float *__restrict__ phi_cols,
                                                  float *__restrict__ out, ChanMap cm, int K,
                                                  const float2 *__restrict__ tw, int tw_n) {
  constexpr int E = 16, T = MR / 16;
  constexpr int TC = (256 / T) < MR ? (256 / T) : MR;
  constexpr int KS = T * TC + 16;
  constexpr int XW = (16 * KS > 80 * TC) ? 16 * KS : 80 * TC;  // float2 words of scratch
  constexpr int WS = MR + 4;                                   // floats per W row
  constexpr int Mc = MR;
  constexpr int JT = LM / T > 0 ? LM / T : 1;
  extern __shared__ float2 lds[];
  float *Wl = reinterpret_cast<float *>(lds + XW);
  const int c = threadIdx.x % TC, t = threadIdx.x / TC;
  const int node = blockIdx.x;
  const size_t plane = static_cast<size_t>(node) * MR * Mc;
  const int step = T * Mc;
  // 128-row nodes (three workgroups per CU, bound by registers): the transforms' twiddles in
  // an LDS table behind W instead of 32 registers, which pays for requesting the next tile
  // before the current one is transformed
  constexpr bool EARLY = MR == 128;
  float2 *wtab = reinterpret_cast<float2 *>(Wl + LM * WS);  // wtab[k T + t], EARLY only
  float2 wt[E];
  if constexpr (EARLY) {
    for (int idx = threadIdx.x; idx < MR; idx += blockDim.x)
      wtab[idx] = tw[(idx / T) * (idx % T) * (tw_n / MR)];
    __syncthreads();
  } else {
    load_twiddles<E, T>(wt, t, tw, tw_n);
  }
  auto column_fft = [&](float2 (&v)[E], auto inv) {
    if constexpr (EARLY)
      fft_core_tab<E, T, decltype(inv)::value>(v, t, lds + c, KS, TC, wtab + t, T);
    else
      fft_core<E, T, decltype(inv)::value>(v, t, lds + c, KS, TC, wt);
  };
  float phr[E];
#pragma unroll
  for (int i = 0; i < E; ++i) phr[i] = phi_rows[t + T * i];
  // PF (used when the node stores its column spectra): the loads of the next tile are
  // issued before the stores of the current one, so that waiting for them never means
  // waiting for those stores to drain (memory operations of a wave retire in order).
  float2 vn[E];
  auto fetch = [&](int c0) {
    const int off0 = t * Mc + c0 + c;
    if (MODE == 0) {
      const float *sp = static_cast<const float *>(src_v) + plane + off0;
#pragma unroll
      for (int i = 0; i < E; ++i) vn[i] = make_float2(sp[i * step], 0.f);
    } else {
      const float2 *sp = static_cast<const float2 *>(src_v) + plane + off0;
#pragma unroll
      for (int i = 0; i < E; ++i) vn[i] = nt_load(sp + i * step);
    }
  };
  if (PF || EARLY) fetch(0);
#pragma unroll 1
  for (int c0 = 0; c0 < Mc; c0 += TC) {
    const int off0 = t * Mc + c0 + c;
    if (!PF && !EARLY) fetch(c0);
    float2 v[E];
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = vn[i];
    if (EARLY && c0 + TC < Mc) fetch(c0 + TC);
    if (MODE != 0) {
      column_fft(v, std::true_type{});
#pragma unroll
      for (int i = 0; i < E; ++i)
        v[i] = make_float2(__builtin_amdgcn_sqrtf(v[i].x * v[i].x + v[i].y * v[i].y), 0.f);
    }
    column_fft(v, std::false_type{});
    if (PF && !EARLY && c0 + TC < Mc) fetch(c0 + TC);
    if (uc != nullptr) {
      if (uc_half) {
        float2 *up = uc + static_cast<size_t>(node) * (MR / 2 + 1) * Mc + off0;
#pragma unroll
        for (int i = 0; i < E; ++i)
          if (t + T * i <= MR / 2) nt_store(up + i * step, v[i]);
      } else {
        float2 *up = uc + plane + off0;
#pragma unroll
        for (int i = 0; i < E; ++i) up[i * step] = v[i];
      }
    }
    // column half of the lowpass: fold in registers, small inverse transform, W tile to LDS
    float2 fm[JT];
#pragma unroll
    for (int j = 0; j < JT; ++j) fm[j] = make_float2(0.f, 0.f);
#pragma unroll
    for (int i = 0; i < E; ++i) {
      fm[i % JT].x += v[i].x * phr[i];
      fm[i % JT].y += v[i].y * phr[i];
    }
#pragma unroll
    for (int j = 0; j < JT; ++j) lds[(t + T * j) * TC + c] = fm[j];
    __syncthreads();
    if (LM == 32) {
      // 4 lanes per column, 8 points each (half the threads of a 32-column tile)
      if (static_cast<int>(threadIdx.x) < 4 * TC) {
        const int tp = threadIdx.x & 3, cc = threadIdx.x >> 2;
        float2 y[8], w2[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = lds[(tp + 4 * i) * TC + cc];
        load_twiddles<8, 4>(w2, tp, tw, tw_n);
        fft_core<8, 4, true, true>(y, tp, lds + LM * TC + cc * 48, 5, 1, w2);
#pragma unroll
        for (int i = 0; i < 8; ++i) Wl[(tp + 4 * i) * WS + c0 + cc] = y[i].x;
      }
    } else {
      if (static_cast<int>(threadIdx.x) < TC) {
        const int cc = threadIdx.x;
        float2 y[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = lds[i * TC + cc];
        DftRegs<8, true>::run(y);
#pragma unroll
        for (int i = 0; i < 8; ++i) Wl[i * WS + c0 + cc] = y[i].x;
      }
    }
    __syncthreads();
  }
  // ---- row half of the lowpass on W (LM rows, two rows per complex transform)
  constexpr int NP = LM / 2;  // row pairs
  if (static_cast<int>(threadIdx.x) >= NP * T) return;
  {
    const int pr = threadIdx.x / T, tr = threadIdx.x % T;
    float2 wr[E];
    load_twiddles<E, T>(wr, tr, tw, tw_n);
    float2 v[E];
    const float *w0 = Wl + (2 * pr) * WS + tr;
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = make_float2(w0[T * i], w0[WS + T * i]);
    float2 *xr = lds + pr * (16 * (T + 1));
    fft_core<E, T, false, true>(v, tr, xr, T + 1, 1, wr);
    float2 fm[JT];
#pragma unroll
    for (int j = 0; j < JT; ++j) fm[j] = make_float2(0.f, 0.f);
    const float *ph = phi_cols + tr;
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const float f = ph[T * i];
      fm[i % JT].x += v[i].x * f;
      fm[i % JT].y += v[i].y * f;
    }
#pragma unroll
    for (int j = 0; j < JT; ++j) xr[tr + T * j] = fm[j];
    wave_sync();
    const int pl = node / cm.G, g = node % cm.G;
    float *op = out + ((static_cast<size_t>(pl) * K + chan_of(cm, g)) * LM + 2 * pr) * LM;
    if (LM == 32) {
      if (tr < 4) {  // 4 lanes per row pair, 8 points each
        float2 y[8], w2[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = xr[tr + 4 * i];
        load_twiddles<8, 4>(w2, tr, tw, tw_n);
        fft_core<8, 4, true, true>(y, tr, xr + 32, 5, 1, w2);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          op[tr + 4 * i] = y[i].x;
          op[LM + tr + 4 * i] = y[i].y;
        }
      }
    } else {
      if (tr == 0) {
        float2 y[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = xr[i];
        DftRegs<8, true>::run(y);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          op[i] = y[i].x;
          op[LM + i] = y[i].y;
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------
// Leaf nodes of N x N points (no children below them) in one pass, the node held by one
// workgroup in LDS: row-pass output src [node][N][N] -> out[plane][channel][M][M], in place
// of the column kernel, its W rows in memory and the row-lowpass kernel, for nodes below the
// whole-node column kernel's range.  The two halves of the separable lowpass are taken one
// after the other, each right after the transform it follows, so that the row stage works
// on the M lowpassed rows only:
//   stage A (all 256 threads, thread = column c, rows t1 + 4 i): inverse column transform,
//     modulus, forward column transform, phi_rows and the alias sum over rows in registers,
//     inverse M-point column transform -> W [M][N] real, in LDS;
//   stage B (the first two wavefronts, 8 lanes per pair of rows of W, the pair travelling as
//     real and imaginary part of one complex row): forward row transform, phi_cols and the
//     alias sum over columns, regrouped through LDS, inverse M-point row transform -> S.
template <int N, int M>
__global__ __launch_bounds__(256) void k_leaf_node(const float2 *__restrict__ src,
                                                    const float *__restrict__ phi_rows,
                                                    const float *__restrict__ phi_cols,
                                                    float *__restrict__ out, ChanMap cm, int K,
                                                    const float2 *__restrict__ tw, int tw_n) {
  static_assert(N == 64 && M == 32, "thread layout below");
  constexpr int T1 = N / 16;  // 4 threads per column
  constexpr int RS = N;       // the exchange areas are accessed along c: no padding needed
  constexpr int WS = N + 1;   // floats per row of W
  extern __shared__ float2 lds[];
  float2 *area = lds;                           // N * RS: exchange areas of stage A
  float2 *wtab = lds + N * RS;                  // N: twiddles of the N-point columns
  // W takes the head of the area once stage A's transforms are done, stage B's exchange
  // areas follow it
  float *wl = reinterpret_cast<float *>(area);  // M * WS floats
  constexpr int WL2 = (M * WS + 1) / 2;         // the same in float2 elements
  const int q = threadIdx.x;
  for (int idx = q; idx < N; idx += 256) wtab[idx] = tw[(idx / T1) * (idx % T1) * (tw_n / N)];
  __syncthreads();
  const long node = blockIdx.x;
  {
    const int c = q % N, t1 = q / N;
    const float2 *sp = src + static_cast<size_t>(node) * N * N + c;
    float2 v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = nt_load(sp + (t1 + T1 * i) * N);
    fft_core_tab<16, T1, true, false>(v, t1, area + c, T1 * RS, RS, wtab + t1, T1);
#pragma unroll
    for (int i = 0; i < 16; ++i)
      v[i] = make_float2(__builtin_amdgcn_sqrtf(v[i].x * v[i].x + v[i].y * v[i].y), 0.f);
    fft_core_tab<16, T1, false, false>(v, t1, area + c, T1 * RS, RS, wtab + t1, T1);
    // rows k and k + M fold onto row k: registers i and i + 8
    float2 f[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float p0 = phi_rows[t1 + T1 * i], p1 = phi_rows[t1 + T1 * (i + 8)];
      f[i] = make_float2(v[i].x * p0 + v[i + 8].x * p1, v[i].y * p0 + v[i + 8].y * p1);
    }
    float2 w8[8];
    load_twiddles<8, T1>(w8, t1, tw, tw_n);
    fft_core<8, T1, true, false>(f, t1, area + c, T1 * RS, RS, w8);
#pragma unroll
    for (int i = 0; i < 8; ++i) wl[(t1 + T1 * i) * WS + c] = f[i].x;
  }
  __syncthreads();
  if (q >= 128) return;  // stage B: M / 2 row pairs, 8 lanes each, wave-level synchronisation only
  const int p = q / 8, t = q % 8;
  float2 z[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
    z[i] = make_float2(wl[(2 * p) * WS + t + 8 * i], wl[(2 * p + 1) * WS + t + 8 * i]);
  float2 *xb = area + WL2 + p * 80;  // 8 * (8 + 1) exchange elements, then the regrouping space
  {
    float2 w8[8];
    load_twiddles<8, 8>(w8, t, tw, tw_n);
    fft_core<8, 8, false, true>(z, t, xb, 9, 1, w8);
  }
  // columns k and k + M fold onto column k: registers i and i + 4
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float p0 = phi_cols[t + 8 * i], p1 = phi_cols[t + 8 * (i + 4)];
    xb[t + 8 * i] = make_float2(z[i].x * p0 + z[i + 4].x * p1, z[i].y * p0 + z[i + 4].y * p1);
  }
  wave_sync();
  if (t >= 4) return;  // 4 lanes per pair share the M-point inverse transform
  float2 g[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) g[i] = xb[t + 4 * i];
  wave_sync();
  {
    float2 w8[8];
    load_twiddles<8, 4>(w8, t, tw, tw_n);
    fft_core<8, 4, true, true>(g, t, xb + 32, 5, 1, w8);
  }
  const long pl = node / cm.G;
  const int gch = static_cast<int>(node - pl * cm.G);
  float *op = out + (static_cast<size_t>(pl) * K + chan_of(cm, gch)) * M * M + (2 * p) * M;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    op[t + 4 * i] = g[i].x;
    op[M + t + 4 * i] = g[i].y;
  }
}

bool leaf_node_supported_impl(int Mr, int Mc, int m_r, int m_c, int tw_n) {
  return Mr == 64 && Mc == 64 && m_r == 32 && m_c == 32 && tw_n % 64 == 0;
}

// True if launch_col_node handles nodes of MR x MR with lowpass length lm on both axes.
bool col_node_supported_impl(int Mr, int Mc, int m_r, int m_c, int tw_n) {
  if (Mr != Mc || m_r != m_c) return false;
  // (measured: the whole-node kernel wins from 128 x 128 up; smaller nodes leave too few
  // lanes busy in its final stage and keep the two-kernel path)
  if (m_r == 32) return (Mr == 128 || Mr == 256) && tw_n >= 32;
  if (m_r == 8) return Mr == 128;
  return false;
}

template <int MR, int LM>
hipError_t launch_col_node_t(int mode, const void *src, long nodes, float2 *uc, bool uc_half,
                             const float *phi_rows, const float *phi_cols, float *out, ChanMap cm,
                             int K, const float2 *tw, int tw_n, hipStream_t st) {
  constexpr int T = MR / 16;
  constexpr int TC = (256 / T) < MR ? (256 / T) : MR;
  constexpr int KS = T * TC + 16;
  constexpr int XW = (16 * KS > 80 * TC) ? 16 * KS : 80 * TC;
  constexpr int WS = MR + 4;
  if (nodes <= 0 || nodes > 0x7fffffffL) return hipErrorInvalidValue;
  size_t lds = static_cast<size_t>(XW) * sizeof(float2) + static_cast<size_t>(LM) * WS * sizeof(float) +
               (MR == 128 ? MR * sizeof(float2) : 0);  // + the twiddle table of the 128-row variant
  const std::string name = "k_col_node<" + std::to_string(MR) + ", " + (mode ? "1" : "0") + ", " +
                           std::to_string(LM) + ((uc != nullptr && MR >= 256) ? ", true>" : ", false>");
  const double pts = static_cast<double>(nodes) * MR * MR;
  const double cols = static_cast<double>(nodes) * MR;
  Observe ob(name.c_str(),
             pts * (mode == 0 ? 4 : 8) + (uc ? (uc_half ? cols * (MR / 2 + 1) : pts) * 8 : 0) +
                 static_cast<double>(nodes) * LM * LM * 4,
             cols * ((mode ? 2 : 1) * fft_flops(MR) + fft_flops(LM) + 2.0 * MR) + (mode ? 4.0 * pts : 0) +
                 static_cast<double>(nodes) * LM * 0.5 * (fft_flops(MR) + fft_flops(LM) + 2.0 * MR),
             st);
  dim3 g(static_cast<unsigned>(nodes)), b(T * TC);
#define SCAT_CN_LAUNCH(MODE_, PF_)                                                                 \
  {                                                                                                \
    static unsigned long long lds_ok = 0;                                        \
    if (lds > 65536) {                                                            \
      hipError_t e = allow_large_lds(reinterpret_cast<const void *>(k_col_node<MR, MODE_, LM, PF_>), lds_ok); \
      if (e != hipSuccess) return e;                                        \
    }                                                                      \
    hipLaunchKernelGGL((k_col_node<MR, MODE_, LM, PF_>), g, b, lds, st, src, uc,                   \
                       static_cast<int>(uc_half), phi_rows, phi_cols, out, cm, K, tw, tw_n);       \
  }
  // (measured: the prefetch pays for 256-row nodes only; it costs 32 registers)
  const bool pf = uc != nullptr && MR >= 256;
  if (mode == 0) {
    if (pf) SCAT_CN_LAUNCH(0, (MR >= 256)) else SCAT_CN_LAUNCH(0, false)
  } else {
    if (pf) SCAT_CN_LAUNCH(1, (MR >= 256)) else SCAT_CN_LAUNCH(1, false)
  }
#undef SCAT_CN_LAUNCH
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// Fused row pass: forward row FFT of column-transformed sources, then for every level
// (one octave of wavelets applied at fold 2^f) filter multiply + fold + inverse row FFT.
// The full 2-D spectrum of the source therefore never goes to memory.
//
// src : [NS][Sr][SC] complex, rows already transformed along columns (k_r, c).
// Rows are processed in groups {q + (Sr/G) a, a < G}, G = 2^fmax, which are closed under
// every level's row fold.  A workgroup takes NGRP consecutive groups of two consecutive
// sources; the two sources share every filter value that is loaded.
// Level output: dst[(src * F + theta)][q_r][.] for q_r < Sr >> f, row length SC >> f.
struct FusedLevelDev {
  int f, F;
  const float *filt;  // [F][Sr][SC], carries the 1/(Sr*SC) normalisation
  float2 *dst;        // [NS*F][Sr>>f][SC>>f]
};
struct FusedArgsDev {
  FusedLevelDev lv[4];
  int nlev;
};

// Filter values of CPL consecutive columns.
template <int CPL>
struct FiltVec;
template <>
struct FiltVec<1> {
  float f[1];
  __device__ __forceinline__ void load(const float *p) { f[0] = *p; }
};
template <>
struct FiltVec<2> {
  float f[2];
  __device__ __forceinline__ void load(const float *p) {
    const float2 v = *reinterpret_cast<const float2 *>(p);
    f[0] = v.x;
    f[1] = v.y;
  }
};
template <>
struct FiltVec<4> {
  float f[4];
  __device__ __forceinline__ void load(const float *p) {
    const float4 v = *reinterpret_cast<const float4 *>(p);
    f[0] = v.x;
    f[1] = v.y;
    f[2] = v.z;
    f[3] = v.w;
  }
};

// CPL consecutive complex values from LDS (16-byte reads where possible).
template <int CPL>
__device__ __forceinline__ void lds_read_cols(float2 (&d)[CPL], const float2 *p) {
  if (CPL == 1) {
    d[0] = p[0];
  } else {
#pragma unroll
    for (int e = 0; e < CPL; e += 2) {
      const float4 u = *reinterpret_cast<const float4 *>(p + e);
      d[e] = make_float2(u.x, u.y);
      d[(e + 1) % CPL] = make_float2(u.z, u.w);
    }
  }
}

// LDS strides (in float2) chosen so that the lanes of half a wavefront fall on distinct
// banks: row stride of the source rows, and slot stride of the product/exchange area for
// transforms of EL points per lane shared by TP lanes (at least EL*(TP+1) for the exchange).
__host__ __device__ constexpr int fused_row_stride(int SC) { return SC + 16; }
__host__ __device__ constexpr int fused_slot_stride(int EL, int TP) {
  return TP == 1 ? EL
         : EL == 8 ? 72  /* TP == 8 */
         : TP == 16 ? 272 : TP == 8 ? 152 : TP == 4 ? 84 : 50;
}
// Transform shape used for an output row of M points: 64 points go as 8 lanes x 8 points so
// that a wave's 8 items fill all lanes; everything else as 16 points per lane.
__host__ __device__ constexpr int fused_el(int M) { return M == 64 ? 8 : 16; }

// One level of the fused row pass for one wavefront.  The wave owns the LDS rows R
// (rows of SC points, natural order, stride fused_row_stride) of its source.  Items =
// (output row, filter), filter index fastest; 64/TP of them form a batch: first every
// item's folded product row is accumulated by the whole wave (lane l owns M/64 consecutive
// output columns, so filter and LDS reads are contiguous across the wave) into B, then each
// group of TP lanes transforms one row.  The source values an output row needs are read
// from LDS once and kept in registers for all filters of that row.  The accumulation runs
// in chunks of IC items (about 32 filter loads per lane); the loads of the next chunk are
// issued before the transforms of the current batch.
// lgG, lgNGRP: log2 of the rows per group and of the groups per wave.
template <int SC, int FL>
__device__ __forceinline__ void fused_level_w(const FusedLevelDev &L, int Sr, int lgG, int lgNGRP,
                                              long src_idx, int grp0, const float2 *R, float2 *B,
                                              int lane, const float2 *twl) {
  constexpr int M = SC >> FL;
  constexpr int EL = fused_el(M);
  constexpr int TP = M / EL;
  constexpr int SLOTS = 64 / TP;
  constexpr int CPL = M >= 64 ? M / 64 : 1;  // output columns per lane
  constexpr int SS = fused_slot_stride(EL, TP);
  constexpr int RS = fused_row_stride(SC);
  constexpr int NF = 1 << FL, TERMS = NF * NF;
  constexpr int IC0 = 32 / TERMS < 1 ? 1 : 32 / TERMS;
  constexpr int IC = IC0 > SLOTS ? SLOTS : IC0;
  constexpr int CPB = SLOTS / IC;                // chunks per batch
  constexpr bool CACHE = TERMS * CPL <= 16;      // keep a row set's source values in registers
  constexpr int NRT = CACHE ? TERMS : 1;
  const int lgGf = lgG - FL;
  const int Gf = 1 << lgGf;
  const int Mr = Sr >> FL;
  const int F = L.F;
  const int items = F << (lgGf + lgNGRP);
  const int rows_step = Sr >> lgG;
  const int slot = lane / TP, t = lane % TP;
  const int lcol = (lane * CPL) % M;  // lanes past M (only when M < 64) repeat valid columns
  const int nchunks = (items + IC - 1) / IC;

  FiltVec<CPL> fv[IC][TERMS];
  int rs_of[IC];            // row set (g, ap) of each item of the chunk in flight
  int nx_theta = 0, nx_rs = 0;  // next item to issue
  auto issue = [&]() {
#pragma unroll
    for (int s = 0; s < IC; ++s) {
      const int g = nx_rs >> lgGf, ap = nx_rs & (Gf - 1);
      const int qr = grp0 + g + rows_step * ap;
      const float *fp = L.filt + (static_cast<size_t>(nx_theta) * Sr + qr) * SC;  // wave-uniform
      rs_of[s] = nx_rs;
#pragma unroll
      for (int a = 0; a < NF; ++a)
#pragma unroll
        for (int b = 0; b < NF; ++b)
          fv[s][a * NF + b].load(fp + static_cast<size_t>(a) * Mr * SC + b * M + lcol);
      // advance; past the last item the last one is recomputed (harmless)
      if (nx_theta + 1 < F) {
        ++nx_theta;
      } else if (nx_rs + 1 < (1 << (lgGf + lgNGRP))) {
        nx_theta = 0;
        ++nx_rs;
      }
    }
  };
  float2 rt[NRT][CPL];
  int cur_rs = -1;
  issue();
  for (int c = 0; c < nchunks; ++c) {
    const int s0 = (c % CPB) * IC;
#pragma unroll
    for (int s = 0; s < IC; ++s) {
      const int rs = rs_of[s];
      const int g = rs >> lgGf, ap = rs & (Gf - 1);
      const float2 *rb = R + static_cast<size_t>((g << lgG) + ap) * RS + lcol;
      if (CACHE && rs != cur_rs) {
        cur_rs = rs;
#pragma unroll
        for (int a = 0; a < NF; ++a)
#pragma unroll
          for (int b = 0; b < NF; ++b)
            lds_read_cols<CPL>(rt[(a * NF + b) % NRT], rb + static_cast<size_t>(a * Gf) * RS + b * M);
      }
      float2 acc[CPL];
#pragma unroll
      for (int e = 0; e < CPL; ++e) acc[e] = make_float2(0.f, 0.f);
#pragma unroll
      for (int a = 0; a < NF; ++a)
#pragma unroll
        for (int b = 0; b < NF; ++b) {
          if (!CACHE) lds_read_cols<CPL>(rt[0], rb + static_cast<size_t>(a * Gf) * RS + b * M);
          const int k = CACHE ? a * NF + b : 0;
#pragma unroll
          for (int e = 0; e < CPL; ++e) {
            acc[e].x += rt[k][e].x * fv[s][a * NF + b].f[e];
            acc[e].y += rt[k][e].y * fv[s][a * NF + b].f[e];
          }
        }
#pragma unroll
      for (int e = 0; e < CPL; ++e) B[(s0 + s) * SS + lcol + e] = acc[e];
    }
    if (c + 1 < nchunks) issue();
    if ((c + 1) % CPB != 0 && c + 1 != nchunks) continue;
    // ---- a batch of product rows is complete: transform and store it
    const int it0 = (c / CPB) * SLOTS;
    wave_sync();
    const int item = it0 + slot;
    const bool active = item < items;
    float2 v[EL];
#pragma unroll
    for (int i = 0; i < EL; ++i) v[i] = B[slot * SS + t + TP * i];
    wave_sync();
    // twiddles come from the workgroup's LDS copy of the table: a global load here would
    // queue behind the filter prefetch and the previous batch's stores
    float2 wt[EL];
#pragma unroll
    for (int k1 = 0; k1 < EL; ++k1) wt[k1] = twl[t * k1 * (SC / M)];
    fft_core<EL, TP, true, true>(v, t, B + slot * SS, TP + 1, 1, wt);
    if (TP == 1) wave_sync();
    if (active) {
      const int rs = item / F, theta = item - rs * F;
      const int g = rs >> lgGf, ap = rs & (Gf - 1);
      const int qr = grp0 + g + rows_step * ap;
      float2 *dp = L.dst + ((static_cast<size_t>(src_idx) * F + theta) * Mr + qr) * M + t;
#pragma unroll
      for (int i = 0; i < EL; ++i) nt_store(dp + TP * i, v[i]);
    }
  }
}

// Workgroup = 4 wavefronts; wave w handles source 4*(block / per_src) + w and NGRP row
// groups starting at grp0, entirely on its own (no workgroup barrier anywhere; the four
// waves only share the filter rows they read through the L1 cache).
// LDS: SC twiddles shared by the workgroup, then per wave rows_w * fused_row_stride(SC)
// (rows) + b_words (product rows / exchange), in float2.  MASK: bit f set = a level with fold 2^f may occur (only those variants are
// compiled in, which keeps the kernel's register allocation at that of its heaviest level).
template <int SC, int MASK>
__global__ __launch_bounds__(256, 2) void k_rows_fused(const float2 *__restrict__ src, int src_half,
                                                    long NS, int Sr, int G, int b_words,
                                                    FusedArgsDev args,
                                                    const float2 *__restrict__ tw, int tw_n) {
  constexpr int T = SC / 16;
  constexpr int RPW = 64 / T;  // rows one wave transforms at a time
  extern __shared__ float2 lds[];
  const int lane = threadIdx.x & 63;
  // the wave number is the same in all lanes: keep it (and all that derives from it) scalar
  const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
  const int rows_w = RPW > G ? RPW : G;
  const int NGRP = rows_w / G;
  const int groups = Sr / G;
  const int per_src = groups / NGRP;
  const long src_idx = 4 * static_cast<long>(blockIdx.x / per_src) + wave;
  const int grp0 = (blockIdx.x % per_src) * NGRP;
  // LDS copy of the SC-point twiddle table, shared by the workgroup
  float2 *twl = lds;
  for (int j = threadIdx.x; j < SC; j += blockDim.x) twl[j] = tw[j * (tw_n / SC)];
  __syncthreads();
  if (src_idx >= NS) return;
  constexpr int RS = fused_row_stride(SC);
  float2 *R = lds + SC + static_cast<size_t>(wave) * (static_cast<size_t>(rows_w) * RS + b_words);
  float2 *B = R + static_cast<size_t>(rows_w) * RS;
  {
    const int t = lane % T, rl = lane / T;
    float2 wt[16];
#pragma unroll
    for (int k1 = 0; k1 < 16; ++k1) wt[k1] = twl[t * k1];
    for (int pass = 0; pass < rows_w / RPW; ++pass) {
      const int rr = pass * RPW + rl;
      const int g = rr / G, ag = rr % G;
      // src_half: the source holds rows 0..Sr/2 only (column spectra of a real signal);
      // row r > Sr/2 is the conjugate of row Sr - r
      const int r = grp0 + g + groups * ag;
      const bool mirror = src_half && r > Sr / 2;
      const int r_st = mirror ? Sr - r : r;
      const int rows_st = src_half ? Sr / 2 + 1 : Sr;
      const float2 *sp = src + (static_cast<size_t>(src_idx) * rows_st + r_st) * SC + t;
      float2 v[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = sp[T * i];
      if (mirror) {
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i].y = -v[i].y;
      }
      fft_core<16, T, false, true>(v, t, B + rl * fused_slot_stride(16, T), T + 1, 1, wt);
#pragma unroll
      for (int i = 0; i < 16; ++i) R[rr * RS + t + T * i] = v[i];
    }
    wave_sync();
  }
  const int lgG = ilog2(G), lgNGRP = ilog2(NGRP);
  for (int l = 0; l < args.nlev; ++l) {
    const FusedLevelDev &L = args.lv[l];
    switch (L.f) {
      case 0: if (MASK & 1) fused_level_w<SC, 0>(L, Sr, lgG, lgNGRP, src_idx, grp0, R, B, lane, twl); break;
      case 1: if (MASK & 2) fused_level_w<SC, 1>(L, Sr, lgG, lgNGRP, src_idx, grp0, R, B, lane, twl); break;
      case 2: if ((MASK & 4) && SC >= 64) fused_level_w<(SC >= 64 ? SC : 64), 2>(L, Sr, lgG, lgNGRP, src_idx, grp0, R, B, lane, twl); break;
      case 3: if ((MASK & 8) && SC >= 128) fused_level_w<(SC >= 128 ? SC : 128), 3>(L, Sr, lgG, lgNGRP, src_idx, grp0, R, B, lane, twl); break;
      default: break;
    }
  }
}


// ------------------------------------------------------------------------------------
// Row half of the separable lowpass with register-resident transforms (row length
// MC = 16 * T).  Two consecutive rows of a node travel as the real and imaginary part of
// one complex signal: the lowpass is a real linear map, so the real part of the result
// belongs to the first row and the imaginary part to the second.  Same contract as
// k_row_lowpass; m_r must be even.  256 / T row pairs per workgroup; the T lanes of a pair
// sit in one wavefront, so only wave-level synchronisation is used.
// LM_C = compile-time output length (32 or 8: fold in registers, small inverse transform by
// 2 lanes or 1 lane of the pair) or 0 = any length (generic tail through lds_fft).
template <int MC, int LM_C>
__global__ __launch_bounds__(256) void k_row_lowpass_fast(const float *__restrict__ w, long pairs,
                                                          int m_r, int m_c,
                                                          const float *__restrict__ phi_cols,
                                                          float *__restrict__ out, ChanMap cm, int K,
                                                          const float2 *__restrict__ tw, int tw_n) {
  constexpr int E = 16, T = MC / 16, RP = 256 / T;
  constexpr int XS = 16 * (T + 1) + (LM_C > 0 ? 48 : 0);
  extern __shared__ float2 lds[];
  const int pr = threadIdx.x / T, t = threadIdx.x % T;
  const long gp0 = static_cast<long>(blockIdx.x) * RP;
  const long gp = gp0 + pr;
  const bool valid = gp < pairs;
  float2 wt[E];
  load_twiddles<E, T>(wt, t, tw, tw_n);
  float2 v[E];
  if (valid) {
    const float *wp = w + static_cast<size_t>(2 * gp) * MC + t;
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = make_float2(wp[T * i], wp[MC + T * i]);
  } else {
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = make_float2(0.f, 0.f);
  }
  float2 *xch = lds + pr * XS;
  if (LM_C > 0) {
    fft_core<E, T, false, true>(v, t, xch, T + 1, 1, wt);
    constexpr int JT = LM_C / T > 0 ? LM_C / T : 1;
    float2 fm[JT];
#pragma unroll
    for (int j = 0; j < JT; ++j) fm[j] = make_float2(0.f, 0.f);
    const float *ph = phi_cols + t;
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const float f = ph[T * i];
      fm[i % JT].x += v[i].x * f;
      fm[i % JT].y += v[i].y * f;
    }
#pragma unroll
    for (int j = 0; j < JT; ++j) xch[t + T * j] = fm[j];
    wave_sync();
    if (!valid) return;
    const long row = 2 * gp;
    const long node = row / m_r;
    const int r = static_cast<int>(row % m_r);
    const long pl = node / cm.G;
    const int g = static_cast<int>(node % cm.G);
    float *op = out + ((static_cast<size_t>(pl) * K + chan_of(cm, g)) * m_r + r) * LM_C;
    if (LM_C == 32 && T >= 4) {
      if (t < 4) {  // 4 lanes per row pair, 8 points each
        float2 y[8], w2[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = xch[t + 4 * i];
        load_twiddles<8, 4>(w2, t, tw, tw_n);
        fft_core<8, 4, true, true>(y, t, xch + 16 * (T + 1), 5, 1, w2);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          op[t + 4 * i] = y[i].x;
          op[LM_C + t + 4 * i] = y[i].y;
        }
      }
    } else if (LM_C == 32) {
      if (t < 2) {
        float2 y[16], w2[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) y[i] = xch[t + 2 * i];
        load_twiddles<16, 2>(w2, t, tw, tw_n);
        fft_core<16, 2, true, true>(y, t, xch + 16 * (T + 1), 3, 1, w2);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          op[t + 2 * i] = y[i].x;
          op[LM_C + t + 2 * i] = y[i].y;
        }
      }
    } else {
      if (t == 0) {
        float2 y[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = xch[i];
        DftRegs<8, true>::run(y);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          op[i] = y[i].x;
          op[LM_C + i] = y[i].y;
        }
      }
    }
    return;
  }
  fft_core<E, T, false>(v, t, xch, T + 1, 1, wt);
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const int k = t + T * i;
    const float f = phi_cols[k];
    xch[k] = make_float2(v[i].x * f, v[i].y * f);
  }
  __syncthreads();
  float2 *low = lds + RP * XS;
  const int log2m = ilog2(m_c);
  const int nf = MC / m_c;
  for (int idx = threadIdx.x; idx < RP * m_c; idx += blockDim.x) {
    const int q = idx / m_c, m = idx % m_c;
    float2 acc = make_float2(0.f, 0.f);
    for (int b = 0; b < nf; ++b) acc = cadd(acc, lds[q * XS + m + b * m_c]);
    low[q * m_c + bitrev(m, log2m)] = acc;
  }
  lds_fft<true, false>(low, log2m, RP, m_c, 1, tw, tw_n);
  for (int idx = threadIdx.x; idx < RP * m_c; idx += blockDim.x) {
    const int q = idx / m_c, m = idx % m_c;
    const long g2 = gp0 + q;
    if (g2 >= pairs) continue;
    const long row = 2 * g2;
    const long node = row / m_r;
    const int r = static_cast<int>(row % m_r);
    const long pl = node / cm.G;
    const int g = static_cast<int>(node % cm.G);
    float *op = out + ((static_cast<size_t>(pl) * K + chan_of(cm, g)) * m_r + r) * m_c + m;
    const float2 val = low[idx];
    op[0] = val.x;
    op[m_c] = val.y;
  }
}

template <int MC>
hipError_t launch_row_lowpass_fast_t(const float *w, long nodes, int m_r, int m_c,
                                     const float *phi_cols, float *out, ChanMap cm, int K,
                                     const float2 *tw, int tw_n, hipStream_t st) {
  constexpr int T = MC / 16, RP = 256 / T;
  const long pairs = nodes * m_r / 2;
  long blocks = (pairs + RP - 1) / RP;
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  // tail variant: registers when the output length is 32 (needs T >= 2 lanes) or 8
  const int lm = (m_c == 32 && T >= 2 && T <= 32 && tw_n >= 32) ? 32 : (m_c == 8 && T <= 8) ? 8 : 0;
  const int XS = 16 * (T + 1) + (lm > 0 ? 48 : 0);
  size_t lds = (static_cast<size_t>(RP) * XS + (lm > 0 ? 0 : static_cast<size_t>(RP) * m_c)) * sizeof(float2);
  const double rws = static_cast<double>(nodes) * m_r;
  const std::string name = "k_row_lowpass_fast<" + std::to_string(MC) + ", " + std::to_string(lm) + ">";
  Observe ob(name.c_str(), rws * (MC + m_c) * 4,
             rws * 0.5 * (fft_flops(MC) + fft_flops(m_c) + 2.0 * MC), st);
  dim3 g(static_cast<unsigned>(blocks)), b(256);
  if (lds > 160 * 1024) return hipErrorInvalidValue;
#define SCAT_RLP_LAUNCH(LM_)                                                                       \
  {                                                                                                \
    static unsigned long long lds_ok = 0;                                        \
    if (lds > 65536) {                                                            \
      hipError_t e = allow_large_lds(reinterpret_cast<const void *>(k_row_lowpass_fast<MC, LM_>), lds_ok); \
      if (e != hipSuccess) return e;                                        \
    }                                                                      \
    hipLaunchKernelGGL((k_row_lowpass_fast<MC, LM_>), g, b, lds, st, w, pairs, m_r, m_c, phi_cols, \
                       out, cm, K, tw, tw_n);                                                      \
  }
  if (lm == 32) SCAT_RLP_LAUNCH((MC >= 32 ? 32 : 0))
  else if (lm == 8) SCAT_RLP_LAUNCH((MC <= 128 ? 8 : 0))
  else SCAT_RLP_LAUNCH(0)
#undef SCAT_RLP_LAUNCH
  return hipGetLastError();
}

constexpr int kThreads = 256;
constexpr int kTileElems = 4096;  // complex elements of one workgroup's LDS tile (32 KB)

int pow2_floor(int v) {
  int p = 1;
  while (2 * p <= v) p *= 2;
  return p;
}

template <int E, int T>
hipError_t launch_mulfold_reg_t(const float2 *src, const float *filt, float2 *dst, long S, int F,
                                int Sr, int Sc, int fr, int fc, int post_tw_m, const float2 *tw,
                                int tw_n, hipStream_t st, const unsigned long long *mask) {
  constexpr int NT = E == 32 ? 128 : 256, RPB = NT / T;
  const int Mr = Sr >> fr, Mc = Sc >> fc;
  int lgMr = 0;
  while ((1 << lgMr) < Mr) ++lgMr;
  const bool split = lgMr >= 3;  // one eighth of the output rows per XCD (see the kernel)
  const long rows = split ? S * F * (Mr / 8) : S * F * Mr;
  const long blocks = ((rows + RPB - 1) / RPB) * (split ? 8 : 1);
  if (rows <= 0 || blocks > 0x7fffffffL || tw_n % (E * T) != 0) return hipErrorInvalidValue;
  if (post_tw_m > 0 && (tw_n % post_tw_m != 0 || (post_tw_m & (post_tw_m - 1)) != 0))
    return hipErrorInvalidValue;
  const size_t lds = static_cast<size_t>(RPB) * (T == 1 ? E : E * (T + 1)) * sizeof(float2);
  const double spts = static_cast<double>(S) * Sr * Sc, opts = static_cast<double>(S) * F * Mr * Mc;
  const bool multi = F >= 2 && (E * T >= 64 || (E * T >= 32 && Sc >= 64));
  // block masks: at most 64 alias blocks
  const unsigned long long *mk = fr + fc <= 6 ? mask : nullptr;
  const std::string name = "k_mulfold_reg<" + std::to_string(E) + ", " + std::to_string(T) +
                           (multi ? ", true>" : ", false>");
  Observe ob(name.c_str(), spts * 8 + static_cast<double>(F) * Sr * Sc * 4 + opts * 8,
             static_cast<double>(S) * F * Mr * fft_flops(Mc) + 4.0 * spts * F, st);
  if (multi)
    hipLaunchKernelGGL((k_mulfold_reg<E, T, true>), dim3(static_cast<unsigned>(blocks)),
                       dim3(NT), lds, st, src, filt, dst, rows, F, Sr, Sc, fr, fc, lgMr, post_tw_m,
                       tw, tw_n, mk);
  else
    hipLaunchKernelGGL((k_mulfold_reg<E, T, false>), dim3(static_cast<unsigned>(blocks)), dim3(NT),
                       lds, st, src, filt, dst, rows, F, Sr, Sc, fr, fc, lgMr, post_tw_m, tw, tw_n, mk);
  return hipGetLastError();
}

template <int E, int T>
hipError_t launch_row_fwd_reg_t(float2 *data, long rows, const float2 *tw, int tw_n,
                                hipStream_t st) {
  constexpr int NT = E == 32 ? 128 : 256, RPB = NT / T;
  const long blocks = (rows + RPB - 1) / RPB;
  if (rows <= 0 || blocks > 0x7fffffffL || tw_n % (E * T) != 0) return hipErrorInvalidValue;
  const size_t lds = T == 1 ? 0 : static_cast<size_t>(RPB) * E * (T + 1) * sizeof(float2);
  const std::string name = "k_row_fwd_reg<" + std::to_string(E) + ", " + std::to_string(T) + ">";
  Observe ob(name.c_str(), static_cast<double>(rows) * E * T * 16,
             static_cast<double>(rows) * fft_flops(E * T), st);
  hipLaunchKernelGGL((k_row_fwd_reg<E, T>), dim3(static_cast<unsigned>(blocks)), dim3(NT), lds, st,
                     data, rows, tw, tw_n);
  return hipGetLastError();
}

}  // namespace

// ----------------------------------------------------------------------------- launchers

void set_launch_observer(LaunchObserver *o) { g_observer = o; }

template <int E, int T>
hipError_t launch_rows1d_reg_t(const float2 *src, long rows, int Sr, const Rows1dArgs &a, double bytes,
                               double flops, const float2 *tw, int tw_n, hipStream_t st, bool half) {
  constexpr int Sc = E * T, RPB = 256 / T;
  constexpr int XS = ((T == 1 ? E : E * (T + 1)) + (T >= 4 ? 16 : 0)) | 1;  // as in the kernel
  const long blocks = (rows + RPB - 1) / RPB;
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const size_t lds = (static_cast<size_t>(Sc) + static_cast<size_t>(RPB) * XS) * sizeof(float2);
  const std::string name = "k_rows1d_reg<" + std::to_string(E) + ", " + std::to_string(T) + (half ? ", true>" : ", false>");
  Observe ob(name.c_str(), bytes, flops, st);
  if (half)
    hipLaunchKernelGGL((k_rows1d_reg<E, T, true>), dim3(static_cast<unsigned>(blocks)), dim3(256), lds, st, src,
                       rows, Sr, a, tw, tw_n);
  else
    hipLaunchKernelGGL((k_rows1d_reg<E, T, false>), dim3(static_cast<unsigned>(blocks)), dim3(256), lds, st, src,
                       rows, Sr, a, tw, tw_n);
  return hipGetLastError();
}

bool rows1d_half_supported(int Sr, int Sc) {
  return Sr >= 4 && (Sr & (Sr - 1)) == 0 && (Sc == 4 || Sc == 8 || Sc == 16 || Sc == 32 || Sc == 64 || Sc == 128 || Sc == 256);
}

hipError_t launch_rows1d(const float2 *src, long nodes, int Sr, int Sc, const Rows1dArgs &a,
                         const float2 *tw, int tw_n, hipStream_t st, bool half_rows) {
  if (nodes <= 0 || a.n <= 0) return hipSuccess;
  if (half_rows && !rows1d_half_supported(Sr, Sc)) return hipErrorInvalidValue;
  if (a.spec_out != nullptr && (half_rows || !rows1d_half_supported(Sr, Sc))) return hipErrorInvalidValue;
  auto is_pow2 = [](int v) { return v > 0 && (v & (v - 1)) == 0; };
  if (a.n > kRows1dMaxChildren || !is_pow2(Sr) || !is_pow2(Sc) || Sc < 2 || Sc > kTileElems ||
      tw_n % Sc != 0)
    return hipErrorInvalidValue;
  int lgSc = 0;
  while ((1 << lgSc) < Sc) ++lgSc;
  const long rows_in = nodes * (half_rows ? Sr / 2 + 1 : Sr);  // stored source rows
  double bytes = static_cast<double>(rows_in) * Sc * 8, flops = fft_flops(Sc) * (half_rows ? 0.5 : 1.0);
  for (int i = 0; i < a.n; ++i) {
    const Rows1dChild &c = a.c[i];
    if (c.filt == nullptr || c.dst == nullptr || c.lg_fold < 0 || c.lg_fold > lgSc ||
        (c.post_tw_m > 0 && (c.post_tw_m != Sr * (Sc >> c.lg_fold) || tw_n % c.post_tw_m != 0)) ||
        (c.K > 0 && (c.cm.G < 1 || c.cm.inner < 1 || nodes % c.cm.G != 0)))
      return hipErrorInvalidValue;
    const double m = static_cast<double>(Sc >> c.lg_fold);
    bytes += static_cast<double>(Sr) * Sc * 4 + static_cast<double>(nodes) * Sr * m * 8;
    flops += 4.0 * Sc + fft_flops(m);
  }
  const double all_flops = static_cast<double>(nodes) * Sr * flops;
  switch (Sc) {
    case 4: return launch_rows1d_reg_t<4, 1>(src, rows_in, Sr, a, bytes, all_flops, tw, tw_n, st, half_rows);
    case 8: return launch_rows1d_reg_t<8, 1>(src, rows_in, Sr, a, bytes, all_flops, tw, tw_n, st, half_rows);
    case 16: return launch_rows1d_reg_t<16, 1>(src, rows_in, Sr, a, bytes, all_flops, tw, tw_n, st, half_rows);
    case 32: return launch_rows1d_reg_t<16, 2>(src, rows_in, Sr, a, bytes, all_flops, tw, tw_n, st, half_rows);
    case 64: return launch_rows1d_reg_t<16, 4>(src, rows_in, Sr, a, bytes, all_flops, tw, tw_n, st, half_rows);
    case 128: return launch_rows1d_reg_t<16, 8>(src, rows_in, Sr, a, bytes, all_flops, tw, tw_n, st, half_rows);
    case 256: return launch_rows1d_reg_t<16, 16>(src, rows_in, Sr, a, bytes, all_flops, tw, tw_n, st, half_rows);
    default: break;
  }
  // other row lengths: spectrum rows and one child's rows side by side in LDS
  // (2 * RB * Sc elements), then the twiddle table
  int RB = pow2_floor(kTileElems / 2 / Sc);
  if (RB < 1) RB = 1;
  if (RB > Sr) RB = Sr;
  const long blocks = nodes * Sr / RB;
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const size_t lds = (2 * static_cast<size_t>(RB) + 1) * Sc * sizeof(float2);
  if (lds > 65536) {
    static unsigned long long lds_ok = 0;
    hipError_t e = allow_large_lds(reinterpret_cast<const void *>(k_rows1d), lds_ok);
    if (e != hipSuccess) return e;
  }
  Observe ob("k_rows1d", bytes, static_cast<double>(nodes) * Sr * flops, st);
  hipLaunchKernelGGL(k_rows1d, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), lds, st, src, Sr,
                     Sc, RB, a, tw, tw_n);
  return hipGetLastError();
}

hipError_t launch_mulfold_invrow(const float2 *src, const float *filt, float2 *dst, long S, int F,
                                 int Sr, int Sc, int fr, int fc, int post_tw_m, const float2 *tw,
                                 int tw_n, hipStream_t st, const unsigned long long *mask) {
  const int Mr = Sr >> fr, Mc = Sc >> fc;
#define SCAT_MF(E_, T_) \
  return launch_mulfold_reg_t<E_, T_>(src, filt, dst, S, F, Sr, Sc, fr, fc, post_tw_m, tw, tw_n, st, mask)
  if (S > 0 && F > 0 && Mr >= 1) {
    switch (Mc) {
      case 4: SCAT_MF(4, 1);
      case 8: SCAT_MF(8, 1);
      case 16: SCAT_MF(16, 1);
      case 32: SCAT_MF(16, 2);
      case 64: SCAT_MF(16, 4);
      case 128: SCAT_MF(16, 8);
      case 256: SCAT_MF(16, 16);
      case 512: SCAT_MF(32, 16);
      default: break;
    }
  }
#undef SCAT_MF
  int RB = pow2_floor(kTileElems / Mc);
  if (RB > Mr) RB = Mr;
  if (RB < 1) return hipErrorInvalidValue;
  long blocks = S * F * (Mr / RB);
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  size_t lds = static_cast<size_t>(RB) * Mc * sizeof(float2);
  const double spts = static_cast<double>(S) * Sr * Sc, opts = static_cast<double>(S) * F * Mr * Mc;
  Observe ob("k_mulfold_invrow", spts * 8 + static_cast<double>(F) * Sr * Sc * 4 + opts * 8,
             static_cast<double>(S) * F * Mr * fft_flops(Mc) + 4.0 * spts * F, st);
  hipLaunchKernelGGL(k_mulfold_invrow, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), lds, st,
                     src, filt, dst, F, Sr, Sc, fr, fc, RB, post_tw_m, tw, tw_n);
  return hipGetLastError();
}

bool col_out_tail_supported(int Mr, int Mc, int tw_n) {
  return Mr == 256 && (Mc == 1 || Mc == 2 || Mc == 4 || Mc == 8 || Mc == 16) && tw_n % Mr == 0;
}

hipError_t launch_col_out_tail(const float2 *src, long nodes, long tail_nodes, int Mc, float *out, ChanMap cm, int K,
                               const float2 *tw, int tw_n, hipStream_t st) {
  if (!col_out_tail_supported(256, Mc, tw_n) || out == nullptr || cm.G < 1) return hipErrorInvalidValue;
  return launch_col_out(src, nodes + tail_nodes, Mc, out, cm, K, tw, tw_n, st, nodes);
}

hipError_t launch_col_segs(const float2 *src, float2 *uc, int Mr, const ColSeg *segs, int n, bool uc_half,
                           const float2 *tw, int tw_n, hipStream_t st) {
  return launch_col_segs_impl(src, uc, Mr, segs, n, uc_half, tw, tw_n, st);
}

hipError_t launch_col(int mode, const void *src, long nodes, int Mr, int Mc, float2 *uc,
                      int post_tw_m, const float *phi_rows, int m_r, float *w_out, float *out,
                      ChanMap cm, int K, const float2 *tw, int tw_n, hipStream_t st, bool uc_half) {
  if (uc_half && (mode == 2 || Mr < 2)) return hipErrorInvalidValue;
  // (with the four-step twiddle, half spectra are written by the register kernel only)
  if (uc_half && post_tw_m != 0 &&
      !(mode == 1 && (Mr == 32 || Mr == 64 || Mr == 128 || Mr == 256) && Mc >= 4 && w_out == nullptr &&
        tw_n % Mr == 0 && post_tw_m == Mr * Mc))
    return hipErrorInvalidValue;
  // register-resident variant: modes 0/1, column length 16*T with T | 16, at least 16
  // columns (4 without a lowpass tail), lowpass length dividing the column length
  if (mode == 2 && Mr == 256 && (Mc == 1 || Mc == 2 || Mc == 4 || Mc == 8 || Mc == 16) && tw_n % Mr == 0 &&
      out != nullptr && cm.G >= 1)
    return launch_col_out(static_cast<const float2 *>(src), nodes, Mc, out, cm, K, tw, tw_n, st);
  if (mode != 2 && (Mc >= 16 || (Mc >= 4 && w_out == nullptr)) && tw_n % Mr == 0 &&
      (w_out == nullptr || (m_r >= 1 && m_r <= Mr))) {
    switch (Mr) {
      case 32: return launch_col_fast_t<32>(mode, src, nodes, Mc, uc, uc_half, post_tw_m, phi_rows, m_r, w_out, tw, tw_n, st);
      case 64: return launch_col_fast_t<64>(mode, src, nodes, Mc, uc, uc_half, post_tw_m, phi_rows, m_r, w_out, tw, tw_n, st);
      case 128: return launch_col_fast_t<128>(mode, src, nodes, Mc, uc, uc_half, post_tw_m, phi_rows, m_r, w_out, tw, tw_n, st);
      case 256: return launch_col_fast_t<256>(mode, src, nodes, Mc, uc, uc_half, post_tw_m, phi_rows, m_r, w_out, tw, tw_n, st);
      case 512: return launch_col_fast_t<512>(mode, src, nodes, Mc, uc, uc_half, post_tw_m, phi_rows, m_r, w_out, tw, tw_n, st);
      default: break;
    }
  }
  int TC = pow2_floor(kTileElems / Mr);
  if (TC > 16) TC = 16;
  if (TC > Mc) TC = Mc;
  if (TC < 1) return hipErrorInvalidValue;
  long blocks = nodes * (Mc / TC);
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  size_t lds = (static_cast<size_t>(Mr) + (w_out ? m_r : 0)) * TC * sizeof(float2);
  dim3 g(static_cast<unsigned>(blocks)), b(kThreads);
  static const char *const names[3] = {"k_col<0>", "k_col<1>", "k_col<2>"};
  const double pts = static_cast<double>(nodes) * Mr * Mc;
  const double cols = static_cast<double>(nodes) * Mc;
  Observe ob(names[mode < 0 || mode > 2 ? 0 : mode],
             pts * (mode == 0 ? 4 : 8) + (uc ? (uc_half ? cols * (Mr / 2 + 1) : pts) * 8 : 0) +
                 (w_out ? cols * m_r * 4 : 0) +
                 (mode == 2 ? pts * 4 : 0),
             cols * ((mode == 1 ? 2 : 1) * fft_flops(Mr) + (w_out ? fft_flops(m_r) + 2.0 * Mr : 0)) +
                 (mode == 1 ? 4.0 * pts : 0),
             st);
  switch (mode) {
    case 0:
      hipLaunchKernelGGL(k_col<0>, g, b, lds, st, src, Mr, Mc, TC, uc, static_cast<int>(uc_half), post_tw_m, phi_rows, m_r,
                         w_out, out, cm, K, tw, tw_n);
      break;
    case 1:
      hipLaunchKernelGGL(k_col<1>, g, b, lds, st, src, Mr, Mc, TC, uc, static_cast<int>(uc_half), post_tw_m, phi_rows, m_r,
                         w_out, out, cm, K, tw, tw_n);
      break;
    case 2:
      hipLaunchKernelGGL(k_col<2>, g, b, lds, st, src, Mr, Mc, TC, uc, static_cast<int>(uc_half), post_tw_m, phi_rows, m_r,
                         w_out, out, cm, K, tw, tw_n);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_row_fwd(float2 *data, long rows, int Mc, const float2 *tw, int tw_n,
                          hipStream_t st) {
  switch (Mc) {
    case 16: return launch_row_fwd_reg_t<16, 1>(data, rows, tw, tw_n, st);
    case 32: return launch_row_fwd_reg_t<16, 2>(data, rows, tw, tw_n, st);
    case 64: return launch_row_fwd_reg_t<16, 4>(data, rows, tw, tw_n, st);
    case 128: return launch_row_fwd_reg_t<16, 8>(data, rows, tw, tw_n, st);
    case 256: return launch_row_fwd_reg_t<16, 16>(data, rows, tw, tw_n, st);
    case 512: return launch_row_fwd_reg_t<32, 16>(data, rows, tw, tw_n, st);
    default: break;
  }
  int RB = pow2_floor(kTileElems / Mc);
  while (RB > 1 && rows % RB != 0) RB >>= 1;
  if (RB < 1) return hipErrorInvalidValue;
  long blocks = rows / RB;
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  size_t lds = static_cast<size_t>(RB) * Mc * sizeof(float2);
  Observe ob("k_row_fwd", static_cast<double>(rows) * Mc * 16, static_cast<double>(rows) * fft_flops(Mc), st);
  hipLaunchKernelGGL(k_row_fwd, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), lds, st, data,
                     Mc, RB, tw, tw_n);
  return hipGetLastError();
}

hipError_t launch_row_lowpass(const float *w, long nodes, int m_r, int Mc, int m_c,
                              const float *phi_cols, float *out, ChanMap cm, int K,
                              const float2 *tw, int tw_n, hipStream_t st) {
  if (m_r % 2 == 0 && m_c <= Mc) {
    switch (Mc) {
      case 32: return launch_row_lowpass_fast_t<32>(w, nodes, m_r, m_c, phi_cols, out, cm, K, tw, tw_n, st);
      case 64: return launch_row_lowpass_fast_t<64>(w, nodes, m_r, m_c, phi_cols, out, cm, K, tw, tw_n, st);
      case 128: return launch_row_lowpass_fast_t<128>(w, nodes, m_r, m_c, phi_cols, out, cm, K, tw, tw_n, st);
      case 256: return launch_row_lowpass_fast_t<256>(w, nodes, m_r, m_c, phi_cols, out, cm, K, tw, tw_n, st);
      default: break;
    }
  }
  int RB = pow2_floor(kTileElems / Mc);
  if (RB > m_r) RB = m_r;
  if (RB < 1) return hipErrorInvalidValue;
  long blocks = nodes * (m_r / RB);
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  size_t lds = static_cast<size_t>(RB) * (Mc + m_c) * sizeof(float2);
  const double rws = static_cast<double>(nodes) * m_r;
  Observe ob("k_row_lowpass", rws * (Mc + m_c) * 4, rws * (fft_flops(Mc) + fft_flops(m_c) + 2.0 * Mc), st);
  hipLaunchKernelGGL(k_row_lowpass, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), lds, st, w,
                     m_r, Mc, m_c, RB, phi_cols, out, cm, K, tw, tw_n);
  return hipGetLastError();
}


bool col_node_supported(int Mr, int Mc, int m_r, int m_c, int tw_n) {
  return col_node_supported_impl(Mr, Mc, m_r, m_c, tw_n);
}

bool leaf_node_supported(int Mr, int Mc, int m_r, int m_c, int tw_n) {
  return leaf_node_supported_impl(Mr, Mc, m_r, m_c, tw_n);
}

hipError_t launch_leaf_node(const float2 *src, long nodes, int Mr, int m, const float *phi_rows,
                            const float *phi_cols, float *out, ChanMap cm, int K, const float2 *tw,
                            int tw_n, hipStream_t st) {
  if (nodes <= 0) return hipSuccess;
  if (!leaf_node_supported_impl(Mr, Mr, m, m, tw_n) || nodes > 0x7fffffffL || cm.G < 1 ||
      cm.inner < 1 || nodes % cm.G != 0)
    return hipErrorInvalidValue;
  const size_t lds = (static_cast<size_t>(64) * 64 + 64) * sizeof(float2);
  const double pts = static_cast<double>(nodes) * 64 * 64;
  Observe ob("k_leaf_node<64, 32>", pts * 8 + static_cast<double>(nodes) * 32 * 32 * 4,
             static_cast<double>(nodes) * (2.0 * 64 * fft_flops(64) + 64 * fft_flops(32) +
                                           16 * (fft_flops(64) + fft_flops(32))) + 8.0 * pts,
             st);
  hipLaunchKernelGGL((k_leaf_node<64, 32>), dim3(static_cast<unsigned>(nodes)), dim3(256), lds, st, src,
                     phi_rows, phi_cols, out, cm, K, tw, tw_n);
  return hipGetLastError();
}

hipError_t launch_col_node(int mode, const void *src, long nodes, int Mr, int m, float2 *uc,
                           bool uc_half, const float *phi_rows, const float *phi_cols, float *out,
                           ChanMap cm, int K, const float2 *tw, int tw_n, hipStream_t st) {
  if (!col_node_supported_impl(Mr, Mr, m, m, tw_n) || (mode != 0 && mode != 1)) return hipErrorInvalidValue;
#define SCAT_CN(MR_, LM_) \
  return launch_col_node_t<MR_, LM_>(mode, src, nodes, uc, uc_half, phi_rows, phi_cols, out, cm, K, tw, tw_n, st)
  if (m == 32) {
    switch (Mr) {
      case 128: SCAT_CN(128, 32);
      case 256: SCAT_CN(256, 32);
      default: break;
    }
  } else {
    if (Mr == 128) SCAT_CN(128, 8);
  }
#undef SCAT_CN
  return hipErrorInvalidValue;
}

bool rows_fused_supported(int Sr, int Sc, int fmax) {
  if (Sc != 32 && Sc != 64 && Sc != 128 && Sc != 256) return false;
  if (fmax < 0 || fmax > 3) return false;
  if ((Sc >> fmax) < 16) return false;
  if ((Sr >> fmax) < 1) return false;
  // a wave transforms 64 / (Sc / 16) rows at a time and owns whole groups of 2^fmax rows:
  // the source needs a whole number of such row sets (thin images take the pass path)
  const int rpw = 64 / (Sc / 16), g = 1 << fmax, rows_w = rpw > g ? rpw : g;
  if (Sr < rows_w || Sr % rows_w != 0) return false;
  return true;
}

hipError_t launch_rows_fused(const float2 *src, bool src_half, long NS, int Sr, int Sc,
                             const FusedLevel *levels, int nlev, const float2 *tw, int tw_n,
                             hipStream_t st) {
  if (nlev < 1 || nlev > 4) return hipErrorInvalidValue;
  int fmax = 0;
  FusedArgsDev args;
  args.nlev = nlev;
  for (int l = 0; l < nlev; ++l) {
    args.lv[l].f = levels[l].f;
    args.lv[l].F = levels[l].F;
    args.lv[l].filt = levels[l].filt;
    args.lv[l].dst = levels[l].dst;
    if (levels[l].f > fmax) fmax = levels[l].f;
  }
  if (!rows_fused_supported(Sr, Sc, fmax)) return hipErrorInvalidValue;
  const int G = 1 << fmax;
  const int T = Sc / 16;
  const int RPW = 64 / T;
  const int rows_w = RPW > G ? RPW : G;
  const int NGRP = rows_w / G;
  const int groups = Sr / G;
  if (groups % NGRP != 0) return hipErrorInvalidValue;
  // per-wave product/exchange area: phase 1 needs RPW transforms of 16*(T+1), a level
  // with TP lanes per transform needs (64/TP) slots of 16*(TP+1) (16 if TP == 1)
  size_t b_words = static_cast<size_t>(RPW) * fused_slot_stride(16, T);
  for (int l = 0; l < nlev; ++l) {
    const int M = Sc >> levels[l].f;
    const int EL = fused_el(M), TP = M / EL;
    size_t need = static_cast<size_t>(64 / TP) * fused_slot_stride(EL, TP);
    if (need > b_words) b_words = need;
  }
  size_t lds = (Sc + 4 * (static_cast<size_t>(rows_w) * fused_row_stride(Sc) + b_words)) * sizeof(float2);
  if (lds > 160 * 1024) return hipErrorInvalidValue;
  long blocks = ((NS + 3) / 4) * (groups / NGRP);
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  dim3 g(static_cast<unsigned>(blocks)), b(256);
  const double spts = static_cast<double>(NS) * Sr * Sc;
  double bytes = static_cast<double>(NS) * (src_half ? Sr / 2 + 1 : Sr) * Sc * 8;
  double flops = static_cast<double>(NS) * Sr * fft_flops(Sc);
  for (int l = 0; l < nlev; ++l) {
    const int f = levels[l].f, F = levels[l].F;
    const double opts = static_cast<double>(NS) * F * (Sr >> f) * (Sc >> f);
    bytes += opts * 8 + static_cast<double>(F) * Sr * Sc * 4;
    flops += static_cast<double>(NS) * F * (Sr >> f) * fft_flops(Sc >> f) + 4.0 * spts * F;
  }
  int mask = 0;
  for (int l = 0; l < nlev; ++l) mask |= 1 << levels[l].f;
  const int hf = static_cast<int>(src_half), bw = static_cast<int>(b_words);
  const bool known_mask = mask == 1 || mask == 2 || mask == 3 || mask == 4 || mask == 6 ||
                          mask == 7 || mask == 8 || mask == 12 || mask == 14;
  const std::string name = "k_rows_fused<" + std::to_string(Sc) + ", " +
                           std::to_string(known_mask ? mask : 15) + ">";
  Observe ob(name.c_str(), bytes, flops, st);
  // one instantiation per (row length, set of fold levels); workgroups may use more than
  // the default 64 KB of LDS, which has to be allowed once per kernel
#define SCAT_RF_LAUNCH(SC_, MASK_)                                                                \
  {                                                                                               \
    static unsigned long long lds_ok = 0;                                                         \
    {                                                                                             \
      hipError_t e =                                                                              \
          allow_large_lds(reinterpret_cast<const void *>(k_rows_fused<SC_, MASK_>), lds_ok);      \
      if (e != hipSuccess) return e;                                                              \
    }                                                                                             \
    hipLaunchKernelGGL((k_rows_fused<SC_, MASK_>), g, b, lds, st, src, hf, NS, Sr, G, bw, args,   \
                       tw, tw_n);                                                                 \
  }
#define SCAT_RF_MASKS(SC_)                                    \
  switch (mask) {                                             \
    case 1: SCAT_RF_LAUNCH(SC_, 1) break;                     \
    case 2: SCAT_RF_LAUNCH(SC_, 2) break;                     \
    case 3: SCAT_RF_LAUNCH(SC_, 3) break;                     \
    case 4: SCAT_RF_LAUNCH(SC_, 4) break;                     \
    case 6: SCAT_RF_LAUNCH(SC_, 6) break;                     \
    case 7: SCAT_RF_LAUNCH(SC_, 7) break;                     \
    case 8: SCAT_RF_LAUNCH(SC_, 8) break;                     \
    case 12: SCAT_RF_LAUNCH(SC_, 12) break;                   \
    case 14: SCAT_RF_LAUNCH(SC_, 14) break;                   \
    default: SCAT_RF_LAUNCH(SC_, 15) break;                   \
  }
  switch (Sc) {
    case 32: SCAT_RF_MASKS(32) break;
    case 64: SCAT_RF_MASKS(64) break;
    case 128: SCAT_RF_MASKS(128) break;
    case 256: SCAT_RF_MASKS(256) break;
    default: return hipErrorInvalidValue;
  }
#undef SCAT_RF_MASKS
#undef SCAT_RF_LAUNCH
  return hipGetLastError();
}

}  // namespace scat
