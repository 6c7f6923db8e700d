// Two-dimensional transforms of small planes ("slabs" of N1 x N2 points, at most 16384)
// held by one workgroup: 16 points per thread in registers, rows and columns each by the
// register transform of fft_regs.hpp, one transpose through LDS between them.  Used by the
// slab kernels of the 3-D cascade and by the node kernel of the 2-D backward pass.
#pragma once

#include <hip/hip_runtime.h>

#include "fft_regs.hpp"

namespace scat {

// row stride of a slab in LDS: room for the row exchange of fft_core (16 (T2 + 1) elements)
// plus a skew that spreads the rows of one wavefront over the banks
__host__ __device__ constexpr int slab_row_stride(int N2) {
  return N2 == 16 ? 17 : N2 == 256 ? N2 + 48 : N2 + 16 + N2 / 16;
}

template <int N1, int N2>
struct Slab {
  static constexpr int T1 = N1 / 16, T2 = N2 / 16;
  static constexpr int TS = N1 * N2 / 16;       // threads per slab, 16 points each
  static constexpr int NT = TS < 256 ? 256 : TS;  // threads per workgroup
  static constexpr int SPW = NT / TS;           // slabs per workgroup
  static constexpr int RS = slab_row_stride(N2);
  static constexpr size_t lds_bytes = static_cast<size_t>(SPW) * N1 * RS * sizeof(float2);
  static_assert(N1 >= 16 && N2 >= 16 && TS <= 1024 && TS >= 16 &&
                    lds_bytes + (N1 + N2) * sizeof(float2) <= 160 * 1024,
                "slab shape");

  // v: this thread's 16 points of row r (columns t + T2 i) -> after the call its 16 points
  // of column c (rows t1 + T1 i) of the slab transformed along both axes.  The twiddles are
  // fetched right before each transform so that they are not live across the whole kernel.
  // (WAVE: the slab's threads are the lanes of one wavefront, TS <= 64, and synchronise among
  // themselves only)
  template <bool INV, bool WAVE = false>
  static __device__ __forceinline__ void transform(float2 (&v)[16], float2 *area, int r, int t, int c,
                                                   int t1, const float2 *__restrict__ tw, int tw_n) {
    {
      float2 wr[16];
      load_twiddles<16, T2>(wr, t, tw, tw_n);
      fft_core<16, T2, INV, WAVE>(v, t, area + r * RS, T2 + 1, 1, wr);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) area[r * RS + t + T2 * i] = v[i];
    group_sync<WAVE>();
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = area[(t1 + T1 * i) * RS + c];
    group_sync<WAVE>();
    float2 wc[16];
    load_twiddles<16, T1>(wc, t1, tw, tw_n);
    fft_core<16, T1, INV, WAVE>(v, t1, area + c, T1 * RS, RS, wc);
  }

  // The way back: v holds 16 points of column c (rows t1 + T1 i); after the call the thread's
  // 16 points of row r (columns t + T2 i) of the slab transformed along both axes.
  template <bool INV>
  static __device__ __forceinline__ void transform_back(float2 (&v)[16], float2 *area, int r, int t,
                                                        int c, int t1, const float2 *__restrict__ tw,
                                                        int tw_n) {
    {
      float2 wc[16];
      load_twiddles<16, T1>(wc, t1, tw, tw_n);
      fft_core<16, T1, INV, false>(v, t1, area + c, T1 * RS, RS, wc);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) area[(t1 + T1 * i) * RS + c] = v[i];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = area[r * RS + t + T2 * i];
    __syncthreads();
    float2 wr[16];
    load_twiddles<16, T2>(wr, t, tw, tw_n);
    fft_core<16, T2, INV, false>(v, t, area + r * RS, T2 + 1, 1, wr);
  }
  // The same two transforms with the threads' twiddles in LDS tables instead of registers
  // (for kernels short of registers): wtr[k T2 + t] = exp(-2 pi i t k / N2), k < 16, t < T2,
  // and wtc[k T1 + t1] likewise for N1; fill_twiddles writes both (tab_elems entries at
  // `tab`, barrier included unless the caller declines it).
  static constexpr int tab_elems = N1 + N2;
  static __device__ __forceinline__ void fill_twiddles(float2 *tab, const float2 *__restrict__ tw,
                                                       int tw_n, bool sync = true) {
    for (int idx = threadIdx.x; idx < N2; idx += blockDim.x)
      tab[idx] = tw[(idx / T2) * (idx % T2) * (tw_n / N2)];
    for (int idx = threadIdx.x; idx < N1; idx += blockDim.x)
      tab[N2 + idx] = tw[(idx / T1) * (idx % T1) * (tw_n / N1)];
    if (sync) __syncthreads();  // (else: the caller has a barrier of its own before the first use)
  }
  template <bool INV>
  static __device__ __forceinline__ void transform_tab(float2 (&v)[16], float2 *area, int r, int t,
                                                       int c, int t1, const float2 *tab) {
    fft_core_tab<16, T2, INV, false>(v, t, area + r * RS, T2 + 1, 1, tab + t, T2);
#pragma unroll
    for (int i = 0; i < 16; ++i) area[r * RS + t + T2 * i] = v[i];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = area[(t1 + T1 * i) * RS + c];
    __syncthreads();
    fft_core_tab<16, T1, INV, false>(v, t1, area + c, T1 * RS, RS, tab + N2 + t1, T1);
  }
  template <bool INV>
  static __device__ __forceinline__ void transform_back_tab(float2 (&v)[16], float2 *area, int r,
                                                            int t, int c, int t1, const float2 *tab) {
    fft_core_tab<16, T1, INV, false>(v, t1, area + c, T1 * RS, RS, tab + N2 + t1, T1);
#pragma unroll
    for (int i = 0; i < 16; ++i) area[(t1 + T1 * i) * RS + c] = v[i];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = area[r * RS + t + T2 * i];
    __syncthreads();
    fft_core_tab<16, T2, INV, false>(v, t, area + r * RS, T2 + 1, 1, tab + t, T2);
  }
};


}  // namespace scat
