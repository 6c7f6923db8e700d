// Register-resident FFT building blocks for gfx950.
//
// A transform of N = E * T points is shared by T threads, each holding E points in
// registers: thread t holds x[t + T*i] in v[i].  One radix-E butterfly in registers, a
// twiddle multiply, one exchange through LDS, and E/T radix-T butterflies leave thread t
// holding X[t + T*i] in v[i] -- the same layout, so transforms chain without reshuffling.
// Sign convention: forward = exp(-2 pi i k n / N); INV = true conjugates every twiddle
// (no 1/N scaling anywhere).
#pragma once

#include <hip/hip_runtime.h>

namespace scat {

__device__ __forceinline__ float2 c_mul(float2 a, float2 b) {
  return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ float2 c_add(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 c_sub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }
// multiply by -i (forward quarter turn) or +i (inverse)
template <bool INV>
__device__ __forceinline__ float2 c_rot(float2 a) {
  return INV ? make_float2(-a.y, a.x) : make_float2(a.y, -a.x);
}
// multiply by the constant (wr, wi) with wi given for the forward direction
template <bool INV>
__device__ __forceinline__ float2 c_mulc(float2 a, float wr, float wi) {
  const float s = INV ? -wi : wi;
  return make_float2(a.x * wr - a.y * s, a.x * s + a.y * wr);
}

// g / sqrt(m2), the factor of the modulus adjoint; 0 where m2 = 0.  The hardware root does not
// take denormal inputs (it would return 0 and the quotient would be infinite), so a tiny m2 is
// first scaled into the normal range by an exact power of two.
__device__ __forceinline__ float over_sqrt(float g, float m2) {
  if (!(m2 > 0.f)) return 0.f;
  const bool tiny = m2 < 1.0e-30f;
  const float r = g / __builtin_amdgcn_sqrtf(tiny ? m2 * 0x1p+64f : m2);
  return tiny ? r * 0x1p+32f : r;
}

template <bool INV>
__device__ __forceinline__ void dft4(float2 &x0, float2 &x1, float2 &x2, float2 &x3) {
  float2 t0 = c_add(x0, x2), t1 = c_sub(x0, x2), t2 = c_add(x1, x3), t3 = c_rot<INV>(c_sub(x1, x3));
  x0 = c_add(t0, t2);
  x2 = c_sub(t0, t2);
  x1 = c_add(t1, t3);
  x3 = c_sub(t1, t3);
}

template <int E, bool INV>
struct DftRegs;

template <bool INV>
struct DftRegs<1, INV> {
  static __device__ __forceinline__ void run(float2 (&)[1]) {}
};

template <bool INV>
struct DftRegs<2, INV> {
  static __device__ __forceinline__ void run(float2 (&v)[2]) {
    float2 a = v[0], b = v[1];
    v[0] = c_add(a, b);
    v[1] = c_sub(a, b);
  }
};

template <bool INV>
struct DftRegs<4, INV> {
  static __device__ __forceinline__ void run(float2 (&v)[4]) { dft4<INV>(v[0], v[1], v[2], v[3]); }
};

template <bool INV>
struct DftRegs<8, INV> {
  // index i = 2a + b, frequency k = c + 4d
  static __device__ __forceinline__ void run(float2 (&v)[8]) {
    constexpr float h = 0.70710678118654752440f;
    dft4<INV>(v[0], v[2], v[4], v[6]);  // b = 0: results Y[0][c] at v[2c]
    dft4<INV>(v[1], v[3], v[5], v[7]);  // b = 1: results Y[1][c] at v[2c+1]
    v[3] = c_mulc<INV>(v[3], h, -h);
    v[5] = c_rot<INV>(v[5]);
    v[7] = c_mulc<INV>(v[7], -h, -h);
    float2 o[8];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      o[c] = c_add(v[2 * c], v[2 * c + 1]);
      o[c + 4] = c_sub(v[2 * c], v[2 * c + 1]);
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = o[k];
  }
};

template <bool INV>
struct DftRegs<16, INV> {
  // index i = 4a + b, frequency k = c + 4d
  static __device__ __forceinline__ void run(float2 (&v)[16]) {
    constexpr float h = 0.70710678118654752440f;
    constexpr float c1 = 0.92387953251128675613f;  // cos(pi/8)
    constexpr float s1 = 0.38268343236508977173f;  // sin(pi/8)
#pragma unroll
    for (int b = 0; b < 4; ++b) dft4<INV>(v[b], v[4 + b], v[8 + b], v[12 + b]);  // Y[b][c] at v[4c+b]
    // twiddles w16^(b*c)
    v[4 * 1 + 1] = c_mulc<INV>(v[4 * 1 + 1], c1, -s1);  // w^1
    v[4 * 1 + 2] = c_mulc<INV>(v[4 * 1 + 2], h, -h);    // w^2
    v[4 * 1 + 3] = c_mulc<INV>(v[4 * 1 + 3], s1, -c1);  // w^3
    v[4 * 2 + 1] = c_mulc<INV>(v[4 * 2 + 1], h, -h);    // w^2
    v[4 * 2 + 2] = c_rot<INV>(v[4 * 2 + 2]);            // w^4
    v[4 * 2 + 3] = c_mulc<INV>(v[4 * 2 + 3], -h, -h);   // w^6
    v[4 * 3 + 1] = c_mulc<INV>(v[4 * 3 + 1], s1, -c1);  // w^3
    v[4 * 3 + 2] = c_mulc<INV>(v[4 * 3 + 2], -h, -h);   // w^6
    v[4 * 3 + 3] = c_mulc<INV>(v[4 * 3 + 3], -c1, s1);  // w^9
    float2 o[16];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      dft4<INV>(v[4 * c], v[4 * c + 1], v[4 * c + 2], v[4 * c + 3]);  // X[c + 4d] at v[4c+d]
#pragma unroll
      for (int d = 0; d < 4; ++d) o[c + 4 * d] = v[4 * c + d];
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = o[k];
  }
};

template <bool INV>
struct DftRegs<32, INV> {
  // even and odd samples as two 16-point transforms: X[k] = E[k] + w32^k O[k],
  // X[k + 16] = E[k] - w32^k O[k]
  static __device__ __forceinline__ void run(float2 (&v)[32]) {
    constexpr float C[16] = {1.00000000000000000000f, 0.98078528040323043058f, 0.92387953251128673848f, 0.83146961230254523567f, 0.70710678118654757274f, 0.55557023301960228867f, 0.38268343236508983729f, 0.19509032201612833135f, 0.00000000000000006123f, -0.19509032201612819257f, -0.38268343236508972627f, -0.55557023301960195560f, -0.70710678118654746172f, -0.83146961230254534669f, -0.92387953251128673848f, -0.98078528040323043058f};
    constexpr float S[16] = {0.00000000000000000000f, 0.19509032201612824808f, 0.38268343236508978178f, 0.55557023301960217765f, 0.70710678118654746172f, 0.83146961230254523567f, 0.92387953251128673848f, 0.98078528040323043058f, 1.00000000000000000000f, 0.98078528040323043058f, 0.92387953251128673848f, 0.83146961230254545772f, 0.70710678118654757274f, 0.55557023301960217765f, 0.38268343236508989280f, 0.19509032201612860891f};
    float2 e[16], o[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      e[i] = v[2 * i];
      o[i] = v[2 * i + 1];
    }
    DftRegs<16, INV>::run(e);
    DftRegs<16, INV>::run(o);
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const float2 t = k == 0 ? o[0] : c_mulc<INV>(o[k], C[k], -S[k]);
      v[k] = c_add(e[k], t);
      v[k + 16] = c_sub(e[k], t);
    }
  }
};

// Twiddles of thread t for an N = E*T point transform: wt[k1] = exp(-2 pi i t k1 / N),
// taken from the table tw[j] = exp(-2 pi i j / tw_n) (N divides tw_n).
template <int E, int T>
__device__ __forceinline__ void load_twiddles(float2 (&wt)[E], int t, const float2 *__restrict__ tw,
                                              int tw_n) {
  const int step = tw_n / (E * T);
#pragma unroll
  for (int k1 = 0; k1 < E; ++k1) wt[k1] = tw[t * k1 * step];
}

// Orders LDS accesses of the lanes of one wavefront: everything written before is visible
// to every lane after.  (LDS operations of one wave complete in issue order; the fences
// keep the compiler from moving accesses across.)
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <bool WAVE>
__device__ __forceinline__ void group_sync() {
  if (WAVE)
    wave_sync();
  else
    __syncthreads();
}

// The transform described at the top of this file.  xch points at this transform's
// exchange area in LDS, already offset for anything but (k1, t): element (k1, t) lives at
// xch[k1 * sk + t * st].  When T > 1 it synchronises twice (before the exchange buffer is
// read, and after): with WAVE = false by workgroup barriers, so every thread of the
// workgroup must call it; with WAVE = true only within the wavefront, which requires the T
// threads of a transform to be lanes of one wave.
template <int E, int T, bool INV, bool WAVE = false>
__device__ __forceinline__ void fft_core(float2 (&v)[E], int t, float2 *xch, int sk, int st,
                                         const float2 (&wt)[E]) {
  DftRegs<E, INV>::run(v);
  if (T == 1) return;
#pragma unroll
  for (int k1 = 1; k1 < E; ++k1) {
    float2 w = wt[k1];
    if (INV) w.y = -w.y;
    v[k1] = c_mul(v[k1], w);
  }
#pragma unroll
  for (int k1 = 0; k1 < E; ++k1) xch[k1 * sk + t * st] = v[k1];
  group_sync<WAVE>();
  constexpr int U = E / T;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float2 a[T];
    const int k1 = t + T * u;
#pragma unroll
    for (int j = 0; j < T; ++j) a[j] = xch[k1 * sk + j * st];
    DftRegs<T, INV>::run(a);
#pragma unroll
    for (int k2 = 0; k2 < T; ++k2) v[u + U * k2] = a[k2];
  }
  group_sync<WAVE>();
}

// fft_core with the E twiddles of this thread read at their point of use from wl[k * ws]
// (a table in LDS) instead of held in registers across the first stage: for kernels that
// run several transforms and are short of registers.
template <int E, int T, bool INV, bool WAVE = false>
__device__ __forceinline__ void fft_core_tab(float2 (&v)[E], int t, float2 *xch, int sk, int st,
                                             const float2 *wl, int ws) {
  DftRegs<E, INV>::run(v);
  if (T == 1) return;
#pragma unroll
  for (int k1 = 1; k1 < E; ++k1) {
    float2 w = wl[k1 * ws];
    if (INV) w.y = -w.y;
    v[k1] = c_mul(v[k1], w);
  }
#pragma unroll
  for (int k1 = 0; k1 < E; ++k1) xch[k1 * sk + t * st] = v[k1];
  group_sync<WAVE>();
  constexpr int U = E / T;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float2 a[T];
    const int k1 = t + T * u;
#pragma unroll
    for (int j = 0; j < T; ++j) a[j] = xch[k1 * sk + j * st];
    DftRegs<T, INV>::run(a);
#pragma unroll
    for (int k2 = 0; k2 < T; ++k2) v[u + U * k2] = a[k2];
  }
  group_sync<WAVE>();
}

}  // namespace scat
