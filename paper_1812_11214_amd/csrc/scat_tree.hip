// Depth-first scattering of small planes entirely in LDS (32 x 32, J = 2).
//
// Paper section 2 ("Implementation") walks the scattering tree depth first so that a
// first-order modulus is dropped as soon as its children are done.  For planes this small
// the whole subtree of one first-order node fits in the LDS share of ONE wavefront, so a
// wave takes the spectrum of x, and produces S1 of its node and S2 of all its children
// without any intermediate going to memory:
//
//   node (j1 = 0, theta1), 32 x 32:
//     Y = X^ . psi^            -> inverse FFT along columns, then rows -> |.| -> forward
//     FFT along rows, lowpass along columns (fold 32 -> 8, inverse 8-point) -> lowpass
//     along rows -> S1;  forward FFT along columns gives U^ (kept in LDS)
//   its children (j2 = 1, theta2), 16 x 16, four at a time (16 lanes each):
//     fold(U^ . psi^) -> inverse 2-D FFT -> |.| -> forward + lowpass -> S2
//   nodes of octave j1 = 1 (16 x 16, no children at J = 2): as the children, from X^.
//
// A 32-point transform is shared by two neighbouring lanes (16 points each) that swap
// halves with a DPP lane permute; 16- and 8-point transforms live in one lane.  Lanes only
// ever meet lanes of their own wavefront, so the kernel has no workgroup barrier.
#include <hip/hip_runtime.h>

#include <string>

#include "fft_regs.hpp"
#include "scat_kernels.hpp"

namespace scat {

namespace {

// value of the other lane of the pair (lanes 2k and 2k+1)
__device__ __forceinline__ float pair_swap(float x) {
  // DPP quad_perm [1, 0, 3, 2]
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, true));
}
__device__ __forceinline__ float2 pair_swap(float2 a) {
  return make_float2(pair_swap(a.x), pair_swap(a.y));
}
__device__ __forceinline__ float2 sel(bool c, float2 a, float2 b) { return c ? a : b; }

// Twiddles of a lane for the 32-point lane-pair transform: w[k1] = exp(-2 pi i tp k1 / 32)
// (all ones in the even lane), and the sign bit that negates a float in the odd lane.
struct PairTw {
  float2 w[16];
  unsigned flip;
};
__device__ __forceinline__ void pair_twiddles(PairTw &pw, int tp) {
  // cos and sin of 2 pi k / 32
  constexpr float C[16] = {1.f,
                           0.98078528040323044913f,
                           0.92387953251128675613f,
                           0.83146961230254523708f,
                           0.70710678118654752440f,
                           0.55557023301960222474f,
                           0.38268343236508977173f,
                           0.19509032201612826785f,
                           0.f,
                           -0.19509032201612826785f,
                           -0.38268343236508977173f,
                           -0.55557023301960222474f,
                           -0.70710678118654752440f,
                           -0.83146961230254523708f,
                           -0.92387953251128675613f,
                           -0.98078528040323044913f};
  constexpr float S[16] = {0.f,
                           0.19509032201612826785f,
                           0.38268343236508977173f,
                           0.55557023301960222474f,
                           0.70710678118654752440f,
                           0.83146961230254523708f,
                           0.92387953251128675613f,
                           0.98078528040323044913f,
                           1.f,
                           0.98078528040323044913f,
                           0.92387953251128675613f,
                           0.83146961230254523708f,
                           0.70710678118654752440f,
                           0.55557023301960222474f,
                           0.38268343236508977173f,
                           0.19509032201612826785f};
  const bool odd = tp != 0;
#pragma unroll
  for (int k = 0; k < 16; ++k) pw.w[k] = make_float2(odd ? C[k] : 1.f, odd ? -S[k] : 0.f);
  pw.flip = odd ? 0x80000000u : 0u;
}
__device__ __forceinline__ float flip_sign(float x, unsigned flip) {
  return __uint_as_float(__float_as_uint(x) ^ flip);
}

// 32-point transform over a lane pair: lane tp (0 or 1) holds x[tp + 2 i] in v[i] and ends
// with X[tp + 2 i] in v[i].  Radix 16 in registers, twiddle w32^(tp k1), then the radix-2
// butterflies between the two lanes: lane tp keeps the k1 = tp + 2 j it owns, receives the
// partner's value for the same k1 and forms sum and difference (the difference is
// even-lane minus odd-lane value, hence the sign flip in the odd lane).
template <bool INV>
__device__ __forceinline__ void fft32_pair(float2 (&v)[16], int tp, const PairTw &pw) {
  DftRegs<16, INV>::run(v);
  const bool odd = tp != 0;
#pragma unroll
  for (int k1 = 1; k1 < 16; ++k1) {
    const float2 w = pw.w[k1];
    // multiply by w (forward) or its conjugate (inverse)
    v[k1] = INV ? make_float2(v[k1].x * w.x + v[k1].y * w.y, v[k1].y * w.x - v[k1].x * w.y)
                : make_float2(v[k1].x * w.x - v[k1].y * w.y, v[k1].y * w.x + v[k1].x * w.y);
  }
  float2 o[16];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float2 mine = sel(odd, v[2 * j + 1], v[2 * j]);
    const float2 send = sel(odd, v[2 * j], v[2 * j + 1]);
    const float2 recv = pair_swap(send);
    o[j] = c_add(mine, recv);
    const float2 d = c_sub(mine, recv);
    o[j + 8] = make_float2(flip_sign(d.x, pw.flip), flip_sign(d.y, pw.flip));
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = o[i];
}

// Inverse 8-point transform over a lane pair: lane tp holds F[tp + 2 j] in f[j] and ends
// with y[tp + 2 j] in f[j] (unnormalised).
__device__ __forceinline__ void idft8_pair(float2 (&f)[4], int tp) {
  constexpr float h = 0.70710678118654752440f;
  DftRegs<4, true>::run(f);
  const bool odd = tp != 0;
  float2 y[4];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const float2 mine = sel(odd, f[2 * u + 1], f[2 * u]);
    const float2 send = sel(odd, f[2 * u], f[2 * u + 1]);
    const float2 recv = pair_swap(send);
    const float2 b0 = sel(odd, recv, mine), b1 = sel(odd, mine, recv);
    // b1 times exp(+2 pi i (tp + 2u) / 8)
    float2 t;
    if (u == 0)
      t = sel(odd, make_float2(h * (b1.x - b1.y), h * (b1.x + b1.y)), b1);
    else
      t = sel(odd, make_float2(-h * (b1.x + b1.y), h * (b1.x - b1.y)), make_float2(-b1.y, b1.x));
    y[u] = c_add(b0, t);
    y[u + 2] = c_sub(b0, t);
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) f[j] = y[j];
}

__device__ __forceinline__ float2 modulus(float2 a) {
  return make_float2(__builtin_amdgcn_sqrtf(a.x * a.x + a.y * a.y), 0.f);
}

constexpr int P1_STRIDE = 33;                   // 32 x 32 plane, padded rows
constexpr int P1_ELEMS = 32 * P1_STRIDE;        // float2
constexpr int P2_STRIDE = 17;                   // 16 x 16 plane, padded rows
constexpr int P2_PLANE = 16 * P2_STRIDE;        // float2
constexpr int P2_ELEMS = 4 * P2_PLANE;          // four small nodes at a time
constexpr int WL_FLOATS = 512;                  // half-lowpassed planes (32 x 9 or 4 x 16 x 8)
constexpr int WAVE_LDS_BYTES = (P1_ELEMS + P2_ELEMS) * 8 + WL_FLOATS * 4;
constexpr int TREE_WAVES = 4;

struct TreeArgs {
  const float2 *xh;
  long planes;
  int L, max_order, K;
  const float *psi_j0, *psi_j1;
  const float *phi_cols0, *phi_cols1;  // lowpass along a row, Fourier samples (32 and 16)
  const float *taps0, *taps1;          // lowpass along a column, spatial taps (32 and 16)
  float *out;
};

// Four 16 x 16 nodes at once, 16 lanes each (lane c of a group owns column c, later row
// c): node g of the batch is filtered by psi_j1[first + g] out of the 32 x 32 spectrum
// `src` (fold 2 on both axes) and its lowpass goes to channel chan0 + g.  SRC_LDS: src is
// the wave's P1 plane (row stride P1_STRIDE), else global memory (row stride 32).
// tp1[r] = taps1[(2 n - r) mod 16] for this lane's output row n = (lane % 16) / 2.
template <bool SRC_LDS>
__device__ __forceinline__ void small_nodes(const TreeArgs &a, const float2 *src, int first,
                                            int chan0, float2 *P2, float *Wl, float *out,
                                            int lane, const float (&tp1)[16]) {
  const int g = lane >> 4, c = lane & 15;
  const bool live = first + g < a.L;
  const int th = live ? first + g : a.L - 1;
  const float *ps = a.psi_j1 + static_cast<size_t>(th) * 1024;
  constexpr int SS = SRC_LDS ? P1_STRIDE : 32;
  float2 v[16];
  // Y[q_r][c] = sum over the four aliases of src . psi, then inverse along q_r
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    float2 acc = make_float2(0.f, 0.f);
#pragma unroll
    for (int aa = 0; aa < 2; ++aa)
#pragma unroll
      for (int bb = 0; bb < 2; ++bb) {
        const int r = i + 16 * aa, cc = c + 16 * bb;
        const float f = ps[r * 32 + cc];
        const float2 u = src[r * SS + cc];
        acc.x += u.x * f;
        acc.y += u.y * f;
      }
    v[i] = acc;
  }
  DftRegs<16, true>::run(v);
  float2 *pl = P2 + g * P2_PLANE;
#pragma unroll
  for (int i = 0; i < 16; ++i) pl[i * P2_STRIDE + c] = v[i];
  wave_sync();
  // rows: inverse, modulus, forward, lowpass along the row (fold 16 -> 8)
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = pl[c * P2_STRIDE + i];
  DftRegs<16, true>::run(v);
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = modulus(v[i]);
  DftRegs<16, false>::run(v);
  float2 f8[8];
#pragma unroll
  for (int m = 0; m < 8; ++m) {
    const float p0 = a.phi_cols1[m], p1 = a.phi_cols1[m + 8];
    f8[m] = make_float2(v[m].x * p0 + v[m + 8].x * p1, v[m].y * p0 + v[m + 8].y * p1);
  }
  DftRegs<8, true>::run(f8);
  float *wl = Wl + g * 128;  // [row 16][col 8], real
#pragma unroll
  for (int n = 0; n < 8; ++n) wl[c * 8 + n] = f8[n].x;
  wave_sync();
  // lowpass along the columns of that 16 x 8 plane, straight from its definition: output
  // row n is the circular correlation with the spatial taps at stride 2.  Lane c forms the
  // four outputs (n = c / 2, columns 4 (c % 2) ...).
  {
    const int n = c >> 1, c4 = 4 * (c & 1);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float t = tp1[r];
      const float4 w = *reinterpret_cast<const float4 *>(wl + r * 8 + c4);
      acc.x += t * w.x;
      acc.y += t * w.y;
      acc.z += t * w.z;
      acc.w += t * w.w;
    }
    if (live) *reinterpret_cast<float4 *>(out + static_cast<size_t>(chan0 + g) * 64 + n * 8 + c4) = acc;
  }
  wave_sync();  // P2 and Wl are free again
}

__device__ __forceinline__ void load_taps1(float (&tp1)[16], const float *taps1, int lane) {
  const int n = (lane & 15) >> 1;
#pragma unroll
  for (int r = 0; r < 16; ++r) tp1[r] = taps1[(2 * n - r) & 15];
}

// One first-order node of octave 0 with all its children.
__device__ __forceinline__ void node_octave0(const TreeArgs &a, const float2 *xh, int th1,
                                             float2 *P1, float2 *P2, float *Wl, float *out,
                                             int lane) {
  const int tp = lane & 1, q = lane >> 1;
  const bool kids = a.max_order == 2;
  const float *ps = a.psi_j0 + static_cast<size_t>(th1) * 1024;
  PairTw pw;
  pair_twiddles(pw, tp);
  float2 v[16];
  // columns: lane pair q owns column q, rows tp + 2 i
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int r = tp + 2 * i;
    const float2 x = xh[r * 32 + q];
    const float f = ps[r * 32 + q];
    v[i] = make_float2(x.x * f, x.y * f);
  }
  fft32_pair<true>(v, tp, pw);
#pragma unroll
  for (int i = 0; i < 16; ++i) P1[(tp + 2 * i) * P1_STRIDE + q] = v[i];
  wave_sync();
  // rows: lane pair q owns row q
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = P1[q * P1_STRIDE + tp + 2 * i];
  fft32_pair<true>(v, tp, pw);
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = modulus(v[i]);
  fft32_pair<false>(v, tp, pw);
  if (kids) {
#pragma unroll
    for (int i = 0; i < 16; ++i) P1[q * P1_STRIDE + tp + 2 * i] = v[i];
  }
  float2 f4[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) f4[j] = make_float2(0.f, 0.f);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const float p = a.phi_cols0[tp + 2 * i];
    f4[i & 3].x += v[i].x * p;
    f4[i & 3].y += v[i].y * p;
  }
  idft8_pair(f4, tp);
#pragma unroll
  for (int j = 0; j < 4; ++j) Wl[q * 9 + tp + 2 * j] = f4[j].x;  // [row 32][col 8], stride 9
  wave_sync();
  // S1: lowpass along the columns of that 32 x 8 plane from its definition (circular
  // correlation with the spatial taps at stride 4), one output sample per lane
  {
    const int n = lane >> 3, nc = lane & 7;
    float acc = 0.f;
#pragma unroll
    for (int r = 0; r < 32; ++r) acc += a.taps0[(4 * n - r) & 31] * Wl[r * 9 + nc];
    out[static_cast<size_t>(1 + th1) * 64 + lane] = acc;
  }
  if (!kids) return;
  // columns of the row spectra: P1 becomes the 2-D spectrum of the modulus
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = P1[(tp + 2 * i) * P1_STRIDE + q];
  fft32_pair<false>(v, tp, pw);
#pragma unroll
  for (int i = 0; i < 16; ++i) P1[(tp + 2 * i) * P1_STRIDE + q] = v[i];
  wave_sync();
  const int chan0 = 1 + 2 * a.L + th1 * a.L;
  float tp1[16];
  load_taps1(tp1, a.taps1, lane);
  for (int first = 0; first < a.L; first += 4)
    small_nodes<true>(a, P1, first, chan0 + first, P2, Wl, out, lane, tp1);
}

// Spectrum and S0 of the inputs: one wavefront per plane.  Rows first (so that the
// row-lowpassed plane is still spatial along the columns for the tap correlation), then
// columns; writes xh [32][32] and channel 0 of the output.
constexpr int INPUT_WAVE_LDS_BYTES = P1_ELEMS * 8 + 32 * 9 * 4;
__global__ __launch_bounds__(64 * TREE_WAVES) void k_tree32_input(const float *__restrict__ x,
                                                                  long planes, float2 *xh,
                                                                  TreeArgs a) {
  extern __shared__ float2 smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
  const long p = static_cast<long>(blockIdx.x) * TREE_WAVES + wave;
  if (p >= planes) return;
  float2 *P1 = smem + static_cast<size_t>(wave) * (INPUT_WAVE_LDS_BYTES / 8);
  float *Wl = reinterpret_cast<float *>(P1 + P1_ELEMS);
  const int tp = lane & 1, q = lane >> 1;
  PairTw pw;
  pair_twiddles(pw, tp);
  const float *xp = x + p * 1024;
  float2 v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = make_float2(xp[q * 32 + tp + 2 * i], 0.f);
  fft32_pair<false>(v, tp, pw);
#pragma unroll
  for (int i = 0; i < 16; ++i) P1[q * P1_STRIDE + tp + 2 * i] = v[i];
  float2 f4[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) f4[j] = make_float2(0.f, 0.f);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const float ph = a.phi_cols0[tp + 2 * i];
    f4[i & 3].x += v[i].x * ph;
    f4[i & 3].y += v[i].y * ph;
  }
  idft8_pair(f4, tp);
#pragma unroll
  for (int j = 0; j < 4; ++j) Wl[q * 9 + tp + 2 * j] = f4[j].x;
  wave_sync();
  {
    const int n = lane >> 3, nc = lane & 7;
    float acc = 0.f;
#pragma unroll
    for (int r = 0; r < 32; ++r) acc += a.taps0[(4 * n - r) & 31] * Wl[r * 9 + nc];
    a.out[p * a.K * 64 + lane] = acc;
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = P1[(tp + 2 * i) * P1_STRIDE + q];
  fft32_pair<false>(v, tp, pw);
  float2 *xo = xh + p * 1024;
#pragma unroll
  for (int i = 0; i < 16; ++i) xo[(tp + 2 * i) * 32 + q] = v[i];
}

__global__ __launch_bounds__(64 * TREE_WAVES) void k_tree32(TreeArgs a) {
  extern __shared__ float2 smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
  const int groups1 = (a.L + 3) / 4;
  const int per_plane = a.L + groups1;
  const long w = static_cast<long>(blockIdx.x) * TREE_WAVES + wave;
  if (w >= a.planes * per_plane) return;  // whole waves leave; nothing below syncs across waves
  const long p = w / per_plane;
  const int it = static_cast<int>(w - p * per_plane);
  float2 *P1 = smem + static_cast<size_t>(wave) * (WAVE_LDS_BYTES / 8);
  float2 *P2 = P1 + P1_ELEMS;
  float *Wl = reinterpret_cast<float *>(P2 + P2_ELEMS);
  const float2 *xh = a.xh + p * 1024;
  float *out = a.out + p * a.K * 64;
  if (it < a.L)
    node_octave0(a, xh, it, P1, P2, Wl, out, lane);
  else {
    float tp1[16];
    load_taps1(tp1, a.taps1, lane);
    small_nodes<false>(a, xh, 4 * (it - a.L), 1 + a.L + 4 * (it - a.L), P2, Wl, out, lane, tp1);
  }
}

}  // namespace

bool tree_supported(int n_r, int n_c, int J) { return n_r == 32 && n_c == 32 && J == 2; }

hipError_t launch_tree32_input(const float *x, long planes, float2 *xh, const float *phi_cols0,
                               const float *taps0, float *out, int K, hipStream_t st) {
  if (planes <= 0) return hipSuccess;
  const long blocks = (planes + TREE_WAVES - 1) / TREE_WAVES;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  TreeArgs a{xh, planes, 0, 1, K, nullptr, nullptr, phi_cols0, nullptr, taps0, nullptr, out};
  const double bytes = planes * (1024.0 * 4 + 1024.0 * 8 + 64.0 * 4);
  const double flops = planes * 64.0 * 5.0 * 32 * 5;
  LaunchScope obs("k_tree32_input", bytes, flops, st);
  hipLaunchKernelGGL(k_tree32_input, dim3(static_cast<unsigned>(blocks)), dim3(64 * TREE_WAVES),
                     static_cast<size_t>(INPUT_WAVE_LDS_BYTES) * TREE_WAVES, st, x, planes, xh, a);
  return hipGetLastError();
}

hipError_t launch_tree32(const float2 *xh, long planes, int L, int max_order, const float *psi_j0,
                         const float *psi_j1, const float *phi_cols0, const float *phi_cols1,
                         const float *taps0, const float *taps1, float *out, int K,
                         hipStream_t st) {
  if (planes <= 0) return hipSuccess;
  if (L < 1 || (max_order != 1 && max_order != 2)) return hipErrorInvalidValue;
  const long per_plane = L + (L + 3) / 4;
  const long waves = planes * per_plane;
  const long blocks = (waves + TREE_WAVES - 1) / TREE_WAVES;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  const size_t lds = static_cast<size_t>(WAVE_LDS_BYTES) * TREE_WAVES;
  static unsigned long long lds_ok = 0;
  {
    hipError_t e = allow_large_lds(reinterpret_cast<const void *>(k_tree32), lds_ok);
    if (e != hipSuccess) return e;
  }
  TreeArgs a{xh, planes, L, max_order, K, psi_j0, psi_j1, phi_cols0, phi_cols1, taps0, taps1, out};
  // least traffic: spectra in, S1 and S2 out, the 2 L wavelet tables once
  const double kids = max_order == 2 ? static_cast<double>(L) * L : 0.0;
  const double bytes = planes * (1024.0 * 8 + (2.0 * L + kids) * 64 * 4) + 2.0 * L * 1024 * 4;
  auto fl = [](double n) { return 5.0 * n * (n == 32 ? 5.0 : n == 16 ? 4.0 : 3.0); };
  // per octave-0 node: 32 x (2 inverse + 2 forward) 32-point transforms (3 without
  // children); per 16 x 16 node: 16 x 3 transforms of 16 points; lowpass transforms are
  // small and left out; 4 flops per filter multiply-accumulate and per modulus
  const double node0 = 32 * (kids > 0 ? 4 : 3) * fl(32) + 4.0 * 1024 * 2;
  const double small = 48 * fl(16) + 4.0 * (1024 + 256);
  const double flops = planes * (L * node0 + (L + kids) * small);
  LaunchScope obs("k_tree32", bytes, flops, st);
  hipLaunchKernelGGL(k_tree32, dim3(static_cast<unsigned>(blocks)), dim3(64 * TREE_WAVES), lds, st,
                     a);
  return hipGetLastError();
}

}  // namespace scat
