// Depth-first 2-D cascade: one workgroup computes one whole node of the scattering tree in LDS.
//
// A node is |x (*) psi| (or ||x (*) psi_1| (*) psi_2|) on its own subsampled grid of M x M
// points, M = 64 (k_node, 256 threads, four workgroups per compute unit) or 128 (k_node_half,
// 512 threads, two per compute unit) (paper, section 2 "Implementation": convolutions as
// Fourier products, every filtered signal downsampled, the tree walked branch by branch so
// that intermediates are dropped as soon as the children are done).  The workgroup
//   1. forms the node's spectrum  Z[k] = sum over sources q and aliases a of
//      src_q[k + M a] * filt_q[k + M a]   (filter product + periodisation = subsampling),
//      reading its parent's spectrum through the caches,
//   2. inverse 2-D transform in registers + LDS, 3. modulus,
//   4. lowpass phi_J and subsampling to the 32 x 32 output grid as a separable FIR filter with
//      the spatial taps of phi (5 sigma each side), straight to the output coefficients,
//   5. (nodes with children only) forward 2-D transform of the modulus, stored as the
//      non-redundant half spectrum for the children.
// Only the input's spectrum, the spectra of first-order moduli that have children, and the
// output coefficients ever go to memory.
//
// Nodes of 2M x 2M points (the first octave of a 256 x 256 image) do not fit the LDS of a
// compute unit; they are split into their four polyphase components u_p[m] = u[2m + p],
// p in {0,1}^2, each an M x M node of its own (POLY):
//   y_p = IFFT_M( conj(w^(p.k)) sum_a (-1)^(a.p) Y[k + M a] ),  w = exp(-2 pi i / 2M),
// and since U[k + M a] = sum_p (-1)^(a.p) w^(p.k) U_p[k], the children read the four stored
// spectra w^(p.k) U_p[k] as four sources with the sign-folded filter tables
// R_p[k] = sum_a (-1)^(a.p) psi[k + M a]  (P = 4).  Each component adds its part of the
// lowpassed output (taps phi[2d - p]); k_sum4 adds the four parts.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <string>
#include <type_traits>

#include "fft_regs.hpp"
#include "slab_fft.hpp"
#include "scat_kernels.hpp"

namespace scat {

namespace {

constexpr int kOut = 32;  // side of the output grid the FIR stage is laid out for

double fft2_flops(double n) { return n > 1 ? 10.0 * n * n * std::log2(n) : 0.0; }

struct NodeArgs {
  const float2 *src;    // [NS][P][S/2+1][S] half spectra, S = M * A (FULL: [NS][S][S], all rows)
  const float *filt;    // [F][P][S][S] real tables (carry the 1/N^2 of the inverse transforms)
  const unsigned long long *mask;  // null, or per filter: bit (q A + ar) A + ac clear = that M x M
                                   // block of table q is negligible everywhere and is skipped
  const unsigned *lane_mask;  // null, or per filter one word per thread (loaders with a source
                              // twice the node's size): which of the thread's loads meet a table
                              // value that is not negligible; the others are left out
  const float *taps_r;  // lowpass taps along a column (row index varies): [2R+1], POLY: [2][2R+1]
  const float *taps_c;  // along a row
  float2 *uout;         // null, or [(NS*I)][M/2+1][M]: half spectrum of every node's modulus
  float *out;           // [planes][K][32][32], POLY: the parts [(NS*I)][32][32]
  long NS;              // sources
  int F;                // filters per source; items per source I = F (POLY: 4 F, component fastest)
  int G;                // sources per plane
  int chan_base, chan_src, chan_f;  // channel = base + (source % G) * chan_src + filter * chan_f
  int K;
  const float2 *tw;     // exp(-2 pi i j / tw_n)
  int tw_n;
};

// Workgroup b serves source 8 (b / 8 / I) + b % 8 and item (b / 8) % I: workgroups are dealt
// to the eight XCDs in turn, so all items of one source run on one XCD, one after the other,
// and its L2 holds the source's spectrum for them.
// The P component values of table entry idx (entries of P floats, side by side)
template <int P>
__device__ __forceinline__ void load_comps(float (&d)[P], const float *tab, int idx) {
  if constexpr (P == 4) {
    const float4 v = reinterpret_cast<const float4 *>(tab)[idx];
    d[0] = v.x;
    d[1] = v.y;
    d[2] = v.z;
    d[3] = v.w;
  } else {
    static_assert(P == 1, "components");
    d[0] = tab[idx];
  }
}

// NF = 2: one workgroup of 512 threads computes the nodes of TWO filters of one source (the
// children of a polyphase parent, which are bound by their loads): the spectrum phase is shared
// -- every source value is loaded once for both -- and each half of the workgroup then takes
// one node through the other phases in an LDS area of its own.
template <int M, int A, int P, bool POLY, bool FULL, int NF>
__device__ __forceinline__ void node_body(const NodeArgs &a) {
  static_assert(!FULL || P == 1, "a full spectrum is one source");
  static_assert(M == 64, "128 x 128 nodes take k_node_half");
  static_assert(NF == 1 || (NF == 2 && A == 2 && P == 4 && !POLY && !FULL), "pairs: four-component loader only");
  using SL = Slab<M, M>;
  // Row slots of 76 elements (rows 24 banks apart: conflict-free for the lanes of eight rows)
  // with an unpadded row exchange (16 x T elements): 39 KB per workgroup, FOUR workgroups per
  // compute unit.
  constexpr int NT = M * M / 16, T = M / 16, S = M * A, RS = 76, SK = T;
  static_assert(RS >= M && RS >= 16 * SK, "row slot holds a row and its exchange");
  constexpr int DEC = M / kOut, R = 4 * DEC, NTAP = 2 * R + 1;
  static_assert(P == 1 || P == 4, "sources");
  static_assert(!POLY || P == 1, "a polyphase node reads a plain spectrum");
  extern __shared__ __attribute__((aligned(16))) float2 lds[];
  // (pairs: thread role `tid` and LDS area of the half-workgroup that owns one of the two nodes)
  const int half = NF == 2 ? static_cast<int>(threadIdx.x) / NT : 0;
  float2 *area = lds + half * (M * RS);
  float2 *wtab = lds + NF * M * RS;
  const int tid = NF == 2 ? static_cast<int>(threadIdx.x) % NT : static_cast<int>(threadIdx.x);
  const int I = a.F * (POLY ? 4 : 1) / NF;
  const long bq = blockIdx.x >> 3;
  const long s = (blockIdx.x & 7) + 8 * (bq / I);
  const int item = static_cast<int>(bq % I);
  if (s >= a.NS) return;
  const int f = POLY ? item >> 2 : item * NF + half;
  const int pr = POLY ? (item >> 1) & 1 : 0, pc = POLY ? item & 1 : 0;
  // (no barrier here: the table is first read after the barrier that ends the spectrum phase,
  // and the workgroup's loads start without waiting for the twiddle fetch)
  SL::fill_twiddles(wtab, a.tw, a.tw_n, false);
  const int tw_step = a.tw_n / (2 * M);  // POLY only: table step of w = exp(-2 pi i / 2M)

  if constexpr (NF == 2) {
    // ---- 1 for two filters at once: as below, with 16 row groups (thread = rows st + 16 i,
    // i < 4) and every source value used for the tables of both filters f0 and f0 + 1.
    const int ltid = threadIdx.x;
    const int f0 = item * 2;
    const float4 *src4 = reinterpret_cast<const float4 *>(a.src + static_cast<size_t>(s) * P * 65 * S);
    const float *ft0 = a.filt + static_cast<size_t>(f0) * P * S * S;
    const int cq = ltid & 31, st = ltid >> 5;
    float2 z2[2][4][2];
    unsigned am[2];
    int zero_e[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      am[c] = a.lane_mask != nullptr ? a.lane_mask[static_cast<size_t>(f0 + c) * (2 * NT) + ltid] : ~0u;
      zero_e[c] = (a.F - f0 - c) * S * S;  // from table f0 + c to the zeros behind the F tables
    }
    auto pick = [](bool on, int idx, int other) { return on ? idx : other; };
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = st + 16 * i;
      const bool first = i == 0 && st == 0;
      const int row2 = first ? 64 : S - row;
      const unsigned b0 = am[0] >> (4 * i), b1 = am[1] >> (4 * i);
      float4 w[2][P];
#pragma unroll
      for (int ac = 0; ac < 2; ++ac) {
        const bool any_d = ((b0 | b1) >> ac) & 1u, any_m = ((b0 | b1) >> (2 + ac)) & 1u;
        const int wc = pick(any_d || (any_m && !first), 32 * ac + cq, 0);
#pragma unroll
        for (int q = 0; q < P; ++q) w[ac][q] = src4[(q * 65 + row) * (S / 2) + wc];
      }
      // Per filter: direct part (table row `row`) and second part (mirrored, table row S - row).
      // Row 0 is special: its second part is row 64 itself, not a mirrored row, so in the first
      // pass the lanes of row 0 fetch row 64 between the direct parts and the second parts of
      // the two filters.
      auto load_tab = [&](float (&tv)[2][2][P], int c, bool mirrored) {
        const float *ft = ft0 + static_cast<size_t>(c) * P * S * S;
        const unsigned bits = (c == 0 ? b0 : b1) >> (mirrored ? 2 : 0);
#pragma unroll
        for (int ac = 0; ac < 2; ++ac) {
          const bool on = (bits >> ac) & 1u;
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const int idx = first ? 32 * ac + cq : (64 - 32 * ac - cq - e) & 63;
            const int entry = mirrored ? ((row2 * 2 + (idx >> 5)) * 2 + e) * 32 + (idx & 31)
                                       : ((row * 2 + ac) * 2 + e) * 32 + cq;
            load_comps<P>(tv[ac][e], ft, pick(on, entry, zero_e[c]));
          }
        }
      };
      auto direct_part = [&](const float (&d)[2][2][P], int c) {
        float4 zd = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int ac = 0; ac < 2; ++ac)
#pragma unroll
          for (int q = 0; q < P; ++q) {
            zd.x = fmaf(w[ac][q].x, d[ac][0][q], zd.x);
            zd.y = fmaf(w[ac][q].y, d[ac][0][q], zd.y);
            zd.z = fmaf(w[ac][q].z, d[ac][1][q], zd.z);
            zd.w = fmaf(w[ac][q].w, d[ac][1][q], zd.w);
          }
        *reinterpret_cast<float4 *>(lds + c * (M * RS) + row * RS + 2 * cq) = zd;
      };
      auto second_part = [&](float (&m)[2][2][P], int c) {
        float4 zs = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int ac = 0; ac < 2; ++ac) {
          // s = (1, sc, -1, -sc), sc = -1 except for column 0
          const float sc0 = first ? 1.f : (ac == 0 && cq == 0) ? 1.f : -1.f;
          const float sc1 = first ? 1.f : -1.f;
          const float sn = first ? 1.f : -1.f;
          m[ac][0][1] *= sc0;
          m[ac][0][2] *= sn;
          m[ac][0][3] *= sn * sc0;
          m[ac][1][1] *= sc1;
          m[ac][1][2] *= sn;
          m[ac][1][3] *= sn * sc1;
#pragma unroll
          for (int q = 0; q < P; ++q) {
            zs.x = fmaf(w[ac][q].x, m[ac][0][q], zs.x);
            zs.y = fmaf(w[ac][q].y, m[ac][0][q], zs.y);
            zs.z = fmaf(w[ac][q].z, m[ac][1][q], zs.z);
            zs.w = fmaf(w[ac][q].w, m[ac][1][q], zs.w);
          }
        }
        const float cj = first ? 1.f : -1.f;
        z2[c][i][0] = make_float2(zs.x, cj * zs.y);
        z2[c][i][1] = make_float2(zs.z, cj * zs.w);
      };
      if (i == 0) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          float d[2][2][P];
          load_tab(d, c, false);
          direct_part(d, c);
        }
        if (first) {
#pragma unroll
          for (int ac = 0; ac < 2; ++ac) {
            const int wc = pick(((b0 | b1) >> (2 + ac)) & 1u, 32 * ac + cq, 0);
#pragma unroll
            for (int q = 0; q < P; ++q) w[ac][q] = src4[(q * 65 + 64) * (S / 2) + wc];
          }
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          float m[2][2][P];
          load_tab(m, c, true);
          second_part(m, c);
        }
      } else {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          float d[2][2][P], m[2][2][P];
          load_tab(d, c, false);
          load_tab(m, c, true);
          direct_part(d, c);
          second_part(m, c);
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = st + 16 * i;
        const bool first = row == 0;
        float2 *tr = lds + c * (M * RS) + (first ? 0 : M - row) * RS;
        const int c0 = first ? 2 * cq : (M - 2 * cq) & (M - 1), c1 = first ? 2 * cq + 1 : M - 1 - 2 * cq;
        float2 o0 = tr[c0], o1 = tr[c1];
        tr[c0] = make_float2(o0.x + z2[c][i][0].x, o0.y + z2[c][i][0].y);
        tr[c1] = make_float2(o1.x + z2[c][i][1].x, o1.y + z2[c][i][1].y);
      }
  } else if constexpr (A == 2 && !FULL) {
    // ---- 1 (source twice as large as the node). Every stored source row (0 .. 64, 128 columns)
    // is read once, by half a wavefront: a lane takes two adjacent columns of both column
    // blocks and of all P components (16-byte loads).  Row rho contributes to row rho of the
    // node directly and, through the conjugate symmetry of the stored spectra
    // W_q[128 - rho][-c] = s_q(c) conj(W_q[rho][c]) (s_q = 1 for a plain spectrum), to row
    // 64 - rho (the alias row 128 - rho); rows 0 and 64, which mirror onto themselves, both
    // fold onto row 0.  The direct parts are written to LDS first, the second parts are added
    // after a barrier.  Filter table: [row][column block][column parity][column pair][component].
    static_assert(!POLY, "polyphase nodes are 128 x 128");
    const float4 *src4 = reinterpret_cast<const float4 *>(a.src + static_cast<size_t>(s) * P * 65 * S);
    const float *ft = a.filt + static_cast<size_t>(f) * P * S * S;
    const int cq = tid & 31, st = tid >> 5;
    float2 z2[8][2];
    // Per-lane activity bits of row i (bits 4 i ..): column block 0 and 1 of the direct part,
    // then of the mirrored part.  Where all table values a load would fetch are negligible
    // (below 1e-7 of the table's peak: about half of a wavelet two octaves above the grid) the
    // lane reads the all-zero entry behind the last table instead, and a source value that only
    // meets such table values is replaced by the first one of its row: the lanes that have
    // nothing to fetch share one address, and no branch is needed.
    // (one component: the kernel is bound by its arithmetic and the selects cost more than the
    // loads they save -- measured; every load is made)
    const unsigned am = (P == 4 && a.lane_mask != nullptr) ? a.lane_mask[static_cast<size_t>(f) * NT + tid] : ~0u;
    const int zero_e = (a.F - f) * S * S;  // entry (of P floats) of the zeros behind the F tables
    auto pick = [](bool on, int idx, int other) { return on ? idx : other; };
    if constexpr (P == 4) {
      // (four components: a row's sixteen 16-byte loads at once; measured faster than the
      // pipelined form below, which is the faster one for a single component)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int row = st + 8 * i;
        const bool first = row == 0;
        const int row2 = first ? 64 : S - row;
        const unsigned bits = am >> (4 * i);
        float4 w[2][P];
        float d[2][2][P], m[2][2][P];
#pragma unroll
        for (int ac = 0; ac < 2; ++ac) {
          const bool on_d = (bits >> ac) & 1u, on_m = (bits >> (2 + ac)) & 1u;
          const int wc = pick(on_d || (on_m && !first), 32 * ac + cq, 0);
#pragma unroll
          for (int q = 0; q < P; ++q) w[ac][q] = src4[(q * 65 + row) * (S / 2) + wc];
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const int idx = first ? 32 * ac + cq : (64 - 32 * ac - cq - e) & 63;
            load_comps<P>(d[ac][e], ft, pick(on_d, ((row * 2 + ac) * 2 + e) * 32 + cq, zero_e));
            load_comps<P>(m[ac][e], ft, pick(on_m, ((row2 * 2 + (idx >> 5)) * 2 + e) * 32 + (idx & 31), zero_e));
          }
        }
        float4 zd = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int ac = 0; ac < 2; ++ac)
#pragma unroll
          for (int q = 0; q < P; ++q) {
            zd.x = fmaf(w[ac][q].x, d[ac][0][q], zd.x);
            zd.y = fmaf(w[ac][q].y, d[ac][0][q], zd.y);
            zd.z = fmaf(w[ac][q].z, d[ac][1][q], zd.z);
            zd.w = fmaf(w[ac][q].w, d[ac][1][q], zd.w);
          }
        *reinterpret_cast<float4 *>(area + row * RS + 2 * cq) = zd;
        if (first) {
#pragma unroll
          for (int ac = 0; ac < 2; ++ac)
#pragma unroll
            for (int q = 0; q < P; ++q)
              w[ac][q] = src4[(q * 65 + 64) * (S / 2) + pick((bits >> (2 + ac)) & 1u, 32 * ac + cq, 0)];
        }
        float4 zs = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int ac = 0; ac < 2; ++ac) {
          if constexpr (P == 4) {
            // s = (1, sc, -1, -sc), sc = -1 except for column 0
            const float sc0 = first ? 1.f : (ac == 0 && cq == 0) ? 1.f : -1.f;
            const float sc1 = first ? 1.f : -1.f;
            const float sn = first ? 1.f : -1.f;
            m[ac][0][1] *= sc0;
            m[ac][0][2] *= sn;
            m[ac][0][3] *= sn * sc0;
            m[ac][1][1] *= sc1;
            m[ac][1][2] *= sn;
            m[ac][1][3] *= sn * sc1;
          }
#pragma unroll
          for (int q = 0; q < P; ++q) {
            zs.x = fmaf(w[ac][q].x, m[ac][0][q], zs.x);
            zs.y = fmaf(w[ac][q].y, m[ac][0][q], zs.y);
            zs.z = fmaf(w[ac][q].z, m[ac][1][q], zs.z);
            zs.w = fmaf(w[ac][q].w, m[ac][1][q], zs.w);
          }
        }
        const float cj = first ? 1.f : -1.f;
        z2[i][0] = make_float2(zs.x, cj * zs.y);
        z2[i][1] = make_float2(zs.z, cj * zs.w);
      }
    } else {
      // One unit of work = one column block (ac) of one source row; the loads of the next units
      // are issued before the arithmetic of the current one (left to itself the compiler waits
      // for each row's loads before it issues the next row's).
      struct Unit {
        float4 w[P];
        float d[2][P], m[2][P];
      };
      constexpr int DEPTH = P == 4 ? 2 : 4;  // units in flight
      auto load_unit = [&](Unit &un, int u) {
        const int i = u >> 1, ac = u & 1;
        const int row = st + 8 * i;
        const bool first = row == 0;
        const int row2 = first ? 64 : S - row;
        const unsigned bits = am >> (4 * i);
        const bool on_d = (bits >> ac) & 1u, on_m = (bits >> (2 + ac)) & 1u;
        const int wc = pick(on_d || (on_m && !first), 32 * ac + cq, 0);
#pragma unroll
        for (int q = 0; q < P; ++q) un.w[q] = src4[(q * 65 + row) * (S / 2) + wc];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int idx = first ? 32 * ac + cq : (64 - 32 * ac - cq - e) & 63;
          load_comps<P>(un.d[e], ft, pick(on_d, ((row * 2 + ac) * 2 + e) * 32 + cq, zero_e));
          load_comps<P>(un.m[e], ft, pick(on_m, ((row2 * 2 + (idx >> 5)) * 2 + e) * 32 + (idx & 31), zero_e));
        }
      };
      Unit buf[DEPTH];
#pragma unroll
      for (int u = 0; u < DEPTH - 1; ++u) load_unit(buf[u], u);
      float4 zd, zs;
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int i = u >> 1, ac = u & 1;
        const int row = st + 8 * i;
        const bool first = row == 0;
        if (u + DEPTH - 1 < 16) load_unit(buf[(u + DEPTH - 1) % DEPTH], u + DEPTH - 1);
        Unit &un = buf[u % DEPTH];
        if (ac == 0) zd = zs = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int q = 0; q < P; ++q) {
          zd.x = fmaf(un.w[q].x, un.d[0][q], zd.x);
          zd.y = fmaf(un.w[q].y, un.d[0][q], zd.y);
          zd.z = fmaf(un.w[q].z, un.d[1][q], zd.z);
          zd.w = fmaf(un.w[q].w, un.d[1][q], zd.w);
        }
        if (first) {  // row 0: its second part is row 64 itself, not a mirrored row
#pragma unroll
          for (int q = 0; q < P; ++q)
            un.w[q] = src4[(q * 65 + 64) * (S / 2) + pick((am >> (2 + ac)) & 1u, 32 * ac + cq, 0)];
        }
        if constexpr (P == 4) {
          // s = (1, sc, -1, -sc), sc = -1 except for column 0
          const float sc0 = first ? 1.f : (ac == 0 && cq == 0) ? 1.f : -1.f;
          const float sc1 = first ? 1.f : -1.f;
          const float sn = first ? 1.f : -1.f;
          un.m[0][1] *= sc0;
          un.m[0][2] *= sn;
          un.m[0][3] *= sn * sc0;
          un.m[1][1] *= sc1;
          un.m[1][2] *= sn;
          un.m[1][3] *= sn * sc1;
        }
#pragma unroll
        for (int q = 0; q < P; ++q) {
          zs.x = fmaf(un.w[q].x, un.m[0][q], zs.x);
          zs.y = fmaf(un.w[q].y, un.m[0][q], zs.y);
          zs.z = fmaf(un.w[q].z, un.m[1][q], zs.z);
          zs.w = fmaf(un.w[q].w, un.m[1][q], zs.w);
        }
        if (ac == 1) {
          *reinterpret_cast<float4 *>(area + row * RS + 2 * cq) = zd;
          const float cj = first ? 1.f : -1.f;
          z2[i][0] = make_float2(zs.x, cj * zs.y);
          z2[i][1] = make_float2(zs.z, cj * zs.w);
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = st + 8 * i;
      const bool first = row == 0;
      float2 *tr = area + (first ? 0 : M - row) * RS;
      const int c0 = first ? 2 * cq : (M - 2 * cq) & (M - 1), c1 = first ? 2 * cq + 1 : M - 1 - 2 * cq;
      float2 o0 = tr[c0], o1 = tr[c1];
      tr[c0] = make_float2(o0.x + z2[i][0].x, o0.y + z2[i][0].y);
      tr[c1] = make_float2(o1.x + z2[i][1].x, o1.y + z2[i][1].y);
    }
  } else
  // ---- 1. spectrum of the node: thread = one column, rows rg + T i (coalesced reads).
  // Measured: the waves of a workgroup reading neighbouring rows at the same time is what the
  // memory system likes (a wave on 16 consecutive rows of its own is 2-3 times slower), and a
  // branch per term instead of per block serialises the loads (also 2-3 times slower).  One
  // pass of the loop takes one alias block of one source (all 16 rows of the thread: 32 loads
  // in flight); blocks on which the filter is negligible are left out.
  {
    constexpr int SROWS = FULL ? S : S / 2 + 1;  // stored rows of a source
    const float2 *src = a.src + static_cast<size_t>(s) * P * SROWS * S;
    const float *filt = a.filt + static_cast<size_t>(f) * P * S * S;
    // (the row group is the same for all lanes of a wave: kept scalar, so that row addresses are
    // scalar bases with one lane offset)
    const int col = tid % M, rg = __builtin_amdgcn_readfirstlane(tid / M);
    {
      float2 acc[16];
      static_assert(P * A * A <= 64, "one mask word per filter");
      constexpr unsigned long long kAll = P * A * A >= 64 ? ~0ull : (1ull << (P * A * A)) - 1ull;
      unsigned long long rem = (a.mask != nullptr ? a.mask[f] : ~0ull) & kAll;  // workgroup-uniform
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = make_float2(0.f, 0.f);
      while (rem != 0ull) {
        const int bit = __builtin_amdgcn_readfirstlane(__ffsll(static_cast<long long>(rem)) - 1);
        rem &= rem - 1ull;
        const int ac = bit % A, ar = (bit / A) % A, q = bit / (A * A);
        const float2 *sq = src + static_cast<size_t>(q) * SROWS * S;
        const float *fq = filt + static_cast<size_t>(q) * S * S + (M * ar) * S;
        const unsigned kc = static_cast<unsigned>(col + M * ac) & (S - 1);
        const unsigned kcm = (S - kc) & (S - 1);
        // sign of the whole block: polyphase alias sign (-1)^(a.p)
        const float sblk = (POLY && ((ar * pr + ac * pc) & 1)) ? -1.f : 1.f;
        // rows above S/2 are not stored: U[kr][kc] = conj(U[S - kr][-kc]); the stored spectra of
        // polyphase components carry w^(p.k), which gives the mirrored value the extra sign
        // (-1)^(q_r) (-1)^(q_c [kc != 0])
        const float smir = (P == 4 && (((q >> 1) & 1) ^ ((q & 1) & (kc != 0 ? 1 : 0)))) ? -sblk : sblk;
        float2 v[16];
        float fv[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int kr = rg + T * i + M * ar;
          const bool mir = !FULL && kr > S / 2;  // the same for every lane of a wave
          v[i] = (sq + (mir ? S - kr : kr) * S)[mir ? kcm : kc];
          fv[i] = (fq + (rg + T * i) * S)[kc];
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const bool mir = !FULL && rg + T * i + M * ar > S / 2;
          const float fx = fv[i] * (mir ? smir : sblk);
          acc[i].x = fmaf(v[i].x, fx, acc[i].x);
          acc[i].y = fmaf(v[i].y, mir ? -fx : fx, acc[i].y);
        }
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int kr0 = rg + T * i;
        float2 z = acc[i];
        if (POLY) {
          const float2 w = a.tw[((pr * kr0 + pc * col) * tw_step) & (a.tw_n - 1)];
          z = make_float2(z.x * w.x + z.y * w.y, z.y * w.x - z.x * w.y);  // * conj(w)
        }
        area[kr0 * RS + col] = z;
      }
    }
  }
  __syncthreads();

  // ---- 2. inverse transform: row layout in, column layout (rows t1 + T i of column c) out
  const int r = tid / T, t = tid % T;
  const int c = tid % M, t1 = tid / M;
  float2 v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = area[r * RS + t + T * i];
  __syncthreads();
  fft_core_tab<16, T, true, false>(v, t, area + r * RS, SK, 1, wtab + t, T);
#pragma unroll
  for (int i = 0; i < 16; ++i) area[r * RS + t + T * i] = v[i];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = area[(t1 + T * i) * RS + c];
  __syncthreads();
  fft_core_tab<16, T, true, false>(v, t1, area + c, T * RS, RS, wtab + M + t1, T);

  // ---- 3. modulus
  float u[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) u[i] = __builtin_amdgcn_sqrtf(v[i].x * v[i].x + v[i].y * v[i].y);

  // ---- 4. lowpass + subsampling by DEC: rows first (H: along a row), then columns (V)
  constexpr int US = M + 1, HS = kOut + 1;
  float *ub = reinterpret_cast<float *>(area);  // [M][US]
  float *hb = ub + M * US;                      // [M][HS]
#pragma unroll
  for (int i = 0; i < 16; ++i) ub[(t1 + T * i) * US + c] = u[i];
  __syncthreads();
  {
    constexpr int OPT = kOut * M / NT;  // outputs per thread, adjacent columns
    constexpr int NIN = DEC * (OPT - 1) + NTAP;
    const int rr = tid % M, mg = tid / M;
    const float *tc = a.taps_c + (POLY ? pc * NTAP : 0);
    float acc[OPT];
#pragma unroll
    for (int j = 0; j < OPT; ++j) acc[j] = 0.f;
    const int e0 = DEC * OPT * mg - R;
    // e0 is a multiple of 8: within a run of 8 inputs the column index does not wrap, so one
    // address per run and constant offsets inside it (no index arithmetic per read)
    constexpr int SEG = 8, NSEG = (NIN + SEG - 1) / SEG;
    static_assert((DEC * OPT) % SEG == 0 && R % SEG == 0, "runs of inputs that do not wrap");
    const float *seg[NSEG];
#pragma unroll
    for (int k = 0; k < NSEG; ++k) seg[k] = ub + rr * US + ((e0 + SEG * k) & (M - 1));
#pragma unroll
    for (int e = 0; e < NIN; ++e) {
      const float val = seg[e / SEG][e % SEG];
#pragma unroll
      for (int j = 0; j < OPT; ++j) {
        const int ti = DEC * j + 2 * R - e;  // tap index d + R of input column DEC m - d
        if (ti >= 0 && ti <= 2 * R) acc[j] = fmaf(tc[ti], val, acc[j]);
      }
    }
#pragma unroll
    for (int j = 0; j < OPT; ++j) hb[rr * HS + OPT * mg + j] = acc[j];
  }
  __syncthreads();
  {
    constexpr int OPV = kOut * kOut / NT;  // outputs per thread, adjacent rows
    constexpr int NIN = DEC * (OPV - 1) + NTAP;
    const int mc = tid % kOut, ng = tid / kOut;
    const float *tr = a.taps_r + (POLY ? pr * NTAP : 0);
    float acc[OPV];
#pragma unroll
    for (int j = 0; j < OPV; ++j) acc[j] = 0.f;
    const int e0 = DEC * OPV * ng - R;
    constexpr int SEG = 8, NSEG = (NIN + SEG - 1) / SEG;  // e0 is a multiple of 8: see above
    static_assert((DEC * OPV) % SEG == 0 && R % SEG == 0, "runs of inputs that do not wrap");
    const float *seg[NSEG];
#pragma unroll
    for (int k = 0; k < NSEG; ++k) seg[k] = hb + ((e0 + SEG * k) & (M - 1)) * HS + mc;
#pragma unroll
    for (int e = 0; e < NIN; ++e) {
      const float val = seg[e / SEG][(e % SEG) * HS];
#pragma unroll
      for (int j = 0; j < OPV; ++j) {
        const int ti = DEC * j + 2 * R - e;
        if (ti >= 0 && ti <= 2 * R) acc[j] = fmaf(tr[ti], val, acc[j]);
      }
    }
    float *op;
    if (POLY) {
      op = a.out + (static_cast<size_t>(s) * I + item) * kOut * kOut;
    } else {
      const long plane = s / a.G;
      const int g = static_cast<int>(s - plane * a.G);
      op = a.out + (static_cast<size_t>(plane) * a.K + a.chan_base + g * a.chan_src + f * a.chan_f) *
                       kOut * kOut;
    }
#pragma unroll
    for (int j = 0; j < OPV; ++j) __builtin_nontemporal_store(acc[j], op + (OPV * ng + j) * kOut + mc);  // (never read here)
  }
  if (a.uout == nullptr) return;

  // ---- 5. spectrum of the modulus for the children (rows 0 .. M/2)
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = make_float2(u[i], 0.f);
  fft_core_tab<16, T, false, false>(v, t1, area + c, T * RS, RS, wtab + M + t1, T);
#pragma unroll
  for (int i = 0; i < 16; ++i) area[(t1 + T * i) * RS + c] = v[i];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = area[r * RS + t + T * i];
  __syncthreads();
  fft_core_tab<16, T, false, false>(v, t, area + r * RS, SK, 1, wtab + t, T);
  if (r > M / 2) return;
  float2 *up = a.uout + ((static_cast<size_t>(s) * I + item) * (M / 2 + 1) + r) * M + t;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    float2 val = v[i];
    if (POLY) val = c_mul(val, a.tw[((pr * r + pc * (t + T * i)) * tw_step) & (a.tw_n - 1)]);
    up[T * i] = val;
  }
}

template <int M, int A, int P, bool POLY, bool FULL>
__global__ __launch_bounds__(M * M / 16, (P == 4 ? 3 : 4)) void k_node(NodeArgs a) {
  node_body<M, A, P, POLY, FULL, 1>(a);
}

// Two 64 x 64 children of a polyphase parent per workgroup (78 KB of LDS, two workgroups and
// sixteen waves per compute unit)
__global__ __launch_bounds__(512, 4) void k_node_pair(NodeArgs a) { node_body<64, 2, 4, false, false, 2>(a); }

// ------------------------------------------------------------------------------------
// k_node for 128 x 128 nodes with HALF the workgroup: 512 threads hold the node in registers
// (32 points each) and use LDS only to exchange one half of it at a time, 81 KB instead of
// 156 KB, so that TWO workgroups share a compute unit and one's memory and LDS phases run
// under the other's arithmetic (a single resident workgroup adds its phases up: measured).
//   spectrum + row transforms: rows 0..63, then rows 64..127 (thread = row r or r + 64,
//     columns t + 8 i), through the same 64 row slots of 152 elements; the spectrum phase
//     reads every stored source row once for the two node rows it serves (the stored half
//     spectra are conjugate-symmetric), a lane taking two adjacent columns per 16-byte load;
//   transposition: columns 0..63, then 64..127, through 128 rows of 72 elements (rows 16
//     banks apart: no conflicts);
//   column transforms: column c, then c + 64 (thread = rows t1 + 8 i), exchange in place;
//   lowpass as in k_node, with the row-filtered values parked in registers while the
//   unfiltered plane is still being read, then written over it;
//   parents: forward transform of the (real) modulus with the thread's two columns as one
//     complex pair, rows 0..64 only.
// Four waves per SIMD: 128 vector registers (launch bounds).
template <int A, int P, bool POLY, bool FULL>
__global__ __launch_bounds__(512, 4) void k_node_half(NodeArgs a) {
  static_assert(!FULL || P == 1, "a full spectrum is one source");
  constexpr int M = 128, T = 8, NT = 512, S = M * A;
  constexpr int RSR = 152, RSC = 72;
  constexpr int DEC = M / kOut, R = 4 * DEC, NTAP = 2 * R + 1;
  extern __shared__ __attribute__((aligned(16))) float2 lds[];
  float2 *area = lds;             // 64 * RSR elements (128 * RSC fit in them)
  float2 *wtab = lds + 64 * RSR;  // twiddles: [k * T + t] for rows, the same again for columns
  const int tid = threadIdx.x;
  const int I = a.F * (POLY ? 4 : 1);
  const long bq = blockIdx.x >> 3;
  const long s = (blockIdx.x & 7) + 8 * (bq / I);
  const int item = static_cast<int>(bq % I);
  if (s >= a.NS) return;
  const int f = POLY ? item >> 2 : item;
  const int pr = POLY ? (item >> 1) & 1 : 0, pc = POLY ? item & 1 : 0;
  for (int idx = tid; idx < M; idx += NT) wtab[idx] = a.tw[(idx / T) * (idx % T) * (a.tw_n / M)];
  const int tw_step = a.tw_n / (2 * M);
  // polyphase nodes: w^k = exp(-2 pi i k / 2M), k < 2M, behind the transforms' twiddles
  float2 *w2m = wtab + M;
  float2 *row64 = w2m + 2 * M;  // 64 elements: row 64 of the packed column spectra (parents only)
  if (POLY)
    for (int idx = tid; idx < 2 * M; idx += NT) w2m[idx] = a.tw[idx * tw_step];
  const int r = tid / T, t = tid % T;    // row roles: rows r and r + 64, columns t + 8 i
  const int c = tid % 64, t1 = tid / 64; // column roles: columns c and c + 64, rows t1 + 8 i
  const float2 *wl = wtab + t, *wlc = wtab + t1;
  // (no barrier here: the tables are first read after the barriers of the spectrum phase)

  // ---- 1 + 2a. spectrum of the node (half of its rows at a time) and inverse row transforms
  float2 vh[2][16];
  if constexpr (A == 1 && P == 4 && !POLY && !FULL) {
    // Children of a polyphase parent.  Every stored source row r (1 .. 63) is read once and
    // serves two rows of the node: row r directly and row M - r through the conjugate symmetry
    // W_q[M - r][-c] = s_q(c) conj(W_q[r][c]) of the stored spectra (s_q: the sign the phase
    // factor of component q leaves, see the top of this file); rows 0 and 64 mirror onto
    // themselves and are read whole.  A lane takes two adjacent columns of all four
    // components (16-byte loads); the filter table is laid out [row][column parity][column
    // pair][component], so that the four component values of a point are one 16-byte load,
    // contiguous across the wave for the direct and for the mirrored columns alike.
    const float4 *src4 = reinterpret_cast<const float4 *>(a.src + static_cast<size_t>(s) * 4 * 65 * M);
    const float4 *f4 = reinterpret_cast<const float4 *>(a.filt + static_cast<size_t>(f) * 4 * M * M);
    const int cp = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col_m0 = (M - 2 * cp) & (M - 1), col_m1 = M - 1 - 2 * cp;
    float2 zm[8][2];  // second rows (64 .. 127), kept until the first half has been transformed
    // The loads of row i + 1 are issued before the arithmetic of row i (two rows in flight: left
    // to itself the compiler waits for each row's loads before it issues the next row's).
    struct Item {
      float4 w[4], d[2], m[2];
    };
    auto load_item = [&](Item &it, int i) {
      const int row = wv + 8 * i;
      const bool first = i == 0 && wv == 0;  // row 0: its partner is row 64, read directly
      const int row2 = first ? 64 : M - row;
#pragma unroll
      for (int q = 0; q < 4; ++q) it.w[q] = src4[(q * 65 + row) * (M / 2) + cp];
      it.d[0] = f4[(row * 2 + 0) * 64 + cp];
      it.d[1] = f4[(row * 2 + 1) * 64 + cp];
      it.m[0] = f4[(row2 * 2 + 0) * 64 + cp];
      it.m[1] = f4[(row2 * 2 + 1) * 64 + cp];
    };
    Item buf[2];
    float4 w64[4];  // row 64 of the four components (first wave only)
    load_item(buf[0], 0);
    if (wv == 0) {
#pragma unroll
      for (int q = 0; q < 4; ++q) w64[q] = src4[(q * 65 + 64) * (M / 2) + cp];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = wv + 8 * i;
      const bool first = i == 0 && wv == 0;
      if (i + 1 < 8) load_item(buf[(i + 1) & 1], i + 1);
      const Item &it = buf[i & 1];
      const float4 *w = it.w, *d = it.d, *m = it.m;
      float4 zd;  // direct: columns 2 cp (x, y) and 2 cp + 1 (z, w)
      zd.x = w[0].x * d[0].x + w[1].x * d[0].y + w[2].x * d[0].z + w[3].x * d[0].w;
      zd.y = w[0].y * d[0].x + w[1].y * d[0].y + w[2].y * d[0].z + w[3].y * d[0].w;
      zd.z = w[0].z * d[1].x + w[1].z * d[1].y + w[2].z * d[1].z + w[3].z * d[1].w;
      zd.w = w[0].w * d[1].x + w[1].w * d[1].y + w[2].w * d[1].z + w[3].w * d[1].w;
      *reinterpret_cast<float4 *>(area + row * RSR + 2 * cp) = zd;
      // partner row: sum_q conj(w_q) m_q (table rows above 64 are stored for that: at the lane's
      // own place and with the sign s_q), or the plain product for row 64
      float4 w2[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) w2[q] = (i == 0 && first) ? w64[q] : w[q];
      const float cj = first ? 1.f : -1.f;  // mirrored parts are conjugated
      zm[i][0].x = w2[0].x * m[0].x + w2[1].x * m[0].y + w2[2].x * m[0].z + w2[3].x * m[0].w;
      zm[i][0].y = cj * (w2[0].y * m[0].x + w2[1].y * m[0].y + w2[2].y * m[0].z + w2[3].y * m[0].w);
      zm[i][1].x = w2[0].z * m[1].x + w2[1].z * m[1].y + w2[2].z * m[1].z + w2[3].z * m[1].w;
      zm[i][1].y = cj * (w2[0].w * m[1].x + w2[1].w * m[1].y + w2[2].w * m[1].z + w2[3].w * m[1].w);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) vh[0][i] = area[r * RSR + t + T * i];
    __syncthreads();
    fft_core_tab<16, T, true, false>(vh[0], t, area + r * RSR, T + 1, 1, wl, T);  // ends with a barrier
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = wv + 8 * i;
      const bool first = i == 0 && wv == 0;
      const int slot = first ? 0 : 64 - row;  // rows 64 .. 127 go through slots 0 .. 63
      area[slot * RSR + (first ? 2 * cp : col_m0)] = zm[i][0];
      area[slot * RSR + (first ? 2 * cp + 1 : col_m1)] = zm[i][1];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) vh[1][i] = area[r * RSR + t + T * i];
    __syncthreads();
    fft_core_tab<16, T, true, false>(vh[1], t, area + r * RSR, T + 1, 1, wl, T);
  } else if constexpr (A == 2 && P == 1 && !FULL) {
    // Source twice as large as the node (the spectrum of x, or of a 256 x 256 parent).  A wave
    // takes one stored source row (0 .. 128; 256 columns) at a time, a lane two adjacent columns
    // of both column blocks (16-byte loads).  Row rho contributes to row rho of the node
    // directly and, as conj(W[rho][c]) = W[256 - rho][-c], to row 128 - rho (the alias row
    // 256 - rho); rows 0 and 128 both fold onto row 0.  The node's rows go through LDS in two
    // halves: first the direct parts are written, then, after a barrier, the mirrored parts
    // are added (every element by exactly one lane).  So every row of the source is read
    // twice (a row's direct part belongs to one half of the node, its mirrored part to the other).
    const float4 *src4 = reinterpret_cast<const float4 *>(a.src + static_cast<size_t>(s) * (S / 2 + 1) * S);
    const float *ft = a.filt + static_cast<size_t>(f) * S * S;
    const int cp = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c0 = (M - 2 * cp) & (M - 1), c1 = M - 1 - 2 * cp;  // columns of the mirrored parts
    // polyphase alias signs (-1)^(a.p): of the direct parts (row block 0), and of the mirrored
    // parts (row block 1, column block of the mirrored column)
    const float4 *ft4 = reinterpret_cast<const float4 *>(ft);
    const float sg1 = (POLY && pc) ? -1.f : 1.f;
    float sm[2][2];
#pragma unroll
    for (int ac = 0; ac < 2; ++ac)
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int idx = (128 - 64 * ac - cp - e) & 127;  // column pair of the mirrored column
        sm[ac][e] = (POLY && ((pr + (idx >> 6) * pc) & 1)) ? -1.f : 1.f;
      }
    // The filter values of a lane's four points of a row (two columns in each column block) are
    // ONE 16-byte load: (block 0, block 1) x column parity, from table row rho for the direct
    // part and from table row 256 - rho, stored in mirrored order, for the mirrored part.
    auto direct = [&](int row, float sr) {  // row of the source and of the table; sr: sign of its row block
      const float4 w0 = src4[row * (S / 2) + cp], w1 = src4[row * (S / 2) + 64 + cp];
      const float4 f = ft4[row * 64 + cp];
      const float d00 = f.x * sr, d01 = f.y * sr, d10 = f.z * (sr * sg1), d11 = f.w * (sr * sg1);
      return make_float4(w0.x * d00 + w1.x * d10, w0.y * d00 + w1.y * d10, w0.z * d01 + w1.z * d11,
                         w0.w * d01 + w1.w * d11);
    };
    auto mirrored = [&](int row) {  // conj of the products with table row 256 - row, mirrored columns
      const float4 w0 = src4[row * (S / 2) + cp], w1 = src4[row * (S / 2) + 64 + cp];
      const float4 f = ft4[(S - row) * 64 + cp];
      const float m00 = f.x * sm[0][0], m01 = f.y * sm[0][1], m10 = f.z * sm[1][0], m11 = f.w * sm[1][1];
      return make_float4(w0.x * m00 + w1.x * m10, -(w0.y * m00 + w1.y * m10), w0.z * m01 + w1.z * m11,
                         -(w0.w * m01 + w1.w * m11));
    };
    auto add_at = [&](int slot, int ca, int cb, float4 z) {
      float2 *tr = area + slot * RSR;
      const float2 oa = tr[ca], ob = tr[cb];
      tr[ca] = make_float2(oa.x + z.x, oa.y + z.y);
      tr[cb] = make_float2(ob.x + z.z, ob.y + z.w);
    };
    auto take_rows = [&](float2 (&v)[16], int h) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        float2 z = area[r * RSR + t + T * i];
        if (POLY) {
          const float2 w = w2m[(pr * (r + 64 * h) + pc * (t + T * i)) & (2 * M - 1)];
          z = make_float2(z.x * w.x + z.y * w.y, z.y * w.x - z.x * w.y);  // * conj(w)
        }
        v[i] = z;
      }
    };
    const float sr1 = (POLY && pr) ? -1.f : 1.f;
    // first half: direct parts of rows 0 .. 63
#pragma unroll 4
    for (int i = 0; i < 8; ++i) {
      const int row = wv + 8 * i;
      *reinterpret_cast<float4 *>(area + row * RSR + 2 * cp) = direct(row, 1.f);
    }
    __syncthreads();
    // mirrored parts of source rows 65 .. 127 (rows 63 .. 1 of the node); row 128 is the alias of row 0
#pragma unroll 4
    for (int i = 0; i < 8; ++i) {
      const int row = 64 + wv + 8 * i;
      if (row != 64) add_at(M - row, c0, c1, mirrored(row));
    }
    if (wv == 0) add_at(0, 2 * cp, 2 * cp + 1, direct(M, sr1));
    __syncthreads();
    take_rows(vh[0], 0);
    __syncthreads();
    fft_core_tab<16, T, true, false>(vh[0], t, area + r * RSR, T + 1, 1, wl, T);  // ends with a barrier
    // second half: rows 64 .. 127 through slots 0 .. 63; direct parts, then the mirrored parts of
    // source rows 1 .. 64
#pragma unroll 4
    for (int i = 0; i < 8; ++i) {
      const int row = 64 + wv + 8 * i;
      *reinterpret_cast<float4 *>(area + (row - 64) * RSR + 2 * cp) = direct(row, 1.f);
    }
    __syncthreads();
#pragma unroll 4
    for (int i = 0; i < 8; ++i) {
      const int row = i == 0 && wv == 0 ? 64 : wv + 8 * i;  // row 0 has no mirrored part: wave 0 takes row 64
      add_at(64 - row, c0, c1, mirrored(row));
    }
    __syncthreads();
    take_rows(vh[1], 1);
    __syncthreads();
    fft_core_tab<16, T, true, false>(vh[1], t, area + r * RSR, T + 1, 1, wl, T);
  } else {
    // Any source: thread = one column, rows rg + 4 i of a half of the node.  One pass of the
    // inner loop takes one alias block of one source (all 16 rows of the thread: 32 loads in
    // flight); alias blocks on which the filter is negligible are left out.
    constexpr int SROWS = FULL ? S : S / 2 + 1;  // stored rows of a source
    const float2 *src = a.src + static_cast<size_t>(s) * P * SROWS * S;
    const float *filt = a.filt + static_cast<size_t>(f) * P * S * S;
    const int col = tid % M;
    const int rg = __builtin_amdgcn_readfirstlane(tid / M);  // 0..3, the same for a wave
    static_assert(P * A * A <= 64, "one mask word per filter");
    constexpr unsigned long long kAll = P * A * A >= 64 ? ~0ull : (1ull << (P * A * A)) - 1ull;
    const unsigned long long used = ((P == 1 && a.mask != nullptr) ? a.mask[f] : ~0ull) & kAll;  // uniform
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float2 acc[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = make_float2(0.f, 0.f);
      unsigned long long rem = used;
      while (rem != 0ull) {
        const int bit = __builtin_amdgcn_readfirstlane(__ffsll(static_cast<long long>(rem)) - 1);
        rem &= rem - 1ull;
        const int ac = bit % A, ar = (bit / A) % A, q = bit / (A * A);
        const float2 *sq = src + static_cast<size_t>(q) * SROWS * S;
        const float *fq = filt + static_cast<size_t>(q) * S * S + (M * ar + 64 * h) * S;
        const unsigned kc = static_cast<unsigned>(col + M * ac) & (S - 1);
        const unsigned kcm = (S - kc) & (S - 1);
        // sign of the whole block: polyphase alias sign (-1)^(a.p)
        const float sblk = (POLY && ((ar * pr + ac * pc) & 1)) ? -1.f : 1.f;
        // rows above S/2 are not stored: U[kr][kc] = conj(U[S - kr][-kc]); the stored spectra of
        // polyphase components carry w^(p.k), which gives the mirrored value the extra sign
        // (-1)^(q_r) (-1)^(q_c [kc != 0])
        const float smir = (P == 4 && (((q >> 1) & 1) ^ ((q & 1) & (kc != 0 ? 1 : 0)))) ? -sblk : sblk;
        float2 v[16];
        float fv[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int kr = 64 * h + rg + 4 * i + M * ar;
          const bool mir = !FULL && kr > S / 2;  // the same for every lane of a wave
          v[i] = (sq + (mir ? S - kr : kr) * S)[mir ? kcm : kc];
          fv[i] = (fq + (rg + 4 * i) * S)[kc];
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const bool mir = !FULL && 64 * h + rg + 4 * i + M * ar > S / 2;
          const float fx = fv[i] * (mir ? smir : sblk);
          acc[i].x = fmaf(v[i].x, fx, acc[i].x);
          acc[i].y = fmaf(v[i].y, mir ? -fx : fx, acc[i].y);
        }
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int lr = rg + 4 * i;  // row within the half
        float2 z = acc[i];
        if (POLY) {
          const float2 w = a.tw[((pr * (64 * h + lr) + pc * col) * tw_step) & (a.tw_n - 1)];
          z = make_float2(z.x * w.x + z.y * w.y, z.y * w.x - z.x * w.y);  // * conj(w)
        }
        area[lr * RSR + col] = z;
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < 16; ++i) vh[h][i] = area[r * RSR + t + T * i];
      __syncthreads();
      fft_core_tab<16, T, true, false>(vh[h], t, area + r * RSR, T + 1, 1, wl, T);
    }
  }
  // ---- 2b. transposition, half of the columns at a time, and inverse column transforms
  float2 w[2][16];
#pragma unroll
  for (int hc = 0; hc < 2; ++hc) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      area[r * RSC + t + T * i] = vh[0][8 * hc + i];
      area[(r + 64) * RSC + t + T * i] = vh[1][8 * hc + i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) w[hc][i] = area[(t1 + T * i) * RSC + c];
    __syncthreads();
  }
#pragma unroll
  for (int hc = 0; hc < 2; ++hc)
    fft_core_tab<16, T, true, false>(w[hc], t1, area + c, T * RSC, RSC, wlc, T);

  // ---- 3. modulus; 4. lowpass + subsampling (rows first, then columns)
  constexpr int US = M + 1, HS = kOut + 1;
  float *ub = reinterpret_cast<float *>(area);  // [M][US], later [M][HS] over it
  float u[2][16];
#pragma unroll
  for (int hc = 0; hc < 2; ++hc)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      u[hc][i] = __builtin_amdgcn_sqrtf(w[hc][i].x * w[hc][i].x + w[hc][i].y * w[hc][i].y);
      ub[(t1 + T * i) * US + c + 64 * hc] = u[hc][i];
    }
  __syncthreads();
  {
    constexpr int OPT = kOut * M / NT;  // 8 outputs per thread, adjacent columns
    constexpr int NIN = DEC * (OPT - 1) + NTAP;
    const int rr = tid % M, mg = tid / M;
    const float *tc = a.taps_c + (POLY ? pc * NTAP : 0);
    float acc[OPT];
#pragma unroll
    for (int j = 0; j < OPT; ++j) acc[j] = 0.f;
    const int e0 = DEC * OPT * mg - R;
    // e0 is a multiple of 16: within a run of 16 inputs the column index does not wrap, so one
    // address per run and constant offsets inside it (no index arithmetic per read)
    constexpr int SEG = 16, NSEG = (NIN + SEG - 1) / SEG;
    static_assert((DEC * OPT) % SEG == 0 && R % SEG == 0, "runs of inputs that do not wrap");
    const float *seg[NSEG];
#pragma unroll
    for (int k = 0; k < NSEG; ++k) seg[k] = ub + rr * US + ((e0 + SEG * k) & (M - 1));
#pragma unroll
    for (int e = 0; e < NIN; ++e) {
      const float val = seg[e / SEG][e % SEG];
#pragma unroll
      for (int j = 0; j < OPT; ++j) {
        const int ti = DEC * j + 2 * R - e;
        if (ti >= 0 && ti <= 2 * R) acc[j] = fmaf(tc[ti], val, acc[j]);
      }
    }
    __syncthreads();  // the plane has been read by everybody: the filtered rows go over it
#pragma unroll
    for (int j = 0; j < OPT; ++j) ub[rr * HS + OPT * mg + j] = acc[j];
  }
  __syncthreads();
  {
    constexpr int OPV = kOut * kOut / NT;  // 2 outputs per thread, adjacent rows
    constexpr int NIN = DEC * (OPV - 1) + NTAP;
    const int mc = tid % kOut, ng = tid / kOut;
    const float *tr = a.taps_r + (POLY ? pr * NTAP : 0);
    float acc[OPV];
#pragma unroll
    for (int j = 0; j < OPV; ++j) acc[j] = 0.f;
    const int e0 = DEC * OPV * ng - R;
    constexpr int SEG = 8, NSEG = (NIN + SEG - 1) / SEG;  // e0 is a multiple of 8: see above
    static_assert((DEC * OPV) % SEG == 0 && R % SEG == 0, "runs of inputs that do not wrap");
    const float *seg[NSEG];
#pragma unroll
    for (int k = 0; k < NSEG; ++k) seg[k] = ub + ((e0 + SEG * k) & (M - 1)) * HS + mc;
#pragma unroll
    for (int e = 0; e < NIN; ++e) {
      const float val = seg[e / SEG][(e % SEG) * HS];
#pragma unroll
      for (int j = 0; j < OPV; ++j) {
        const int ti = DEC * j + 2 * R - e;
        if (ti >= 0 && ti <= 2 * R) acc[j] = fmaf(tr[ti], val, acc[j]);
      }
    }
    float *op;
    if (POLY) {
      op = a.out + (static_cast<size_t>(s) * I + item) * kOut * kOut;
    } else {
      const long plane = s / a.G;
      const int g = static_cast<int>(s - plane * a.G);
      op = a.out + (static_cast<size_t>(plane) * a.K + a.chan_base + g * a.chan_src + f * a.chan_f) *
                       kOut * kOut;
    }
#pragma unroll
    for (int j = 0; j < OPV; ++j) __builtin_nontemporal_store(acc[j], op + (OPV * ng + j) * kOut + mc);  // (never read here)
  }
  if (a.uout == nullptr) return;

  // ---- 5. spectrum of the modulus for the children; rows 0 .. 64 are stored.  The modulus is
  // real: a thread's two columns c and c + 64 travel through ONE column transform as
  // z = (u_c + i u_(c+64)) / 2, and the row threads take them apart again on the way in,
  // U_c[k] = Z[k] + conj(Z[-k]), U_(c+64)[k] = -i (Z[k] - conj(Z[-k])); only rows 0 .. 64 are
  // transformed along the rows (row 64 by eight lanes of the first wavefront on their own).
  __syncthreads();
  {
    float2 z[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = make_float2(0.5f * u[0][i], 0.5f * u[1][i]);
    fft_core_tab<16, T, false, false>(z, t1, area + c, T * RSC, RSC, wlc, T);
#pragma unroll
    for (int i = 0; i < 16; ++i) area[(t1 + T * i) * RSC + c] = z[i];
  }
  __syncthreads();
  {
    const int rm = (M - r) & (M - 1);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float2 za = area[r * RSC + t + T * i], zb = area[rm * RSC + t + T * i];
      vh[0][i] = make_float2(za.x + zb.x, za.y - zb.y);
      vh[0][8 + i] = make_float2(za.y + zb.y, zb.x - za.x);
    }
    if (tid < 64) row64[tid] = area[64 * RSC + tid];  // kept aside: the row transforms reuse the area
  }
  __syncthreads();
  fft_core_tab<16, T, false, false>(vh[0], t, area + r * RSR, T + 1, 1, wl, T);  // ends with a barrier
  {
    float2 *up = a.uout + ((static_cast<size_t>(s) * I + item) * (M / 2 + 1) + r) * M + t;
    // (the same table entries were read for the node's own rows at the start; hidden from the
    // compiler, which would otherwise keep all sixteen alive, and spill them, to save these reads)
    int wbase = pr * r + pc * t;
    asm volatile("" : "+v"(wbase));
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      float2 val = vh[0][i];
      if (POLY) val = c_mul(val, w2m[(wbase + pc * T * i) & (2 * M - 1)]);
      if constexpr (POLY) {
        // the first octave's spectra (0.8 GB per launch) are read by a later launch, from
        // memory in any case: kept out of the caches' way, the parents' own reads of the
        // image's spectrum and of the tables hit more often (the later octaves' spectra fit
        // the last-level cache and are stored the plain way)
        __builtin_nontemporal_store(val.x, &up[T * i].x);
        __builtin_nontemporal_store(val.y, &up[T * i].y);
      } else {
        up[T * i] = val;
      }
    }
  }
  if (tid < T) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float2 za = row64[t + T * i];
      vh[0][i] = make_float2(2.f * za.x, 0.f);
      vh[0][8 + i] = make_float2(2.f * za.y, 0.f);
    }
    fft_core_tab<16, T, false, true>(vh[0], t, area, T + 1, 1, wl, T);
    float2 *up = a.uout + ((static_cast<size_t>(s) * I + item) * (M / 2 + 1) + 64) * M + t;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      float2 val = vh[0][i];
      if (POLY) val = c_mul(val, w2m[(pr * 64 + pc * (t + T * i)) & (2 * M - 1)]);
      up[T * i] = val;
    }
  }
}

// out[plane][chan_base + g][.] = sum of the four parts of node (plane, g)
__global__ __launch_bounds__(256) void k_sum4(const float *__restrict__ part, float *__restrict__ out,
                                               long nodes, int G, int K, int chan_base) {
  const long idx = static_cast<long>(blockIdx.x) * 256 + threadIdx.x;
  constexpr int PL = kOut * kOut;
  if (idx >= nodes * PL) return;
  const long node = idx / PL;
  const int e = static_cast<int>(idx - node * PL);
  const float *p = part + node * 4 * PL + e;
  const long plane = node / G;
  const int g = static_cast<int>(node - plane * G);
  out[(plane * K + chan_base + g) * PL + e] = (p[0] + p[PL]) + (p[2 * PL] + p[3 * PL]);
}

template <int M, int A, int P, bool POLY, bool FULL = false>
hipError_t launch_node_t(const NodeArgs &a, hipStream_t st) {
  constexpr int S = M * A;
  const int I = a.F * (POLY ? 4 : 1);
  const long blocks = 8 * ((a.NS + 7) / 8) * I;
  if (a.NS <= 0 || blocks > 0x7fffffffL || a.tw_n % (POLY ? 2 * M : M) != 0) return hipErrorInvalidValue;
  // k_node: rows + twiddles (39 KB: four workgroups per compute unit).  The four-component
  // variant is bound by its loads and measured faster with THREE workgroups per compute unit
  // (fewer loads in flight): it asks for 44 KB.
  const size_t lds = P == 4 ? static_cast<size_t>(44) << 10 : (static_cast<size_t>(M) * 76 + 2 * M) * sizeof(float2);
  constexpr bool kPairs = M == 64 && A == 2 && P == 4 && !POLY && !FULL;  // two filters per workgroup
  const bool pairs = kPairs && a.F % 2 == 0;
  const std::string name = pairs ? std::string("k_node_pair")
                                 : (M == 128 ? "k_node_half<" : "k_node<64, ") + std::to_string(A) + ", " +
                                       std::to_string(P) + (POLY ? ", true" : ", false") + (FULL ? ", full>" : ">");
  const double items = static_cast<double>(a.NS) * I;
  const double pts = static_cast<double>(M) * M;
  LaunchScope obs(name.c_str(),
                  static_cast<double>(a.NS) * P * (FULL ? S : S / 2 + 1) * S * 8 +
                      static_cast<double>(a.F) * P * S * S * 4 + items * kOut * kOut * 4 +
                      (a.uout ? items * (M / 2 + 1) * M * 8 : 0),
                  items * ((a.uout ? 2 : 1) * fft2_flops(M) + fft2_flops(kOut) +
                           pts * (4.0 * P * A * A + 4.0 + 2.0) + fft2_flops(M) * (a.uout ? 0 : 1)),
                  st);
  if constexpr (kPairs) {
    if (pairs) {
      // pairs of filters: half as many workgroups of twice the size
      const size_t lds_p = (static_cast<size_t>(2) * M * 76 + 2 * M) * sizeof(float2);
      static unsigned long long lds_ok = 0;
      hipError_t e = allow_large_lds(reinterpret_cast<const void *>(k_node_pair), lds_ok);
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL(k_node_pair, dim3(static_cast<unsigned>(blocks / 2)), dim3(512), lds_p, st, a);
      return hipGetLastError();
    }
  }
  if constexpr (M == 128) {
    const size_t lds_h = (64 * 152 + 128 + 256 + 64) * sizeof(float2);
    static unsigned long long lds_ok = 0;
    hipError_t e = allow_large_lds(reinterpret_cast<const void *>(k_node_half<A, P, POLY, FULL>), lds_ok);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((k_node_half<A, P, POLY, FULL>), dim3(static_cast<unsigned>(blocks)), dim3(512), lds_h, st,
                       a);
  } else {
    hipLaunchKernelGGL((k_node<M, A, P, POLY, FULL>), dim3(static_cast<unsigned>(blocks)), dim3(M * M / 16), lds,
                       st, a);
  }
  return hipGetLastError();
}

}  // namespace

bool node_supported(int M, int A, int P, bool poly, bool full) {
  if (full)  // children (no spectrum of their own) of parents whose whole spectrum is stored
    return !poly && P == 1 && ((M == 128 && (A == 2 || A == 4)) || (M == 64 && (A == 2 || A == 4 || A == 8)));
  if (poly) return M == 128 && A == 2 && P == 1;
  if (M == 128) return (A == 1 && (P == 1 || P == 4)) || (A == 2 && P == 1);
  if (M == 64) return (A == 2 && (P == 1 || P == 4)) || (A == 4 && P == 1);
  return false;
}

hipError_t launch_node(const NodeLaunch &n, hipStream_t st) {
  if (!node_supported(n.M, n.A, n.P, n.poly, n.full) || n.G < 1 || n.F < 1) return hipErrorInvalidValue;
  if (n.full && n.uout != nullptr) return hipErrorInvalidValue;
  NodeArgs a;
  a.src = n.src;
  a.filt = n.filt;
  a.mask = n.mask;
  a.lane_mask = n.lane_mask;
  a.taps_r = n.taps_r;
  a.taps_c = n.taps_c;
  a.uout = n.uout;
  a.out = n.out;
  a.NS = n.NS;
  a.F = n.F;
  a.G = n.G;
  a.chan_base = n.chan_base;
  a.chan_src = n.chan_src;
  a.chan_f = n.chan_f;
  a.K = n.K;
  a.tw = n.tw;
  a.tw_n = n.tw_n;
#define SCAT_NODE_FULL(M_, A_) \
  if (n.full && n.M == M_ && n.A == A_) return launch_node_t<M_, A_, 1, false, true>(a, st)
  SCAT_NODE_FULL(128, 2);
  SCAT_NODE_FULL(128, 4);
  SCAT_NODE_FULL(64, 2);
  SCAT_NODE_FULL(64, 4);
  SCAT_NODE_FULL(64, 8);
#undef SCAT_NODE_FULL
#define SCAT_NODE(M_, A_, P_, POLY_) \
  if (n.M == M_ && n.A == A_ && n.P == P_ && n.poly == POLY_) return launch_node_t<M_, A_, P_, POLY_>(a, st)
  SCAT_NODE(128, 2, 1, true);
  SCAT_NODE(128, 2, 1, false);
  SCAT_NODE(128, 1, 1, false);
  SCAT_NODE(128, 1, 4, false);
  SCAT_NODE(64, 2, 4, false);
  SCAT_NODE(64, 2, 1, false);
  SCAT_NODE(64, 4, 1, false);
#undef SCAT_NODE
  return hipErrorInvalidValue;
}

hipError_t launch_sum4(const float *part, float *out, long nodes, int G, int K, int chan_base,
                       hipStream_t st) {
  if (nodes <= 0) return hipSuccess;
  const long total = nodes * kOut * kOut;
  const long blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  LaunchScope obs("k_sum4", static_cast<double>(total) * 20.0, static_cast<double>(total) * 3.0, st);
  hipLaunchKernelGGL(k_sum4, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, part, out, nodes, G, K,
                     chan_base);
  return hipGetLastError();
}

}  // namespace scat
