// Launch wrappers of the generic scattering kernels (see scat_kernels.hip).
#pragma once

#include <hip/hip_runtime.h>

namespace scat {

// Optional per-thread hook called around every kernel launch of this file: `before` gets
// the kernel's name as a profiler prints it, the bytes the launch must move at the least
// (inputs and filter tables read once, outputs written once) and its model flops
// (5 n log2 n per transform plus the pointwise work).
struct LaunchObserver {
  virtual void before(const char *name, double bytes, double flops, hipStream_t st) = 0;
  virtual void after(hipStream_t st) = 0;
  virtual ~LaunchObserver() = default;
};
void set_launch_observer(LaunchObserver *o);

// Reports one launch to the installed observer: construct right before the launch,
// destroy right after it.
struct LaunchScope {
  LaunchScope(const char *name, double bytes, double flops, hipStream_t st);
  ~LaunchScope();
  LaunchScope(const LaunchScope &) = delete;
  LaunchScope &operator=(const LaunchScope &) = delete;

 private:
  hipStream_t st_;
  bool on_;
};

// Lets kernel `fn` use up to 160 KB of dynamic LDS on the current device.  The attribute is
// per device; `done` (one static per kernel at the call site) remembers the devices served.
inline hipError_t allow_large_lds(const void *fn, unsigned long long &done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const unsigned long long bit = 1ull << (dev & 63);
  if (done & bit) return hipSuccess;
  e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e == hipSuccess) done |= bit;
  return e;
}

// Where a kernel's node number g (within one input plane p) lands in the output:
// channel = base + (g / inner) * outer_stride + (g % inner), node = p * G + g.
struct ChanMap {
  int G, inner, outer_stride, base;
};

// mask (optional, device): per filter a 64-bit word, bit a_r * 2^fc + a_c set = the alias block
// (a_r, a_c) of (Sr >> fr) x (Sc >> fc) points holds values that matter; blocks whose bit is
// clear for every filter processed together are skipped (needs 2^(fr + fc) <= 64).
hipError_t launch_mulfold_invrow(const float2 *src, const float *filt, float2 *dst, long S, int F,
                                 int Sr, int Sc, int fr, int fc, int post_tw_m, const float2 *tw,
                                 int tw_n, hipStream_t st, const unsigned long long *mask = nullptr);

hipError_t launch_col(int mode, const void *src, long nodes, int Mr, int Mc, float2 *uc,
                      int post_tw_m, const float *phi_rows, int m_r, float *w_out, float *out,
                      ChanMap cm, int K, const float2 *tw, int tw_n, hipStream_t st,
                      bool uc_half = false);

// launch_col mode 1 with the four-step twiddle (post_tw_m = Mr * Mc) over up to kColMaxSegs
// arrays of nodes in one launch: segment i holds `nodes` signals of Mr x Mc elements at
// src + src_off and writes their column spectra to uc + uc_off (Mr = 256, Mc a multiple of 16).
constexpr int kColMaxSegs = 8;
struct ColSeg {
  long nodes;
  int Mc;
  long long src_off, uc_off;
};
// uc_half: the columns are real after the modulus, so only rows 0 .. Mr/2 of every node's
// spectrum are written ([nodes][Mr/2+1][Mc] at uc + uc_off; launch_rows1d with half_rows reads them)
hipError_t launch_col_segs(const float2 *src, float2 *uc, int Mr, const ColSeg *segs, int n, bool uc_half,
                           const float2 *tw, int tw_n, hipStream_t st);

// launch_col mode 2 for 256-row nodes of Mc <= 16 columns, over `nodes` nodes mapped by cm and,
// stored right behind them, `tail_nodes` nodes that are channel 0 of signals 0, 1, ...
bool col_out_tail_supported(int Mr, int Mc, int tw_n);
hipError_t launch_col_out_tail(const float2 *src, long nodes, long tail_nodes, int Mc, float *out, ChanMap cm, int K,
                               const float2 *tw, int tw_n, hipStream_t st);

// 1-D cascade: forward row FFT of src [nodes][Sr][Sc] (column spectra, left untouched) and,
// for each child, filter product + fold of the row by 2^lg_fold + inverse row FFT + four-step
// twiddle, stored to the child's dst [nodes][Sr][Sc >> lg_fold] (see k_rows1d).
constexpr int kRows1dMaxChildren = 32;
struct Rows1dChild {
  const float *filt;  // [Sr][Sc], carries the inverse-transform normalisation
  float2 *dst;
  int lg_fold;
  int post_tw_m;  // 0 = no twiddle, else Sr * (Sc >> lg_fold): the child's signal length
  // K > 0: node p * cm.G + g is stored as signal number p * K + channel(cm, g) instead of at
  // its own number (the lowpass children of a whole transform gathered channel-major)
  ChanMap cm;
  int K;
  // null, or cm.G device words: the channel of node g comes from this table instead of cm's
  // formula (nodes of several parent octaves in one launch)
  const int *chan_tab;
};
struct Rows1dArgs {
  int n;
  Rows1dChild c[kRows1dMaxChildren];
  // null, or where the forward row spectra themselves are stored ([nodes][Sr][Sc]; may be the
  // source: in place).  Register kernel with all rows stored only.
  float2 *spec_out = nullptr;
};
// half_rows: src holds rows 0 .. Sr/2 of every node only ([nodes][Sr/2+1][Sc], written by the
// column pass with uc_half for real columns); the other rows are derived from them
// (rows1d_half_supported: the row lengths for which that form exists)
bool rows1d_half_supported(int Sr, int Sc);
hipError_t launch_rows1d(const float2 *src, long nodes, int Sr, int Sc, const Rows1dArgs &a,
                         const float2 *tw, int tw_n, hipStream_t st, bool half_rows = false);

// Adjoint of launch_rows1d: dst [nodes][Sr][Sc] (= or +=) the inverse row FFT of
// sum_c filt_c * tile(forward row FFT of child c), child rows of Sc >> lg_fold points (see
// k_rows1d_adj).  Node g of dst reads node number
//   K == 0:  g * cm.G + cm.base                       (one of the cm.G nodes under each parent)
//   K  > 0:  (g / cm.G) * K + channel(cm, g % cm.G)   (channel-major arrays, as Rows1dChild)
// of c.src.
struct Rows1dAdjChild {
  const float2 *src;
  const float *filt;  // [Sr][Sc], the table of the forward pass
  int lg_fold;
  ChanMap cm;
  int K;
};
struct Rows1dAdjArgs {
  int n;
  int accumulate;  // 0: dst is overwritten; 1: added to
  Rows1dAdjChild c[kRows1dMaxChildren];
};
bool rows1d_adj_supported(int Sc);
hipError_t launch_rows1d_adj(float2 *dst, long nodes, int Sr, int Sc, const Rows1dAdjArgs &a,
                             const float2 *tw, int tw_n, hipStream_t st);

// 2-D: dst [nodes][Sr][Sc] (= or +=) sum_c filt_c * tile(src_c), child planes of
// (Sr >> lg_fr) x (Sc >> lg_fc) gradient spectra, then (inverse != 0) the inverse row
// transform (see k_rows2d_adj).  filt_row != nullptr: the filter is filt_row[kr] * filt[kc].
// Child nodes as in Rows1dAdjChild.  Row lengths 4 ... 512, with the inverse transform up to 256.
struct Rows2dAdjChild {
  const float2 *src;
  const float *filt;
  const float *filt_row;
  int lg_fr, lg_fc;
  ChanMap cm;
  int K;
  int pre_rows;  // 1: src is given before its forward row transform (lg_fc == 0, rows <= 256)
};
struct Rows2dAdjArgs {
  int n;
  int accumulate;
  int inverse;
  int lg_rows, any_pre_rows;  // set by the launcher
  Rows2dAdjChild c[kRows1dMaxChildren];
};
bool rows2d_adj_supported(int Sc, bool inverse);
hipError_t launch_rows2d_adj(float2 *dst, long nodes, int Sr, int Sc, const Rows2dAdjArgs &a,
                             const float2 *tw, int tw_n, hipStream_t st);

hipError_t launch_row_fwd(float2 *data, long rows, int Mc, const float2 *tw, int tw_n,
                          hipStream_t st);

hipError_t launch_row_lowpass(const float *w, long nodes, int m_r, int Mc, int m_c,
                              const float *phi_cols, float *out, ChanMap cm, int K,
                              const float2 *tw, int tw_n, hipStream_t st);

// Column pass of whole square nodes (Mr x Mr) with both halves of the lowpass (length m on
// both axes) fused: like launch_col mode 0/1 followed by launch_row_lowpass, but S goes
// straight to `out` and the intermediate W never to memory.
bool col_node_supported(int Mr, int Mc, int m_r, int m_c, int tw_n);
hipError_t launch_col_node(int mode, const void *src, long nodes, int Mr, int m, float2 *uc,
                           bool uc_half, const float *phi_rows, const float *phi_cols, float *out,
                           ChanMap cm, int K, const float2 *tw, int tw_n, hipStream_t st);

// Leaf nodes (no children; 64 x 64 with a 32 x 32 output) from the row pass's output to the
// output coefficients in one kernel (see k_leaf_node).
bool leaf_node_supported(int Mr, int Mc, int m_r, int m_c, int tw_n);
hipError_t launch_leaf_node(const float2 *src, long nodes, int Mr, int m, const float *phi_rows,
                            const float *phi_cols, float *out, ChanMap cm, int K, const float2 *tw,
                            int tw_n, hipStream_t st);

// One level of the fused row pass: wavelets `filt` ([F][Sr][Sc] real, pre-scaled) applied
// with fold 2^f on both axes, outputs to dst [NS*F][Sr>>f][Sc>>f].
struct FusedLevel {
  int f, F;
  const float *filt;
  float2 *dst;
};

// True if launch_rows_fused can handle sources of Sr x Sc with largest fold 2^fmax.
bool rows_fused_supported(int Sr, int Sc, int fmax);

// Forward row FFT of column-transformed sources [NS][Sr][Sc] (or half, see below), then every level's filter
// multiply + fold + inverse row FFT (see k_rows_fused).
// src_half: the sources hold rows 0..Sr/2 only ([NS][Sr/2+1][Sc], column spectra of real
// signals as written by launch_col with uc_half); the other rows are their conjugates.
hipError_t launch_rows_fused(const float2 *src, bool src_half, long NS, int Sr, int Sc,
                             const FusedLevel *levels, int nlev, const float2 *tw, int tw_n,
                             hipStream_t st);

// Whole scattering tree of 32 x 32 planes at J = 2 below the input spectrum: one wavefront
// per first-order node keeps the node, the spectrum of its modulus and its second-order
// children in LDS and writes only S1 and S2 (see scat_tree.hip).
//   xh        [planes][32][32] spectra of the inputs (forward 2-D FFT, unnormalised)
//   psi_j0/1  [L][32][32] first-order wavelets of octaves 0 and 1, pre-scaled by 1/1024
//   phi_cols* lowpass along a row (the column frequency axis) at resolutions 0 (32 samples)
//             and 1 (16 samples), Fourier domain, pre-scaled by 1/length
//   taps*     lowpass along a column at the same resolutions as spatial taps: the inverse
//             DFT (unnormalised) of the pre-scaled Fourier samples, 32 and 16 values
//   out       [planes][K][8][8]; channel 0 (S0) is not written here
bool tree_supported(int n_r, int n_c, int J);
// x [planes][32][32] real -> xh (its unnormalised 2-D spectrum) and S0 (channel 0 of out)
hipError_t launch_tree32_input(const float *x, long planes, float2 *xh, const float *phi_cols0,
                               const float *taps0, float *out, int K, hipStream_t st);
hipError_t launch_tree32(const float2 *xh, long planes, int L, int max_order, const float *psi_j0,
                         const float *psi_j1, const float *phi_cols0, const float *phi_cols1,
                         const float *taps0, const float *taps1, float *out, int K,
                         hipStream_t st);

// Whole nodes of the 2-D tree in one kernel each (scat_node.hip): spectrum of the node from
// its parent's stored half spectra (P sources of S x S, S = M * A, with A x A aliases folded),
// inverse transform, modulus, lowpass to the 32 x 32 output grid by a separable FIR filter
// (taps: 2 R + 1 values, R = 4 M / 32; polyphase nodes: two sets, for p = 0 and p = 1), and
// optionally the half spectrum of the modulus for the node's children.
//   src    [NS][P][S/2+1][S]; filt [F][P][S][S]; items per source: F (poly: 4 F, the four
//          polyphase components of each filter's node, component index 2 p_r + p_c fastest)
//   mask   filters that vanish on whole M x M alias blocks of their table: the blocks to skip
//   uout   null or [NS * items][M/2+1][M] (poly: times w^(p.k), w = exp(-2 pi i / 2M))
//   out    [planes][K][32][32] with channel = chan_base + (source % G) * chan_src +
//          filter * chan_f and plane = source / G; poly: parts [NS * items][32][32]
struct NodeLaunch {
  int M, A, P;
  bool poly;
  bool full;  // src holds all S rows of one spectrum per node ([NS][S][S]) instead of rows 0 .. S/2
  const float2 *src;
  const float *filt;
  const unsigned long long *mask;  // null, or [F] device words: bit (q A + a_r) A + a_c set = block in use
  // null, or [F][words per workgroup] device words for the loaders whose source is twice the
  // node's size: per thread, which of its loads meet table values that are not negligible
  // (node_lane_mask builds them from the table itself)
  const unsigned *lane_mask;
  const float *taps_r, *taps_c;
  float2 *uout;
  float *out;
  long NS;
  int F, G;
  int chan_base, chan_src, chan_f, K;
  const float2 *tw;
  int tw_n;
};
bool node_supported(int M, int A, int P, bool poly, bool full = false);
hipError_t launch_node(const NodeLaunch &n, hipStream_t st);
// out[plane][chan_base + g][32][32] = sum of the four parts of node plane * G + g
hipError_t launch_sum4(const float *part, float *out, long nodes, int G, int K, int chan_base,
                       hipStream_t st);

// Modulus backward step of whole nodes in one pass (k_node_modback): data [nodes][Mr][Mc]
// gradient spectra in, gradient spectra of the taped y [nodes][Mr][Mc] out, in place.  The
// _low form starts from the node's adjoint lowpass instead (arguments as
// launch_lowpass_adj_rows; ghat is scratch for nodes * m_r * m_c elements); with y_rows, y is
// the node before its inverse column transform (the forward row pass's output) and the
// kernel transforms the columns itself.
bool node_modback_supported(int Mr, int Mc);
// ghat [node][m_r][m_c] = 2-D transform of the nodes' output gradient planes
bool small_fft2_supported(int m_r, int m_c);
hipError_t launch_small_fft2(const float *gout, long nodes, ChanMap cm, int K, int m_r, int m_c,
                             float2 *ghat, const float2 *tw, int tw_n, hipStream_t st);
hipError_t launch_node_modback(float2 *data, const float2 *y, long nodes, int Mr, int Mc,
                               const float2 *tw, int tw_n, hipStream_t st, bool y_rows = false);
hipError_t launch_node_modback_low(const float *gout, long nodes, ChanMap cm, int K, int m_r, int m_c,
                                   int Mr, int Mc, const float *phi_rows, const float *phi_cols,
                                   float2 *ghat, const float2 *y, float2 *dst, const float2 *tw,
                                   int tw_n, hipStream_t st, bool y_rows = false);

// ---- backward pass (scat_backward.hip): plain 2-D transforms in place and the adjoints of
// the lowpass, the modulus and the filter-multiply-fold step.  Sides 4...512.
bool backward_side_supported(int m);
// rows only: data [rows][Mc]
hipError_t launch_fft_rows_inplace(float2 *data, long rows, int Mc, bool inverse, const float2 *tw,
                                   int tw_n, hipStream_t st);
// columns of data [nodes][Mr][Mc]: inverse transform, a = Re(a) y / |y| (0 where y = 0)
// against y of the same layout, forward transform
// tw_m > 0: with the four-step twiddles exp(+-2 pi i k1 b / tw_m) around the column passes
hipError_t launch_cols_modback(float2 *data, const float2 *y, long nodes, int Mr, int Mc,
                               const float2 *tw, int tw_n, hipStream_t st, int tw_m = 0,
                               bool y_rows = false);
// columns only (any power-of-two number of columns up to 512)
hipError_t launch_fft_cols_inplace(float2 *data, long nodes, int Mr, int Mc, bool inverse,
                                   const float2 *tw, int tw_n, hipStream_t st);
// 1-D signals as n1 x Mc matrices: data[node][k1][b] *= exp(-+2 pi i k1 b / (n1 Mc))
hipError_t launch_twiddle(float2 *data, long nodes, int n1, int Mc, bool conj, const float2 *tw,
                          int tw_n, hipStream_t st);
// dst[node][i] = (g_out[plane][chan(cm, g)][i], 0) for i < m
hipError_t launch_gather_real(const float *gout, long nodes, ChanMap cm, int K, int m, float2 *dst,
                              hipStream_t st);
// dst[node][k1][k2] = ghat[node][k1][k2 mod mc] * filt[k1][k2]
hipError_t launch_tile_filter(const float2 *ghat, const float *filt, float2 *dst, long nodes, int n1,
                              int Mc, int mc, hipStream_t st);
// the same followed by the inverse row transform, in one pass over dst; `ghat` is scratch
// of nodes * m_r * m_c elements
hipError_t launch_lowpass_adj_rows(const float *gout, long nodes, ChanMap cm, int K, int m_r,
                                   int m_c, int Mr, int Mc, const float *phi_rows,
                                   const float *phi_cols, float2 *ghat, float2 *dst,
                                   const float2 *tw, int tw_n, hipStream_t st);
hipError_t launch_take_real(const float2 *a, float *out, long count, hipStream_t st);
// dst [S][Sr][Sc] += sum_f filt[f] * G[s F + f][k_r mod Mr][k_c mod Mc]
hipError_t launch_tile_accum(float2 *dst, const float *filt, const float2 *G, long S, int F, int Sr,
                             int Sc, int Mr, int Mc, hipStream_t st);

// ---- 3-D solid harmonic scattering (scat_3d.hip): a 3-D transform in place over
// [volumes][n0][n1][n2] (sides 4...256) and the pointwise steps of the cascade
// fused 3-D passes (slabs of axes 1 and 2 held by one workgroup); see scat_3d.hip
bool fused3_supported(int n0, int n1, int n2, int J);
hipError_t launch3_slab_mul_inv(const float2 *Fh, const float2 *tab, float2 *W, long volumes, int n0,
                                int n1, int n2, int M, const float2 *tw, int tw_n, hipStream_t st);
hipError_t launch3_slab_fwd_low(const float2 *Tin, float2 *Uout, const float *phi, float2 *P,
                                long volumes, int n0, int n1, int n2, int J, int K, int chan,
                                const float2 *tw, int tw_n, hipStream_t st);
hipError_t launch3_axis0_rho(const float2 *W, const float *xreal, float2 *dst, long volumes, int n0,
                             int Mc, int M, const float2 *tw, int tw_n, hipStream_t st);
hipError_t launch3_fold0(const float2 *P, float2 *Q, long groups, int n0, int m0, int slab,
                         hipStream_t st);
hipError_t launch3_real_part(const float2 *src, float *out, long total, hipStream_t st);
hipError_t launch3_fft(float2 *data, long volumes, int n0, int n1, int n2, bool inverse,
                       const float2 *tw, int tw_n, hipStream_t st);
hipError_t launch3_real_to_complex(const float *x, float2 *out, long total, hipStream_t st);
// dst[v][e] = src[v][e] * filt[e], e < n
hipError_t launch3_mul_table(const float2 *src, const float *filt, float2 *dst, long volumes, long n,
                             hipStream_t st, int fstride = 1, bool accumulate = false);
// backward pass of the 3-D transform: lowpass adjoint, pair-table products, gradient through rho
hipError_t launch3_tile_phi(const float2 *Gs, const float *phi, float2 *dst, long volumes, int K,
                            int chan, int n0, int n1, int n2, int J, bool accumulate, hipStream_t st);
hipError_t launch3_mul_ctable(const float2 *src, const float2 *ctab, float2 *dst, long volumes, long n,
                              bool conj_table, bool accumulate, hipStream_t st);
// fused backward passes (plans whose slabs fit a workgroup): axis 0 of the P pair signals in
// place (mode 0: inverse transform + sum of squared moduli; mode 1: gradient through rho +
// forward transform), and the adjoint of launch3_slab_mul_inv accumulated into A
hipError_t launch3_axis0_back(int mode, float2 *W, float *acc, const float2 *gu, long volumes, int n0,
                              int Mc, int P, const float2 *tw, int tw_n, hipStream_t st);
hipError_t launch3_slab_fwd_mulacc(const float2 *W, const float2 *tab, float2 *A, long volumes, int n0,
                                   int n1, int n2, int P, const float2 *tw, int tw_n, hipStream_t st);
hipError_t launch3_rho_back(const float2 *gu, const float *acc, float2 *y, long total,
                            hipStream_t st);
// acc[i] = |y[i]|^2 (first) or acc[i] + |y[i]|^2
hipError_t launch3_accum_abs2(const float2 *y, float *acc, long total, bool first, hipStream_t st);
// out[i] = (sqrt(acc[i]), 0)
hipError_t launch3_sqrt(const float *acc, float2 *out, long total, hipStream_t st);
// out[v][chan][a][b][c] = Re src[v][a 2^J][b 2^J][c 2^J], out has K channels per volume
hipError_t launch3_sample(const float2 *src, float *out, long volumes, int K, int chan, int n0,
                          int n1, int n2, int J, hipStream_t st);

}  // namespace scat
