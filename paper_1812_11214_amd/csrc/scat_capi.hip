// C ABI of the scattering library: plan life cycle, table upload, and the schedule that
// walks the scattering tree one first-order octave after the other (paper section 2,
// "Implementation": depth-first traversal, downsampled intermediates).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "../../include/scat.h"
#include "scat_host.hpp"
#include "scat_host3d.hpp"
#include "scat_kernels.hpp"

// Records a HIP event pair around launches (all, or those of one kernel name) and sums
// their durations per kernel name.
struct LaunchTimer : scat::LaunchObserver {
  struct Row {
    std::string name;
    long launches = 0;
    double ms = 0, bytes = 0, flops = 0;
  };
  bool enabled = false;
  std::string only;  // empty = every kernel
  std::vector<Row> rows;
  std::vector<hipEvent_t> pool;  // pairs: 2*i = start, 2*i+1 = stop
  std::vector<int> pair_row;     // row of each recorded pair
  bool recording = false;
  bool failed = false;

  void before(const char *name, double bytes, double flops, hipStream_t st) override {
    recording = false;
    if (!enabled || (!only.empty() && only != name)) return;
    size_t r = 0;
    while (r < rows.size() && rows[r].name != name) ++r;
    if (r == rows.size()) {
      rows.emplace_back();
      rows.back().name = name;
    }
    rows[r].launches += 1;
    rows[r].bytes += bytes;
    rows[r].flops += flops;
    const size_t i = pair_row.size();
    while (pool.size() < 2 * (i + 1)) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) {
        failed = true;
        return;
      }
      pool.push_back(e);
    }
    if (hipEventRecord(pool[2 * i], st) != hipSuccess) failed = true;
    pair_row.push_back(static_cast<int>(r));
    recording = true;
  }
  void after(hipStream_t st) override {
    if (!recording) return;
    if (hipEventRecord(pool[2 * (pair_row.size() - 1) + 1], st) != hipSuccess) failed = true;
    recording = false;
  }
  // Waits for every recorded pair and adds up the elapsed times.
  bool collect() {
    for (size_t i = 0; i < pair_row.size(); ++i) {
      float ms = 0.f;
      if (hipEventSynchronize(pool[2 * i + 1]) != hipSuccess ||
          hipEventElapsedTime(&ms, pool[2 * i], pool[2 * i + 1]) != hipSuccess) {
        failed = true;
        continue;
      }
      rows[pair_row[i]].ms += ms;
    }
    pair_row.clear();
    return !failed;
  }
  void release() {
    for (hipEvent_t e : pool) (void)hipEventDestroy(e);
    pool.clear();
  }
};

struct scat_plan {
  scat::HostPlan host;
  LaunchTimer timer;
  bool has_device = false;
  int device = -1;
  // Grid the kernels see: 2-D (rows, cols); 1-D the four-step factorisation N = n1 * n2,
  // signal sample n1_index * n2 + n2_index.
  int n1 = 1, n2 = 1;
  float *d_tables = nullptr;
  float2 *d_tw = nullptr;
  int tw_n = 0;
  void *d_scratch = nullptr;
  size_t scratch_bytes = 0;
  // scratch of the call in progress: d_scratch, or the library's static array for
  // scat_forward_static (set by the entry points before any schedule runs)
  void *work = nullptr;
  void *static_scratch = nullptr;  // device address of the library's static scratch array
  // offsets (in floats) into d_tables
  std::vector<size_t> psi1_off;                    // per octave; LQ tables contiguous
  std::map<std::pair<int, int>, size_t> psi2_off;  // (res, j2) -> tables (2-D: L contiguous)
  std::vector<size_t> phi_rows_off, phi_cols_off;  // 2-D, per res
  std::vector<size_t> phi_off;                     // 1-D, per res
  bool fused = false;  // 2-D: the fused row pass can serve every level of this plan
  bool tree = false;   // 2-D: planes small enough for the whole-tree-in-LDS kernel
  // 2-D: every node of the tree is computed by one workgroup (scat_node.hip): forward calls
  // keep only the spectra of x and of the first-order moduli with children in scratch
  bool node = false;
  bool node_tables = false;  // shapes the whole-node schedule serves: its filter tables are uploaded
  bool node_taps = false;    // square grids with a 32 x 32 output grid: the spatial lowpass taps of the
                             // whole-node kernels are uploaded (children of 64 or 128 points a side)
  std::map<int, size_t> poly_psi_off;          // j2 -> [L][4][N/2][N/2] sign-folded wavelets
  // (res, j) -> the L wavelets of octave j on the grid of resolution res in the layout of the
  // whole-node kernels whose source is twice as large as the node (M = side / 2).  M = 128:
  // [row][column pair][column block][column parity] = psi[row][c], c = M block + 2 pair + parity,
  // for rows 0 .. side / 2 and psi[row][-c] for the rows above (read for the mirrored parts);
  // M = 64: [row][column block][column parity][column pair] = psi[row][c] (the layouts each
  // kernel measured faster with)
  std::map<std::pair<int, int>, size_t> node2_off;
  std::vector<size_t> taps_r_off, taps_c_off;  // per res: spatial lowpass taps [2R+1]
  size_t ptaps_r_off = 0, ptaps_c_off = 0;     // polyphase taps of resolution 0: [2][2R+1]
  // per wavelet table: which (n1 >> j) x (n2 >> j) alias blocks of it are not negligible (bit
  // a_r * A_c + a_c); mask64_off[{res, j}] -> L words in d_masks64 (absent when A_r * A_c > 64).
  // Read by the whole-node kernels and by the row pass of the general 2-D schedule.
  unsigned long long *d_masks64 = nullptr;
  std::map<std::pair<int, int>, size_t> mask64_off;
  // per table of node2_off ((res, j)) and poly_psi_off ((-1, j2)) read by a whole-node kernel whose
  // source is twice the node's size: per thread of the workgroup, which of its loads meet a
  // table value above 1e-7 of the table's peak (lane_words_64); L tables contiguous
  unsigned *d_lane_masks = nullptr;
  std::map<std::pair<int, int>, size_t> lane_mask_off;
  // 3-D solid harmonic plans (host.dims == 3; host carries J, LQ = L, max_order, K only)
  scat::HostPlan3D h3;
  std::vector<size_t> psi3_off;  // per (j, l): its 2l+1 tables, contiguous
  size_t phi3_off = 0;
  bool fused3 = false;  // 3-D: slabs of the two fast axes fit a workgroup (fused passes)
  int user_shape3[3] = {0, 0, 0};  // padded 3-D plans: the caller's volume and output sides
  int user_out3[3] = {0, 0, 0};
  // signals of any size: the caller's shape, symmetrically extended to the plan's periodic
  // grid before the transform; the output is cropped to user_out
  bool padded = false;
  int user_shape[2] = {1, 1};  // 2-D (rows, cols); 1-D (1, n)
  int user_out[2] = {1, 1};
  std::vector<size_t> taps_off;  // tree: spatial taps of the lowpass along a column, per res
  // 1-D, second order: the nodes of child octave j2 under ALL parent octaves j1 < j2 go through
  // one column launch and one lowpass launch, numbered (signal, j1, k); chan1d_off[j2] -> the
  // j2 * Q output channels (minus one: channel 0 is kept apart) of that numbering in d_chan1d
  int *d_chan1d = nullptr;
  std::vector<size_t> chan1d_off;
};

namespace {

using scat::ChanMap;
using scat::FilterTable;

// ---- scratch of scat_forward_static: one array per GPU in the library's device image, for
// callers that may not allocate.  Host code never uses the array's name as an address: the
// device address is looked up once per device (static_scratch_ptr) and passed to the
// schedules like any other scratch pointer.
constexpr size_t kStaticScratchBytes = size_t(SCAT_STATIC_SCRATCH_MB) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
void *g_static_ptr[kMaxDevices] = {};

// Device address of `scratch` on the CURRENT device (`dev`), looked up on first use.
scat_status static_scratch_ptr(int dev, void **out) {
  if (dev < 0 || dev >= kMaxDevices) return SCAT_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (g_static_ptr[dev] == nullptr) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
      (void)hipGetLastError();
      return SCAT_ERR_DEVICE;
    }
    g_static_ptr[dev] = ptr;
  }
  *out = g_static_ptr[dev];
  return SCAT_OK;
}

// Set-up step of every device plan: remember where `scratch` lives on the plan's device.
scat_status note_static_scratch(scat_plan *p) { return static_scratch_ptr(p->device, &p->static_scratch); }


// Bytes of scratch one chunk of planes may use (a forward call walks the batch in chunks).
// SCAT_SCRATCH_MB in the environment overrides the default of 12 GiB.
size_t scratch_budget() {
  static const size_t v = [] {
    const char *e = std::getenv("SCAT_SCRATCH_MB");
    long mb = e ? std::atol(e) : 0;
    return mb > 0 ? static_cast<size_t>(mb) << 20 : size_t(12) << 30;
  }();
  return v;
}

struct Layout {
  long chunk = 0;       // planes per chunk
  size_t per_plane = 0; // scratch bytes per plane
  // element offsets are expressed per plane; buffers are laid out chunk-major
  size_t xh = 0, t = 0, u = 0, v = 0, w = 0;  // per-plane sizes in bytes
  size_t pad_in = 0, pad_out = 0;             // padded plans: extended input, uncropped output
};

size_t bytes_per_volume_3d(const scat_plan &p);

// 1-D: elements per signal of the row-pass output buffer T.  It first holds one octave's Q
// first-order signals (consumed by the column pass) and then, at once, that octave's
// second-order row-pass outputs of all coarser octaves.
size_t t_elems_1d(const scat::HostPlan &h, size_t n) {
  size_t most = 0;
  for (int j1 = 0; j1 < h.J; ++j1) {
    size_t first = n >> h.res(j1), kids = 0;
    if (h.max_order == 2)
      for (int j2 = j1 + 1; j2 < h.J; ++j2) kids += n >> h.res(j2);
    most = std::max(most, std::max(first, kids));
  }
  return most * static_cast<size_t>(h.LQ);
}

// 1-D forward pass (no tape): elements per signal of the second-order row-pass outputs, kept
// for ALL parent octaves and grouped by child octave j2 (j2 * Q signals of n >> res(j2)
// elements each).
size_t kids_elems_1d(const scat::HostPlan &h, size_t n) {
  size_t all = 0;
  for (int j2 = 1; h.max_order == 2 && j2 < h.J; ++j2) all += static_cast<size_t>(j2) * h.LQ * (n >> h.res(j2));
  return all;
}

// budget: bytes of scratch one chunk may use (0 = scratch_budget())
Layout make_layout(const scat_plan &p, long batch, size_t budget = 0) {
  Layout L;
  if (budget == 0) budget = scratch_budget();
  const scat::HostPlan &h = p.host;
  if (h.dims == 3) {
    L.per_plane = bytes_per_volume_3d(p);
    if (p.padded) {
      // extended input and uncropped output behind the transform's buffers
      L.pad_in = p.h3.points() * sizeof(float);
      L.pad_out = static_cast<size_t>(h.K) * (p.h3.points() >> (3 * p.h3.out_shift())) * sizeof(float);
      L.xh = L.per_plane;  // offset of those two per volume
      L.per_plane += L.pad_in + L.pad_out;
    }
    long c = static_cast<long>(budget / L.per_plane);
    if (c < 1) c = 1;
    L.chunk = c > batch ? batch : c;
    return L;
  }
  const size_t n = static_cast<size_t>(p.n1) * p.n2;
  const bool second = h.max_order == 2 && h.J >= 2;
  const size_t c8 = sizeof(float2);
  if (h.dims == 2 && p.tree) {
    // xh: spectra of x; everything else stays in LDS
    L.xh = n * c8;
  } else if (h.dims == 2 && p.node) {
    // xh: spectrum of x; u: half spectra of one octave's first-order moduli (the first
    // octave of a 256 x 256 image as four polyphase components each); w: that octave's four
    // partial lowpass outputs per node
    const size_t l = h.LQ;
    L.xh = n * c8;
    size_t most = 0;
    for (int j = 0; second && j + 1 < h.J; ++j) {
      const size_t M1 = static_cast<size_t>(p.n1) >> j;
      const size_t per = M1 > 128 ? 4 * (M1 / 4 + 1) * (M1 / 2) : (M1 / 2 + 1) * M1;
      most = std::max(most, l * per);
    }
    L.u = most * c8;
    L.w = p.n1 > 128 ? l * 4 * 32 * 32 * sizeof(float) : 0;
  } else if (h.dims == 2 && p.fused) {
    // xh: column spectra of x; t: first-order row-pass outputs of all octaves at once
    // (sum over j of L*n/4^j); u: column spectra of one octave's moduli; v: second-order
    // row-pass outputs of all child octaves of one first-order octave
    const size_t l = h.LQ;
    L.xh = n * c8;
    size_t t1 = 0;
    for (int j = 0; j < h.J; ++j) t1 += l * (n >> (2 * h.res(j)));
    L.t = t1 * c8;
    L.u = second ? l * n * c8 : 0;
    size_t t2 = 0;
    for (int j = 1; j < h.J; ++j) t2 += l * l * (n >> (2 * h.res(j)));
    L.v = second ? t2 * c8 : 0;
    const size_t m_r = p.n1 >> h.res(h.J);
    size_t w0 = l * m_r * p.n2;
    size_t w2 = second ? l * l * m_r * (p.n2 >> h.res(1)) : 0;
    L.w = (w0 > w2 ? w0 : w2) * sizeof(float);
  } else if (h.dims == 2) {
    const size_t l = h.LQ;
    L.xh = n * c8;
    size_t t1 = l * n, t2 = second ? l * l * (n >> (2 * h.res(1))) : 0;
    L.t = (t1 > t2 ? t1 : t2) * c8;
    L.u = second ? l * n * c8 : 0;
    L.v = 0;
    const size_t m_r = p.n1 >> h.res(h.J);
    size_t w0 = l * m_r * p.n2;                       // first order at octave 0
    size_t w2 = second ? l * l * m_r * (p.n2 >> h.res(1)) : 0;  // second order at octave 1
    L.w = (w0 > w2 ? w0 : w2) * sizeof(float);
  } else {
    // t: see t_elems_1d; u: one octave's moduli (column spectra); v: one second-order
    // level's; w: row-pass outputs of the lowpass for all K channels
    const size_t q = h.LQ;
    L.xh = n * c8;
    // t: the first-order row-pass outputs of all octaves, then the second-order ones grouped
    // by child octave; u, v: their column spectra, laid out alike
    const size_t kids = kids_elems_1d(h, n);
    size_t first = 0;
    for (int j = 0; j < h.J; ++j) first += q * (n >> h.res(j));
    L.t = (first + kids) * c8;
    L.u = first * c8;
    L.v = kids * c8;
    L.w = static_cast<size_t>(h.K) * (n >> h.res(h.J)) * c8;
  }
  if (p.padded) {
    L.pad_in = n * sizeof(float);
    const size_t m_r = h.dims == 2 ? h.shape[0] >> h.res(h.J) : 1;
    L.pad_out = static_cast<size_t>(h.K) * m_r * (h.shape[1] >> h.res(h.J)) * sizeof(float);
  }
  L.per_plane = L.xh + L.t + L.u + L.v + L.w + L.pad_in + L.pad_out;
  long c = static_cast<long>(budget / L.per_plane);
  if (c < 1) c = 1;
  if (c > batch) c = batch;
  L.chunk = c;
  return L;
}

void free_device(scat_plan *p) {
  if (p->d_tables) (void)hipFree(p->d_tables);
  if (p->d_tw) (void)hipFree(p->d_tw);
  if (p->d_scratch) (void)hipFree(p->d_scratch);
  if (p->d_masks64) (void)hipFree(p->d_masks64);
  p->d_masks64 = nullptr;
  if (p->d_lane_masks) (void)hipFree(p->d_lane_masks);
  p->d_lane_masks = nullptr;
  if (p->d_chan1d) (void)hipFree(p->d_chan1d);
  p->d_chan1d = nullptr;
  p->d_tables = nullptr;
  p->d_tw = nullptr;
  p->d_scratch = nullptr;
  p->scratch_bytes = 0;
}

// Append one table in the kernels' layout, scaled by 1 / (number of grid points).
size_t append_table(std::vector<float> &pool, const FilterTable &t, int dims, int n1) {
  const size_t off = pool.size();
  const size_t cnt = t.v.size();
  const double scale = 1.0 / static_cast<double>(cnt);
  pool.resize(off + cnt);
  if (dims == 2) {
    for (size_t i = 0; i < cnt; ++i) pool[off + i] = static_cast<float>(t.v[i] * scale);
  } else {
    // four-step layout: [k1][k2] holds frequency k1 + n1 * k2
    const size_t cols = cnt / n1;
    for (size_t k1 = 0; k1 < static_cast<size_t>(n1); ++k1)
      for (size_t k2 = 0; k2 < cols; ++k2)
        pool[off + k1 * cols + k2] = static_cast<float>(t.v[k1 + n1 * k2] * scale);
  }
  return off;
}

// Activity words of the threads of k_node<64, 2, P> (groups = 8: 256 threads) or k_node_pair
// (groups = 16: 512 threads) for one table `ft` in those kernels'
// layout [row][column block][column parity][column pair][component]: thread (st, cq) =
// (tid / 32, tid % 32) takes source rows st + groups i, i < 64 / groups; bits 4 i + ac: the table values
// of the direct part of column block ac (both parities, all components) are not all negligible;
// bits 4 i + 2 + ac: the same for the part it adds to the mirrored row (row 0: to row 64).
// The index arithmetic is the kernel's own.
void lane_words_64(const float *ft, int P, int groups, std::vector<unsigned> &out) {
  const int S = 128;
  double peak = 0.0;
  for (size_t i = 0; i < static_cast<size_t>(P) * S * S; ++i) peak = std::max(peak, std::fabs(static_cast<double>(ft[i])));
  const double thr = 1e-7 * peak;
  auto live = [&](int entry) {
    for (int q = 0; q < P; ++q)
      if (std::fabs(static_cast<double>(ft[static_cast<size_t>(entry) * P + q])) > thr) return true;
    return false;
  };
  for (int tid = 0; tid < 32 * groups; ++tid) {
    const int cq = tid & 31, st = tid >> 5;
    unsigned w = 0;
    for (int i = 0; i < 64 / groups; ++i) {
      const int row = st + groups * i;
      const bool first = row == 0;
      const int row2 = first ? 64 : S - row;
      for (int ac = 0; ac < 2; ++ac)
        for (int e = 0; e < 2; ++e) {
          const int idx = first ? 32 * ac + cq : (64 - 32 * ac - cq - e) & 63;
          if (live(((row * 2 + ac) * 2 + e) * 32 + cq)) w |= 1u << (4 * i + ac);
          if (live(((row2 * 2 + (idx >> 5)) * 2 + e) * 32 + (idx & 31))) w |= 1u << (4 * i + 2 + ac);
        }
    }
    out.push_back(w);
  }
}

size_t append_vec(std::vector<float> &pool, const std::vector<double> &v) {
  const size_t off = pool.size();
  const double scale = 1.0 / static_cast<double>(v.size());
  for (double d : v) pool.push_back(static_cast<float>(d * scale));
  return off;
}

scat_status upload(scat_plan *p) {
  const scat::HostPlan &h = p->host;
  std::vector<float> pool;
  p->psi1_off.assign(h.J, 0);
  for (int j = 0; j < h.J; ++j)
    for (int l = 0; l < h.LQ; ++l) {
      size_t off = append_table(pool, *h.find(1, j * h.LQ + l, 0), h.dims, p->n1);
      if (l == 0) p->psi1_off[j] = off;
    }
  if (h.max_order == 2) {
    for (int j2 = 1; j2 < h.J; ++j2)
      for (int r = 0; r < j2; ++r) {
        if (h.dims == 2) {
          if (r == 0) {
            p->psi2_off[{0, j2}] = p->psi1_off[j2];
            continue;
          }
          for (int l = 0; l < h.LQ; ++l) {
            size_t off = append_table(pool, *h.find(2, j2 * h.LQ + l, r), 2, p->n1);
            if (l == 0) p->psi2_off[{r, j2}] = off;
          }
        } else {
          p->psi2_off[{r, j2}] = append_table(pool, *h.find(2, j2, r), 1, p->n1);
        }
      }
  }
  if (h.dims == 2) {
    for (int r = 0; r < h.J; ++r) {
      p->phi_rows_off.push_back(append_vec(pool, h.phi_rows[r]));
      p->phi_cols_off.push_back(append_vec(pool, h.phi_cols[r]));
    }
  } else {
    for (int r = 0; r < h.J; ++r)
      p->phi_off.push_back(append_table(pool, *h.find(0, 0, r), 1, p->n1));
  }
  if (p->tree) {
    // the lowpass along a column as spatial taps: g[m] = sum_k phi[k] / len * cos(2 pi k m / len)
    // (phi is even, so the inverse transform is real)
    const double two_pi_ = 6.283185307179586476925286766559;
    for (int r = 0; r < h.J; ++r) {
      const std::vector<double> &ph = h.phi_rows[r];
      const size_t len = ph.size();
      p->taps_off.push_back(pool.size());
      for (size_t m = 0; m < len; ++m) {
        double acc = 0.0;
        for (size_t k = 0; k < len; ++k) acc += ph[k] * std::cos(two_pi_ * static_cast<double>((k * m) % len) / len);
        pool.push_back(static_cast<float>(acc / static_cast<double>(len)));
      }
    }
  }
  if (h.dims == 2 && !p->tree && h.oversampling == 0) {
    // alias blocks of (n1 >> j) x (n2 >> j) points on which a wavelet of octave j stays below
    // 1e-7 of its peak: skipped by the row pass of the general schedule
    std::vector<unsigned long long> m64;
    for (int j = 1; j < h.J; ++j)
      for (int r = 0; r < j; ++r) {
        if (r > 0 && h.max_order < 2) continue;
        const int sr = p->n1 >> r, sc = p->n2 >> r;
        const int br = p->n1 >> j, bc = p->n2 >> j;
        if (br < 1 || bc < 1) continue;
        const int Ar = sr / br, Ac = sc / bc;
        if (Ar * Ac > 64 || Ar * Ac < 2) continue;
        p->mask64_off[{r, j}] = m64.size();
        for (int l = 0; l < h.LQ; ++l) {
          const FilterTable &t = *h.find(r == 0 ? 1 : 2, j * h.LQ + l, r);
          double peak = 0.0;
          for (double v : t.v) peak = std::max(peak, std::fabs(v));
          unsigned long long m = 0;
          for (int ar = 0; ar < Ar; ++ar)
            for (int ac = 0; ac < Ac; ++ac) {
              double big = 0.0;
              for (int i = 0; i < br; ++i)
                for (int k = 0; k < bc; ++k)
                  big = std::max(big, std::fabs(t.v[static_cast<size_t>(ar * br + i) * sc + ac * bc + k]));
              if (big > 1e-7 * peak) m |= 1ull << (ar * Ac + ac);
            }
          m64.push_back(m);
        }
      }
    if (!m64.empty()) {
      if (hipMalloc(&p->d_masks64, m64.size() * sizeof(unsigned long long)) != hipSuccess) return SCAT_ERR_ALLOC;
      if (hipMemcpy(p->d_masks64, m64.data(), m64.size() * sizeof(unsigned long long),
                    hipMemcpyHostToDevice) != hipSuccess)
        return SCAT_ERR_DEVICE;
    }
  }
  if (h.dims == 1 && h.oversampling == 0) {
    // 1-D, first order: the row pass folds the second digit of the four-step frequency index
    // only, so alias block b of octave j is the band [b, b + 1) N / 2^j of frequencies
    std::vector<unsigned long long> m64;
    const size_t N = static_cast<size_t>(p->n1) * p->n2;
    for (int j = 1; j < h.J && j <= 6; ++j) {
      const size_t band = N >> j;
      if (band < 1 || (static_cast<size_t>(p->n2) >> j) < 1) continue;
      p->mask64_off[{0, j}] = m64.size();
      for (int q = 0; q < h.LQ; ++q) {
        const FilterTable &t = *h.find(1, j * h.LQ + q, 0);
        double peak = 0.0;
        for (double v : t.v) peak = std::max(peak, std::fabs(v));
        unsigned long long m = 0;
        for (int b = 0; b < (1 << j); ++b) {
          double big = 0.0;
          for (size_t k = b * band; k < (b + 1) * band; ++k) big = std::max(big, std::fabs(t.v[k]));
          if (big > 1e-7 * peak) m |= 1ull << b;
        }
        m64.push_back(m);
      }
    }
    // the lowpass at full resolution, folded by 2^J (key {-1, J})
    if (h.J >= 1 && h.J <= 6 && (static_cast<size_t>(p->n2) >> h.J) >= 1) {
      const size_t band = N >> h.J;
      const FilterTable &t = *h.find(0, 0, 0);
      double peak = 0.0;
      for (double v : t.v) peak = std::max(peak, std::fabs(v));
      unsigned long long m = 0;
      for (int b = 0; b < (1 << h.J); ++b) {
        double big = 0.0;
        for (size_t k = b * band; k < (b + 1) * band; ++k) big = std::max(big, std::fabs(t.v[k]));
        if (big > 1e-7 * peak) m |= 1ull << b;
      }
      p->mask64_off[{-1, h.J}] = m64.size();
      m64.push_back(m);
    }
    if (!m64.empty()) {
      if (hipMalloc(&p->d_masks64, m64.size() * sizeof(unsigned long long)) != hipSuccess) return SCAT_ERR_ALLOC;
      if (hipMemcpy(p->d_masks64, m64.data(), m64.size() * sizeof(unsigned long long),
                    hipMemcpyHostToDevice) != hipSuccess)
        return SCAT_ERR_DEVICE;
    }
  }
  if (p->node_taps) {
    const int N = p->n1;
    const double two_pi_ = 6.283185307179586476925286766559;
    // spatial taps of a lowpass factor: g[d] = (1/len) sum_k phi[k] cos(2 pi k d / len)
    auto spatial = [&](const std::vector<double> &ph) {
      const size_t len = ph.size();
      std::vector<double> g(len);
      for (size_t d = 0; d < len; ++d) {
        double acc = 0.0;
        for (size_t k = 0; k < len; ++k) acc += ph[k] * std::cos(two_pi_ * static_cast<double>((k * d) % len) / len);
        g[d] = acc / static_cast<double>(len);
      }
      return g;
    };
    auto push_taps = [&](const std::vector<double> &g, int R, int stride, int shift) {
      // taps[d + R] = g[(stride d - shift) mod len], |d| <= R
      const long len = static_cast<long>(g.size());
      const size_t off = pool.size();
      for (int d = -R; d <= R; ++d) {
        long i = (static_cast<long>(stride) * d - shift) % len;
        if (i < 0) i += len;
        pool.push_back(static_cast<float>(g[i]));
      }
      return off;
    };
    p->taps_r_off.assign(h.J, 0);
    p->taps_c_off.assign(h.J, 0);
    for (int r = 0; r < h.J; ++r) {
      const int len = N >> r;
      if (len > 256) continue;  // no whole-node kernel for such nodes
      const std::vector<double> gr = spatial(h.phi_rows[r]), gc = spatial(h.phi_cols[r]);
      if (len > 128) {
        // components of len/2 points: taps phi[2 d - p], p = 0, 1
        const int R = 4 * (len / 2 / 32);
        p->ptaps_r_off = push_taps(gr, R, 2, 0);
        push_taps(gr, R, 2, 1);
        p->ptaps_c_off = push_taps(gc, R, 2, 0);
        push_taps(gc, R, 2, 1);
      } else {
        const int R = 4 * (len / 32);
        p->taps_r_off[r] = push_taps(gr, R, 1, 0);
        p->taps_c_off[r] = push_taps(gc, R, 1, 0);
      }
    }
    if (p->node_tables) {
      std::vector<std::pair<int, int>> want;
      if (N > 128) want.push_back({0, 0});
      for (int r = 0; r + 1 < h.J; ++r)
        if (r == 0 || h.max_order == 2) want.push_back({r, r + 1});
      for (const auto &rj : want) {
        const int r = rj.first, j = rj.second;
        const int side = N >> r, M = side / 2;
        if (M != 64 && M != 128) continue;
        const double scale = 1.0 / (static_cast<double>(side) * side);
        while (pool.size() % 4 != 0) pool.push_back(0.f);
        p->node2_off[rj] = pool.size();
        for (int l = 0; l < h.LQ; ++l) {
          const FilterTable &t = *h.find(r == 0 ? 1 : 2, j * h.LQ + l, r);
          if (M == 128) {
            for (int kr = 0; kr < side; ++kr)
              for (int cp = 0; cp < M / 2; ++cp)
                for (int ac = 0; ac < 2; ++ac)
                  for (int e = 0; e < 2; ++e) {
                    const int c = M * ac + 2 * cp + e;
                    const int col = kr <= side / 2 ? c : (side - c) & (side - 1);
                    pool.push_back(static_cast<float>(t.v[static_cast<size_t>(kr) * side + col] * scale));
                  }
          } else {
            for (int kr = 0; kr < side; ++kr)
              for (int ac = 0; ac < 2; ++ac)
                for (int e = 0; e < 2; ++e)
                  for (int cp = 0; cp < M / 2; ++cp)
                    pool.push_back(static_cast<float>(
                        t.v[static_cast<size_t>(kr) * side + M * ac + 2 * cp + e] * scale));
          }
        }
        // the entry that lanes with nothing to fetch read instead (lane_words_64)
        for (int z = 0; z < 4; ++z) pool.push_back(0.f);
      }
    }
    if (p->node && N > 128 && h.max_order == 2) {
      // children of the polyphase octave: R_q[k] = sum_a (-1)^(a.q) psi[k + M a], M = N/2
      const int M = N / 2;
      const double scale = 1.0 / (static_cast<double>(N) * N);
      for (int j2 = 1; j2 < h.J; ++j2) {
        while (pool.size() % 4 != 0) pool.push_back(0.f);  // 16-byte loads of the table
        p->poly_psi_off[j2] = pool.size();
        for (int l = 0; l < h.LQ; ++l) {
          const FilterTable &t = *h.find(1, j2 * h.LQ + l, 0);
          auto folded = [&](int q, int kr, int kc) {
            const int qr = q >> 1, qc = q & 1;
            double acc = 0.0;
            for (int ar = 0; ar < 2; ++ar)
              for (int ac = 0; ac < 2; ++ac) {
                const double v = t.v[static_cast<size_t>(kr + M * ar) * N + kc + M * ac];
                acc += ((ar * qr + ac * qc) & 1) ? -v : v;
              }
            return static_cast<float>(acc * scale);
          };
          if ((N >> j2) == M) {
            // children as large as a component: [row][column parity][column pair][component],
            // the four component values of a point side by side (one 16-byte load)
            // rows above M / 2 are only read for mirrored parts (the stored half spectra have
            // W_q[M - r][-c] = s_q(c) conj(W_q[r][c])): they hold s_q(c) R_q[row][-c] at c's place
            for (int kr = 0; kr < M; ++kr)
              for (int e = 0; e < 2; ++e)
                for (int cp = 0; cp < M / 2; ++cp)
                  for (int q = 0; q < 4; ++q) {
                    const int c = 2 * cp + e;
                    if (kr <= M / 2) {
                      pool.push_back(folded(q, kr, c));
                    } else {
                      const bool neg = ((q >> 1) & 1) ^ ((q & 1) & (c != 0 ? 1 : 0));
                      const float v = folded(q, kr, (M - c) & (M - 1));
                      pool.push_back(neg ? -v : v);
                    }
                  }
          } else if ((N >> j2) == M / 2) {
            // children half as large: [row][column block][column parity][column pair][component]
            for (int kr = 0; kr < M; ++kr)
              for (int ac = 0; ac < 2; ++ac)
                for (int e = 0; e < 2; ++e)
                  for (int cp = 0; cp < M / 4; ++cp)
                    for (int q = 0; q < 4; ++q) pool.push_back(folded(q, kr, (M / 2) * ac + 2 * cp + e));
          } else {
            for (int q = 0; q < 4; ++q)
              for (int kr = 0; kr < M; ++kr)
                for (int kc = 0; kc < M; ++kc) pool.push_back(folded(q, kr, kc));
          }
        }
        for (int z = 0; z < 4; ++z) pool.push_back(0.f);  // see above
      }
    }
  }
  if (h.dims == 1 && h.max_order == 2 && h.J >= 2) {
    std::vector<int> chans;
    p->chan1d_off.assign(h.J, 0);
    for (int j2 = 1; j2 < h.J; ++j2) {
      p->chan1d_off[j2] = chans.size();
      int s2_base = 1 + h.J * h.LQ;
      for (int j1 = 0; j1 < j2; ++j1) {
        const int octs = h.J - 1 - j1;
        for (int k = 0; k < h.LQ; ++k) chans.push_back(s2_base + k * octs + (j2 - j1 - 1) - 1);
        s2_base += h.LQ * octs;
      }
    }
    if (hipMalloc(&p->d_chan1d, chans.size() * sizeof(int)) != hipSuccess) return SCAT_ERR_ALLOC;
    if (hipMemcpy(p->d_chan1d, chans.data(), chans.size() * sizeof(int), hipMemcpyHostToDevice) != hipSuccess)
      return SCAT_ERR_DEVICE;
  }
  if (p->node_taps) {
    std::vector<unsigned> words;
    for (const auto &kv : p->node2_off) {
      const int side = p->n1 >> kv.first.first;
      if (side != 128) continue;  // tables of k_node<64, 2, 1>
      p->lane_mask_off[kv.first] = words.size();
      for (int l = 0; l < h.LQ; ++l)
        lane_words_64(pool.data() + kv.second + static_cast<size_t>(l) * side * side, 1, 8, words);
    }
    for (const auto &kv : p->poly_psi_off) {
      const int M = p->n1 / 2;
      if ((p->n1 >> kv.first) != M / 2 || M != 128) continue;  // tables of k_node<64, 2, 4>
      p->lane_mask_off[{-1, kv.first}] = words.size();
      for (int l = 0; l < h.LQ; ++l)
        lane_words_64(pool.data() + kv.second + static_cast<size_t>(l) * 4 * M * M, 4, h.LQ % 2 == 0 ? 16 : 8, words);
    }
    if (!words.empty()) {
      if (hipMalloc(&p->d_lane_masks, words.size() * sizeof(unsigned)) != hipSuccess) return SCAT_ERR_ALLOC;
      if (hipMemcpy(p->d_lane_masks, words.data(), words.size() * sizeof(unsigned), hipMemcpyHostToDevice) !=
          hipSuccess)
        return SCAT_ERR_DEVICE;
    }
  }
  // twiddles exp(-2 pi i j / tw_n), evaluated in double
  p->tw_n = h.dims == 2 ? (p->n1 > p->n2 ? p->n1 : p->n2) : p->n1 * p->n2;
  std::vector<float2> tw(p->tw_n);
  const double two_pi = 6.283185307179586476925286766559;
  for (int j = 0; j < p->tw_n; ++j) {
    double a = -two_pi * j / p->tw_n;
    tw[j] = make_float2(static_cast<float>(std::cos(a)), static_cast<float>(std::sin(a)));
  }
  if (hipGetDevice(&p->device) != hipSuccess) return SCAT_ERR_DEVICE;
  if (hipMalloc(&p->d_tables, pool.size() * sizeof(float)) != hipSuccess) return SCAT_ERR_ALLOC;
  if (hipMalloc(&p->d_tw, tw.size() * sizeof(float2)) != hipSuccess) return SCAT_ERR_ALLOC;
  if (hipMemcpy(p->d_tables, pool.data(), pool.size() * sizeof(float), hipMemcpyHostToDevice) !=
      hipSuccess)
    return SCAT_ERR_DEVICE;
  if (hipMemcpy(p->d_tw, tw.data(), tw.size() * sizeof(float2), hipMemcpyHostToDevice) !=
      hipSuccess)
    return SCAT_ERR_DEVICE;
  p->has_device = true;
  return note_static_scratch(p);
}

// Activity words of the table `key` (scat_plan::lane_mask_off), or null: every load is made
const unsigned *lane_mask_of(const scat_plan *p, std::pair<int, int> key) {
  auto it = p->lane_mask_off.find(key);
  return (p->d_lane_masks != nullptr && it != p->lane_mask_off.end()) ? p->d_lane_masks + it->second : nullptr;
}

scat_status upload_3d(scat_plan *p);

// 3-D solid harmonic plan: LQ is the largest degree L (degrees 0 .. L).
scat_status create_3d(scat_plan **out_plan, const int *user_shape, int J, int L, int max_order,
                      bool device, bool padded, int oversampling) {
  int grid[3];
  const int *shape = user_shape;
  if (padded) {
    // periodic grid: smallest power of two >= n + 2^J per axis
    if (J < 1 || J > 8) return SCAT_ERR_ARG;
    for (int d = 0; d < 3; ++d) {
      if (user_shape[d] < 1 || user_shape[d] > 256) return SCAT_ERR_SHAPE;
      int g = 1;
      while (g < user_shape[d] + (1 << J)) g *= 2;
      grid[d] = g;
    }
    shape = grid;
  }
  int v = scat::validate_3d(shape, J, L, max_order);
  if (v != 0) return static_cast<scat_status>(v);
  scat_plan *p = new (std::nothrow) scat_plan;
  if (p == nullptr) return SCAT_ERR_ALLOC;
  try {
    scat::build_host_plan_3d(p->h3, shape, J, L, max_order);
  } catch (const std::bad_alloc &) {
    delete p;
    return SCAT_ERR_ALLOC;
  }
  p->h3.oversampling = oversampling;
  p->host.dims = 3;
  p->host.J = J;
  p->host.LQ = L;
  p->host.max_order = max_order;
  p->host.K = p->h3.K;
  p->host.oversampling = oversampling;
  const int Jo = p->h3.out_shift();
  p->fused3 = scat::fused3_supported(shape[0], shape[1], shape[2], Jo);
  if (padded) {
    p->padded = true;
    for (int d = 0; d < 3; ++d) {
      p->user_shape3[d] = user_shape[d];
      p->user_out3[d] = (user_shape[d] + (1 << Jo) - 1) >> Jo;
    }
  }
  if (device) {
    scat_status s;
    try {
      s = upload_3d(p);
    } catch (const std::bad_alloc &) {
      s = SCAT_ERR_ALLOC;
    }
    if (s != SCAT_OK) {
      free_device(p);
      delete p;
      return s;
    }
  }
  *out_plan = p;
  return SCAT_OK;
}

scat_status create_common(scat_plan **out_plan, int dims, const int *user_shape, int J, int LQ,
                          int max_order, bool device, bool padded = false, int oversampling = 0,
                          bool node_kernels = true) {
  if (out_plan == nullptr) return SCAT_ERR_NULL;
  *out_plan = nullptr;
  if (user_shape == nullptr) return SCAT_ERR_NULL;
  if (oversampling < 0 || oversampling > 24) return SCAT_ERR_ARG;
  if (dims == 3) return create_3d(out_plan, user_shape, J, LQ, max_order, device, padded, oversampling);
  int grid[2] = {1, 1};
  const int *shape = user_shape;
  if (padded) {
    // periodic grid: smallest power of two >= n + 2^J per axis
    if ((dims != 1 && dims != 2) || J < 1 || J > 24) return SCAT_ERR_ARG;
    for (int d = 0; d < dims; ++d) {
      if (user_shape[d] < 1 || user_shape[d] > (1 << 24)) return SCAT_ERR_SHAPE;
      long need = static_cast<long>(user_shape[d]) + (1L << J), g = 1;
      while (g < need) g *= 2;
      if (g > (1L << 24)) return SCAT_ERR_SHAPE;
      grid[d] = static_cast<int>(g);
    }
    shape = grid;
  }
  int v = scat::validate(dims, shape, J, LQ, max_order);
  if (v != 0) return static_cast<scat_status>(v);
  scat_plan *p = new (std::nothrow) scat_plan;
  if (p == nullptr) return SCAT_ERR_ALLOC;
  try {
    scat::build_host_plan(p->host, dims, shape, J, LQ, max_order);
    p->host.oversampling = oversampling;
  } catch (const std::bad_alloc &) {
    delete p;
    return SCAT_ERR_ALLOC;
  }
  if (dims == 2) {
    p->n1 = shape[0];
    p->n2 = shape[1];
  } else {
    // four-step split N = n1 * n2 with n2 >= 2^J (folds act on the n2 digit only) and
    // both factors as close to sqrt(N) as that allows
    int lg = 0;
    while ((1 << lg) < shape[0]) ++lg;
    int lg2 = (lg + 1) / 2;
    if (lg2 < J) lg2 = J;
    p->n2 = 1 << lg2;
    p->n1 = shape[0] >> lg2;
  }
  // fused row pass: every launch of the schedule must be one the kernel takes -- the first
  // order from the image itself and, per octave with children, from that octave's grid
  p->fused = dims == 2 && J <= 4 && scat::rows_fused_supported(p->n1, p->n2, p->host.res(J - 1));
  if (p->fused && max_order == 2)
    for (int j1 = 0; j1 + 1 < J; ++j1) {
      const int r1 = p->host.res(j1);
      if (!scat::rows_fused_supported(p->n1 >> r1, p->n2 >> r1, p->host.res(J - 1) - r1))
        p->fused = false;
    }
  p->tree = dims == 2 && oversampling == 0 && scat::tree_supported(p->n1, p->n2, J);
  // whole-node kernels: square grids whose octaves are 128 or 64 points a side, or 256 as four
  // polyphase components, with the 32 x 32 output grid their lowpass stage is laid out for
  p->node_tables = dims == 2 && oversampling == 0 && p->n1 == p->n2 &&
                   ((p->n1 == 256 && J == 3) || (p->n1 == 128 && J == 2));
  p->node = node_kernels && p->node_tables;
  p->node_taps = dims == 2 && oversampling == 0 && p->n1 == p->n2 && J < 31 && (p->n1 >> J) == 32;
  if (padded) {
    p->padded = true;
    for (int d = 0; d < dims; ++d) {
      const int k = dims == 2 ? d : 1;
      p->user_shape[k] = user_shape[d];
      const int rj = p->host.res(J);
      p->user_out[k] = (user_shape[d] + (1 << rj) - 1) >> rj;
    }
  }
  if (device) {
    scat_status s;
    try {
      s = upload(p);
    } catch (const std::bad_alloc &) {
      s = SCAT_ERR_ALLOC;
    }
    if (s != SCAT_OK) {
      free_device(p);
      delete p;
      return s;
    }
  }
  *out_plan = p;
  return SCAT_OK;
}

// Symmetric periodic extension of `planes` signals of n_r x n_c to P_r x P_c: the margin's
// first half mirrors the right/bottom edge, the rest mirrors the left/top edge of the next
// period, so the periodic signal has no jump; reflections repeat with period 2n.
__device__ __forceinline__ int pad_source(int i, int n, int P) {
  const int h = (P - n + 1) / 2;
  int v = i < n + h ? i : i - P;
  v %= 2 * n;
  if (v < 0) v += 2 * n;
  return v < n ? v : 2 * n - 1 - v;
}

__global__ __launch_bounds__(256) void k_pad_symmetric(const float *__restrict__ in,
                                                       float *__restrict__ out, long planes,
                                                       int n_r, int n_c, int P_r, int P_c) {
  const long total = planes * P_r * P_c;
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int c = static_cast<int>(i % P_c);
    const long t = i / P_c;
    const int r = static_cast<int>(t % P_r);
    const long p = t / P_r;
    out[i] = in[(p * n_r + pad_source(r, n_r, P_r)) * n_c + pad_source(c, n_c, P_c)];
  }
}

// 3-D versions of the symmetric extension and of the crop
__global__ __launch_bounds__(256) void k_pad_symmetric3(const float *__restrict__ in,
                                                        float *__restrict__ out, long volumes, int u0,
                                                        int u1, int u2, int P0, int P1, int P2) {
  const long per = static_cast<long>(P0) * P1 * P2;
  const long total = volumes * per;
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const long v = i / per;
    long e = i - v * per;
    const int c = static_cast<int>(e % P2);
    e /= P2;
    const int b = static_cast<int>(e % P1);
    const int a = static_cast<int>(e / P1);
    out[i] = in[((v * u0 + pad_source(a, u0, P0)) * u1 + pad_source(b, u1, P1)) * u2 +
                pad_source(c, u2, P2)];
  }
}

__global__ __launch_bounds__(256) void k_crop3(const float *__restrict__ in, float *__restrict__ out,
                                               long maps, int m0, int m1, int m2, int o0, int o1,
                                               int o2) {
  const long per = static_cast<long>(o0) * o1 * o2;
  const long total = maps * per;
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const long g = i / per;
    long e = i - g * per;
    const int c = static_cast<int>(e % o2);
    e /= o2;
    const int b = static_cast<int>(e % o1);
    const int a = static_cast<int>(e / o1);
    out[i] = in[((g * m0 + a) * m1 + b) * m2 + c];
  }
}

// out [planes*K][o_r][o_c] = in [planes*K][m_r][m_c] restricted to the top-left corner
__global__ __launch_bounds__(256) void k_crop(const float *__restrict__ in, float *__restrict__ out,
                                              long maps, int m_r, int m_c, int o_r, int o_c) {
  const long total = maps * o_r * o_c;
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int c = static_cast<int>(i % o_c);
    const long t = i / o_c;
    const int r = static_cast<int>(t % o_r);
    const long m = t / o_r;
    out[i] = in[(m * m_r + r) * m_c + c];
  }
}

// Adjoint of k_crop: out [maps][m_r][m_c] = in [maps][o_r][o_c] in the top-left corner, 0 elsewhere
__global__ __launch_bounds__(256) void k_uncrop(const float *__restrict__ in, float *__restrict__ out,
                                                long maps, int m_r, int m_c, int o_r, int o_c) {
  const long total = maps * m_r * m_c;
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int c = static_cast<int>(i % m_c);
    const long t = i / m_c;
    const int r = static_cast<int>(t % m_r);
    const long m = t / m_r;
    out[i] = (r < o_r && c < o_c) ? in[(m * o_r + r) * o_c + c] : 0.f;
  }
}

// Positions of the period-P extension that mirror sample r of n (see pad_source): virtual
// positions v = r + 2 n t and v = 2 n - 1 - r + 2 n t inside [-(P - n - h), n + h), stored
// at v (v >= 0) or v + P.  Calls f(position) for each.
template <class Fn>
__device__ __forceinline__ void for_each_image(int r, int n, int P, Fn f) {
  const int h = (P - n + 1) / 2, lo = P - n - h;
  const int reps = P / (2 * n) + 1;
  for (int t = -reps; t <= reps; ++t) {
    const int v0 = r + 2 * n * t, v1 = 2 * n - 1 - r + 2 * n * t;
    if (v0 >= -lo && v0 < n + h) f(v0 >= 0 ? v0 : v0 + P);
    if (v1 >= -lo && v1 < n + h) f(v1 >= 0 ? v1 : v1 + P);
  }
}

// Adjoint of k_pad_symmetric: every sample collects the gradients of all its mirror images.
__global__ __launch_bounds__(256) void k_unpad_symmetric(const float *__restrict__ gp,
                                                         float *__restrict__ gx, long planes,
                                                         int n_r, int n_c, int P_r, int P_c) {
  const long total = planes * n_r * n_c;
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int c = static_cast<int>(i % n_c);
    const long t = i / n_c;
    const int r = static_cast<int>(t % n_r);
    const long p = t / n_r;
    const float *plane = gp + p * P_r * P_c;
    float acc = 0.f;
    for_each_image(r, n_r, P_r, [&](int ir) {
      for_each_image(c, n_c, P_c, [&](int ic) { acc += plane[static_cast<size_t>(ir) * P_c + ic]; });
    });
    gx[i] = acc;
  }
}

// 3-D versions: adjoint of k_crop3 (zero extension) and of k_pad_symmetric3
__global__ __launch_bounds__(256) void k_uncrop3(const float *__restrict__ in, float *__restrict__ out,
                                                 long maps, int m0, int m1, int m2, int o0, int o1,
                                                 int o2) {
  const long per = static_cast<long>(m0) * m1 * m2;
  const long total = maps * per;
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const long g = i / per;
    long e = i - g * per;
    const int c = static_cast<int>(e % m2);
    e /= m2;
    const int b = static_cast<int>(e % m1);
    const int a = static_cast<int>(e / m1);
    out[i] = (a < o0 && b < o1 && c < o2) ? in[((g * o0 + a) * o1 + b) * o2 + c] : 0.f;
  }
}

__global__ __launch_bounds__(256) void k_unpad_symmetric3(const float *__restrict__ gp,
                                                          float *__restrict__ gx, long volumes, int u0,
                                                          int u1, int u2, int P0, int P1, int P2) {
  const long per = static_cast<long>(u0) * u1 * u2;
  const long total = volumes * per;
  const long stride = static_cast<long>(gridDim.x) * blockDim.x;
  for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const long v = i / per;
    long e = i - v * per;
    const int c = static_cast<int>(e % u2);
    e /= u2;
    const int b = static_cast<int>(e % u1);
    const int a = static_cast<int>(e / u1);
    const float *vol = gp + v * static_cast<long>(P0) * P1 * P2;
    float acc = 0.f;
    for_each_image(a, u0, P0, [&](int ia) {
      for_each_image(b, u1, P1, [&](int ib) {
        for_each_image(c, u2, P2, [&](int ic) {
          acc += vol[(static_cast<size_t>(ia) * P1 + ib) * P2 + ic];
        });
      });
    });
    gx[i] = acc;
  }
}

unsigned stream_blocks(long total) {
  long b = (total + 255) / 256;
  if (b > 65536 * 16) b = 65536 * 16;
  return static_cast<unsigned>(b < 1 ? 1 : b);
}

#define SCAT_TRY(expr)                               \
  do {                                               \
    if ((expr) != hipSuccess) return SCAT_ERR_DEVICE; \
  } while (0)

// Where the backward pass keeps the complex signals before every modulus: per-plane element
// offsets into one array (chunk-major like all scratch: array of octave j1 starts at
// y1_off[j1] * planes_in_chunk).  Each signal is kept as the row pass leaves it, i.e. BEFORE
// its inverse column transform, which the backward kernels do themselves.
struct Tape {
  float2 *base = nullptr;
  std::vector<size_t> y1_off;                     // per j1: [planes*L][M1r][M1c]
  std::map<std::pair<int, int>, size_t> y2_off;   // per (j1, j2): [planes*L*L][M2r][M2c]
  size_t total = 0;                               // elements per plane
};

Tape make_tape(const scat_plan &p) {
  Tape t;
  const scat::HostPlan &h = p.host;
  const size_t n = static_cast<size_t>(p.n1) * p.n2, l = h.LQ;
  const int d = h.dims;  // grid points at resolution r: n >> (d r)
  size_t off = 0;
  for (int j1 = 0; j1 < h.J; ++j1) {
    t.y1_off.push_back(off);
    // (fused 2-D plans read the first-order signals of nodes with children from the forward
    // pass's own buffer: no tape slot)
    const bool kids = h.max_order == 2 && j1 < h.J - 1;
    if (!(d == 2 && p.fused && kids)) off += l * (n >> (d * h.res(j1)));
  }
  if (h.max_order == 2)
    for (int j1 = 0; j1 < h.J; ++j1)
      for (int j2 = j1 + 1; j2 < h.J; ++j2) {
        t.y2_off[{j1, j2}] = off;
        // 2-D: L*L children per (j1, j2); 1-D: one second-order wavelet per octave, Q parents
        off += (d == 2 ? l * l : l) * (n >> (d * h.res(j2)));
      }
  t.total = off;
  return t;
}

// ---- 2-D schedule for one chunk of `pc` planes starting at plane p0.  With a tape the
// signals before each modulus are kept (see Tape) and the outputs S are not formed (`out`
// unused).
scat_status forward_2d(scat_plan *p, const float *in, float *out, long p0, long pc,
                       const Layout &lay, hipStream_t st, const Tape *tape = nullptr) {
  const scat::HostPlan &h = p->host;
  const int J = h.J, L = h.LQ, K = h.K;
  const int Nr = p->n1, Nc = p->n2;
  const int rJ = h.res(J);
  const int m_r = Nr >> rJ, m_c = Nc >> rJ;
  char *base = static_cast<char *>(p->work);
  float2 *XH = reinterpret_cast<float2 *>(base);
  float2 *T = reinterpret_cast<float2 *>(base + lay.xh * pc);
  float2 *U = reinterpret_cast<float2 *>(base + (lay.xh + lay.t) * pc);
  float *W = reinterpret_cast<float *>(base + (lay.xh + lay.t + lay.u + lay.v) * pc);
  const float *tab = p->d_tables;
  const float2 *tw = p->d_tw;
  const int tw_n = p->tw_n;
  const float *x = in + static_cast<size_t>(p0) * Nr * Nc;
  float *o = out ? out + static_cast<size_t>(p0) * K * m_r * m_c : nullptr;
  const ChanMap none{1, 1, 0, 0};

  const bool lp = tape == nullptr;  // form the lowpassed outputs
  // x -> column spectra (+ column half of the lowpass for S0), then rows
  SCAT_TRY(scat::launch_col(0, x, pc, Nr, Nc, XH, 0, tab + p->phi_rows_off[0], m_r,
                            lp ? W : nullptr, nullptr, none, K, tw, tw_n, st));
  if (lp)
    SCAT_TRY(scat::launch_row_lowpass(W, pc, m_r, Nc, m_c, tab + p->phi_cols_off[0], o,
                                      ChanMap{1, 1, 0, 0}, K, tw, tw_n, st));
  SCAT_TRY(scat::launch_row_fwd(XH, pc * Nr, Nc, tw, tw_n, st));

  int s2_base = 1 + J * L;
  for (int j1 = 0; j1 < J; ++j1) {
    const int r1 = h.res(j1);
    const int M1r = Nr >> r1, M1c = Nc >> r1;
    const bool kids = h.max_order == 2 && j1 < J - 1;
    // Taped pass: every node is taped as its row pass leaves it, before the inverse column
    // transform (the backward kernels transform the columns themselves): the row pass writes
    // into the tape, a leaf needs no column kernel, a node with children only its spectra.
    float2 *t1 = tape ? tape->base + tape->y1_off[j1] * pc : T;
    auto mask_of = [&](int r, int j) -> const unsigned long long * {
      auto it = p->mask64_off.find({r, j});
      return (p->d_masks64 != nullptr && it != p->mask64_off.end() && h.res(j) == j && h.res(r) == r)
                 ? p->d_masks64 + it->second
                 : nullptr;
    };
    SCAT_TRY(scat::launch_mulfold_invrow(XH, tab + p->psi1_off[j1], t1, pc, L, Nr, Nc, r1, r1, 0,
                                         tw, tw_n, st, mask_of(0, j1)));
    if (tape != nullptr && !kids) continue;
    if (lp && !kids && scat::leaf_node_supported(M1r, M1c, m_r, m_c, tw_n)) {
      SCAT_TRY(scat::launch_leaf_node(t1, pc * L, M1r, m_r, tab + p->phi_rows_off[r1],
                                      tab + p->phi_cols_off[r1], o, ChanMap{L, L, 0, 1 + j1 * L}, K, tw,
                                      tw_n, st));
      continue;
    }
    SCAT_TRY(scat::launch_col(1, t1, pc * L, M1r, M1c, kids ? U : nullptr, 0,
                              tab + p->phi_rows_off[r1], m_r, lp ? W : nullptr, nullptr, none, K,
                              tw, tw_n, st));
    if (lp)
      SCAT_TRY(scat::launch_row_lowpass(W, pc * L, m_r, M1c, m_c, tab + p->phi_cols_off[r1], o,
                                        ChanMap{L, L, 0, 1 + j1 * L}, K, tw, tw_n, st));
    if (!kids) continue;
    SCAT_TRY(scat::launch_row_fwd(U, pc * L * M1r, M1c, tw, tw_n, st));
    const int octs = J - 1 - j1;
    for (int j2 = j1 + 1; j2 < J; ++j2) {
      const int r2 = h.res(j2);
      const int M2r = Nr >> r2, M2c = Nc >> r2;
      if (lp && p->node_taps && M2r == M2c && (M2r == 64 || M2r == 128) && m_r == 32 &&
          mask_of(j1, j2) != nullptr && scat::node_supported(M2r, M1r / M2r, 1, false, true)) {
        // children of 64 or 128 points a side: one workgroup per child, fed by its parent's
        // whole spectrum (no row-pass output, column pass or lowpass pass through memory)
        scat::NodeLaunch c{};
        c.M = M2r;
        c.A = M1r / M2r;
        c.P = 1;
        c.poly = false;
        c.full = true;
        c.src = U;
        c.filt = tab + p->psi2_off[{r1, j2}];
        c.mask = mask_of(j1, j2);
        c.taps_r = tab + p->taps_r_off[r2];
        c.taps_c = tab + p->taps_c_off[r2];
        c.uout = nullptr;
        c.out = o;
        c.NS = pc * L;
        c.F = L;
        c.G = L;
        c.chan_base = s2_base + (j2 - j1 - 1) * L;
        c.chan_src = octs * L;
        c.chan_f = 1;
        c.K = K;
        c.tw = tw;
        c.tw_n = tw_n;
        SCAT_TRY(scat::launch_node(c, st));
        continue;
      }
      float2 *t2 = tape ? tape->base + tape->y2_off.at({j1, j2}) * pc : T;
      SCAT_TRY(scat::launch_mulfold_invrow(U, tab + p->psi2_off[{r1, j2}], t2, pc * L, L, M1r, M1c,
                                           r2 - r1, r2 - r1, 0, tw, tw_n, st, mask_of(j1, j2)));
      if (tape != nullptr) continue;
      const ChanMap cm2{L * L, L, octs * L, s2_base + (j2 - j1 - 1) * L};
      if (scat::leaf_node_supported(M2r, M2c, m_r, m_c, tw_n)) {  // the whole leaf in one kernel
        SCAT_TRY(scat::launch_leaf_node(t2, pc * L * L, M2r, m_r, tab + p->phi_rows_off[r2],
                                        tab + p->phi_cols_off[r2], o, cm2, K, tw, tw_n, st));
        continue;
      }
      SCAT_TRY(scat::launch_col(1, t2, pc * L * L, M2r, M2c, nullptr, 0, tab + p->phi_rows_off[r2],
                                m_r, W, nullptr, none, K, tw, tw_n, st));
      SCAT_TRY(scat::launch_row_lowpass(W, pc * L * L, m_r, M2c, m_c, tab + p->phi_cols_off[r2], o, cm2,
                                        K, tw, tw_n, st));
    }
    s2_base += L * L * octs;
  }
  return SCAT_OK;
}


// ---- 2-D schedule with the fused row pass (no full 2-D spectrum is ever stored).  With a
// tape the signals before each modulus are kept and the outputs S are not formed.
// Taped forward pass, 2-D: a node is taped as the row pass leaves it, before its inverse
// column transform -- the backward kernels (whole-node or column) transform the columns
// themselves, and the forward pass runs no column kernel for leaves (nodes without children).
// Fused plans do not tape first-order nodes with children at all: their row-pass output
// stays in the forward pass's buffer T, and the backward pass reads it there the same way.
bool first_order_in_forward_buffer(const scat_plan &p) { return p.fused; }

scat_status forward_2d_fused(scat_plan *p, const float *in, float *out, long p0, long pc,
                             const Layout &lay, hipStream_t st, const Tape *tape = nullptr) {
  const scat::HostPlan &h = p->host;
  const int J = h.J, L = h.LQ, K = h.K;
  const int Nr = p->n1, Nc = p->n2;
  const int rJ = h.res(J);
  const int m_r = Nr >> rJ, m_c = Nc >> rJ;
  const size_t n = static_cast<size_t>(Nr) * Nc;
  char *base = static_cast<char *>(p->work);
  float2 *XC = reinterpret_cast<float2 *>(base);
  float2 *T = reinterpret_cast<float2 *>(base + lay.xh * pc);
  float2 *U = reinterpret_cast<float2 *>(base + (lay.xh + lay.t) * pc);
  float2 *V = reinterpret_cast<float2 *>(base + (lay.xh + lay.t + lay.u) * pc);
  float *W = reinterpret_cast<float *>(base + (lay.xh + lay.t + lay.u + lay.v) * pc);
  const float *tab = p->d_tables;
  const float2 *tw = p->d_tw;
  const int tw_n = p->tw_n;
  const float *x = in + static_cast<size_t>(p0) * n;
  float *o = out ? out + static_cast<size_t>(p0) * K * m_r * m_c : nullptr;
  const ChanMap none{1, 1, 0, 0};
  // Column pass (+ modulus) of `nodes` planes of Mr x Mc at resolution `res`, then the
  // lowpass to the output channels `cm`: one kernel when the whole-node variant applies,
  // else the column pass followed by the row half of the lowpass.  Column spectra of the
  // real signals go to `uc` (may be null) as their non-redundant half (rows 0..Mr/2).
  auto col_and_lowpass = [&](int mode, const void *src, long nodes, int Mr, int Mc, int res,
                             float2 *uc, ChanMap cm) -> hipError_t {
    const float *pr = tab + p->phi_rows_off[res], *pcs = tab + p->phi_cols_off[res];
    if (tape != nullptr)  // taped pass: the column pass only, for the children's spectra
      return scat::launch_col(mode, src, nodes, Mr, Mc, uc, 0, pr, m_r, nullptr, nullptr, none, K,
                              tw, tw_n, st, true);
    if (scat::col_node_supported(Mr, Mc, m_r, m_c, tw_n))
      return scat::launch_col_node(mode, src, nodes, Mr, m_r, uc, true, pr, pcs, o, cm, K, tw, tw_n,
                                   st);
    if (mode == 1 && uc == nullptr && scat::leaf_node_supported(Mr, Mc, m_r, m_c, tw_n))
      return scat::launch_leaf_node(static_cast<const float2 *>(src), nodes, Mr, m_r, pr, pcs, o, cm, K,
                                    tw, tw_n, st);
    hipError_t e = scat::launch_col(mode, src, nodes, Mr, Mc, uc, 0, pr, m_r, W, nullptr, none, K,
                                    tw, tw_n, st, true);
    if (e != hipSuccess) return e;
    return scat::launch_row_lowpass(W, nodes, m_r, Mc, m_c, pcs, o, cm, K, tw, tw_n, st);
  };

  SCAT_TRY(col_and_lowpass(0, x, pc, Nr, Nc, 0, XC, ChanMap{1, 1, 0, 0}));
  // every first-order octave in one row pass over x's column spectra
  std::vector<float2 *> t1(J);
  {
    scat::FusedLevel lv[4];
    size_t off = 0;
    for (int j1 = 0; j1 < J; ++j1) {
      const bool kids = h.max_order == 2 && j1 < J - 1;
      t1[j1] = T + off;
      if (tape != nullptr && !kids)
        t1[j1] = tape->base + tape->y1_off[j1] * pc;  // straight to the tape, no column pass
      lv[j1] = scat::FusedLevel{h.res(j1), L, tab + p->psi1_off[j1], t1[j1]};
      off += static_cast<size_t>(pc) * L * (n >> (2 * h.res(j1)));
    }
    SCAT_TRY(scat::launch_rows_fused(XC, true, pc, Nr, Nc, lv, J, tw, tw_n, st));
  }
  int s2_base = 1 + J * L;
  for (int j1 = 0; j1 < J; ++j1) {
    const int r1 = h.res(j1);
    const int M1r = Nr >> r1, M1c = Nc >> r1;
    const bool kids = h.max_order == 2 && j1 < J - 1;
    if (tape != nullptr && !kids) continue;
    SCAT_TRY(col_and_lowpass(1, t1[j1], pc * L, M1r, M1c, r1, kids ? U : nullptr,
                             ChanMap{L, L, 0, 1 + j1 * L}));
    if (!kids) continue;
    const int octs = J - 1 - j1;
    // 64 x 64 children of 128 x 128 nodes (one child octave): one workgroup per child, fed by
    // the nodes' full row-and-column spectra (measured faster than the row pass + leaf kernel
    // pair, and no row-pass output goes to memory)
    if (tape == nullptr && p->node_tables && M1r == 128 && M1c == 128 && octs == 1 && m_r == 32) {
      const int j2 = j1 + 1;
      SCAT_TRY(scat::launch_row_fwd(U, pc * L * (M1r / 2 + 1), M1c, tw, tw_n, st));
      scat::NodeLaunch c{};
      c.M = 64;
      c.A = 2;
      c.P = 1;
      c.poly = false;
      c.src = U;
      c.filt = tab + p->node2_off.at({r1, j2});
      c.mask = nullptr;
      c.lane_mask = lane_mask_of(p, {r1, j2});
      c.taps_r = tab + p->taps_r_off[j2];
      c.taps_c = tab + p->taps_c_off[j2];
      c.uout = nullptr;
      c.out = o;
      c.NS = pc * L;
      c.F = L;
      c.G = L;
      c.chan_base = s2_base;
      c.chan_src = L;
      c.chan_f = 1;
      c.K = K;
      c.tw = tw;
      c.tw_n = tw_n;
      SCAT_TRY(scat::launch_node(c, st));
      s2_base += L * L * octs;
      continue;
    }
    std::vector<float2 *> t2(J);
    {
      scat::FusedLevel lv[4];
      size_t off = 0;
      for (int j2 = j1 + 1; j2 < J; ++j2) {
        t2[j2] = V + off;
        if (tape != nullptr)
          t2[j2] = tape->base + tape->y2_off.at({j1, j2}) * pc;
        lv[j2 - j1 - 1] = scat::FusedLevel{h.res(j2) - r1, L, tab + p->psi2_off[{r1, j2}], t2[j2]};
        off += static_cast<size_t>(pc) * L * L * (n >> (2 * h.res(j2)));
      }
      SCAT_TRY(scat::launch_rows_fused(U, true, pc * L, M1r, M1c, lv, octs, tw, tw_n, st));
    }
    for (int j2 = j1 + 1; j2 < J; ++j2) {
      const int r2 = h.res(j2);
      const int M2r = Nr >> r2, M2c = Nc >> r2;
      if (tape != nullptr) continue;
      SCAT_TRY(col_and_lowpass(1, t2[j2], pc * L * L, M2r, M2c, r2, nullptr,
                               ChanMap{L * L, L, octs * L, s2_base + (j2 - j1 - 1) * L}));
    }
    s2_base += L * L * octs;
  }
  return SCAT_OK;
}

// ---- 2-D schedule with one workgroup per node (scat_node.hip): the spectrum of x, then per
// first-order octave one launch for its L nodes (four polyphase components each when the
// octave has 256 points a side) and one launch per child octave; a node's inverse transform,
// modulus, lowpass and (for parents) forward transform all stay in the LDS of one workgroup.
scat_status forward_2d_node(scat_plan *p, const float *in, float *out, long p0, long pc,
                            const Layout &lay, hipStream_t st) {
  const scat::HostPlan &h = p->host;
  const int J = h.J, L = h.LQ, K = h.K;
  const int N = p->n1;
  const int m = N >> J;
  const size_t n = static_cast<size_t>(N) * N;
  char *base = static_cast<char *>(p->work);
  float2 *XH = reinterpret_cast<float2 *>(base);
  float2 *U = reinterpret_cast<float2 *>(base + lay.xh * pc);
  float *PART = reinterpret_cast<float *>(base + (lay.xh + lay.u) * pc);
  const float *tab = p->d_tables;
  const float2 *tw = p->d_tw;
  const int tw_n = p->tw_n;
  const float *x = in + static_cast<size_t>(p0) * n;
  float *o = out + static_cast<size_t>(p0) * K * m * m;
  // x -> column spectra (rows 0 .. N/2) and S0, then the row transform: the spectrum of x
  SCAT_TRY(scat::launch_col_node(0, x, pc, N, m, XH, true, tab + p->phi_rows_off[0],
                                 tab + p->phi_cols_off[0], o, ChanMap{1, 1, 0, 0}, K, tw, tw_n, st));
  SCAT_TRY(scat::launch_row_fwd(XH, pc * (N / 2 + 1), N, tw, tw_n, st));
  int s2_base = 1 + J * L;
  for (int j1 = 0; j1 < J; ++j1) {
    const int M1 = N >> j1;
    const bool kids = h.max_order == 2 && j1 < J - 1;
    const bool poly = M1 > 128;
    scat::NodeLaunch a{};
    a.M = poly ? M1 / 2 : M1;
    a.A = N / a.M;
    a.P = 1;
    a.poly = poly;
    a.src = XH;
    const bool a2 = a.A == 2;  // kernels that read the paired-column table
    a.filt = tab + (a2 ? p->node2_off.at({0, j1}) : p->psi1_off[j1]);
    a.mask = (!poly && j1 > 0 && !a2) ? p->d_masks64 + p->mask64_off.at({0, j1}) : nullptr;
    a.taps_r = tab + (poly ? p->ptaps_r_off : p->taps_r_off[j1]);
    a.taps_c = tab + (poly ? p->ptaps_c_off : p->taps_c_off[j1]);
    a.uout = kids ? U : nullptr;
    a.out = poly ? PART : o;
    a.NS = pc;
    a.F = L;
    a.G = 1;
    a.chan_base = 1 + j1 * L;
    a.chan_src = 0;
    a.chan_f = 1;
    a.K = K;
    a.tw = tw;
    a.tw_n = tw_n;
    SCAT_TRY(scat::launch_node(a, st));
    if (poly) SCAT_TRY(scat::launch_sum4(PART, o, pc * L, L, K, 1 + j1 * L, st));
    if (!kids) continue;
    const int octs = J - 1 - j1;
    for (int j2 = j1 + 1; j2 < J; ++j2) {
      scat::NodeLaunch c{};
      c.M = N >> j2;
      c.P = poly ? 4 : 1;
      c.A = (poly ? M1 / 2 : M1) / c.M;
      c.poly = false;
      c.src = U;
      const bool c2 = !poly && c.A == 2;
      c.filt = tab + (poly ? p->poly_psi_off.at(j2) : c2 ? p->node2_off.at({j1, j2}) : p->psi2_off.at({j1, j2}));
      c.mask = (poly || c2) ? nullptr : p->d_masks64 + p->mask64_off.at({j1, j2});
      c.lane_mask = (poly && c.A == 2) ? lane_mask_of(p, {-1, j2}) : c2 ? lane_mask_of(p, {j1, j2}) : nullptr;
      c.taps_r = tab + p->taps_r_off[j2];
      c.taps_c = tab + p->taps_c_off[j2];
      c.uout = nullptr;
      c.out = o;
      c.NS = pc * L;
      c.F = L;
      c.G = L;
      c.chan_base = s2_base + (j2 - j1 - 1) * L;
      c.chan_src = octs * L;
      c.chan_f = 1;
      c.K = K;
      c.tw = tw;
      c.tw_n = tw_n;
      SCAT_TRY(scat::launch_node(c, st));
    }
    s2_base += L * L * octs;
  }
  return SCAT_OK;
}

// ---- 2-D schedule for planes whose whole tree fits in LDS: x -> X^ and S0 by the pass
// kernels, then one kernel for everything below
scat_status forward_2d_tree(scat_plan *p, const float *in, float *out, long p0, long pc,
                            const Layout &lay, hipStream_t st) {
  const scat::HostPlan &h = p->host;
  const int J = h.J, L = h.LQ, K = h.K;
  const int Nr = p->n1, Nc = p->n2;
  const int m_r = Nr >> J, m_c = Nc >> J;
  char *base = static_cast<char *>(p->work);
  float2 *XH = reinterpret_cast<float2 *>(base);
  (void)lay;
  const float *tab = p->d_tables;
  const float *x = in + static_cast<size_t>(p0) * Nr * Nc;
  float *o = out + static_cast<size_t>(p0) * K * m_r * m_c;
  SCAT_TRY(scat::launch_tree32_input(x, pc, XH, tab + p->phi_cols_off[0], tab + p->taps_off[0], o,
                                     K, st));
  SCAT_TRY(scat::launch_tree32(XH, pc, L, h.max_order, tab + p->psi1_off[0], tab + p->psi1_off[1],
                               tab + p->phi_cols_off[0], tab + p->phi_cols_off[1],
                               tab + p->taps_off[0], tab + p->taps_off[1], o, K, st));
  return SCAT_OK;
}

// ---- backward pass of the 2-D cascade for one chunk: forward with a tape, then the chain
// of adjoints from the leaves to x (see scat_backward.hip)
struct BwdLayout {
  long chunk = 0;
  size_t per_plane = 0;         // bytes
  Layout fwd;                   // xh, t, u of the taped forward pass
  Tape tape;
  size_t gx = 0, gu = 0, ga = 0, gh = 0;  // elements per plane
  size_t pad_floats = 0;  // padded plans: extended input + extended gradients, floats per plane
};

// 1-D backward pass: the schedule built on the adjoint of the forward row kernel needs every
// octave's row length (second digit of the four-step order) within that kernel's range.
bool bwd_rows_adjoint(const scat_plan &p) {
  const scat::HostPlan &h = p.host;
  for (int j = 0; j < h.J; ++j)
    if (!scat::rows1d_adj_supported(p.n2 >> h.res(j))) return false;
  return true;
}

BwdLayout make_bwd_layout(const scat_plan &p, long batch) {
  BwdLayout b;
  const scat::HostPlan &h = p.host;
  const size_t n = static_cast<size_t>(p.n1) * p.n2, l = h.LQ, c8 = sizeof(float2);
  const bool second = h.max_order == 2 && h.J >= 2;
  if (h.dims == 1) {
    // forward buffers as in make_layout; gradients: x spectrum, one octave's first-order
    // spectra, one (j1, j2) level's second-order spectra, output-grid spectra
    b.fwd.xh = n * c8;
    b.fwd.t = t_elems_1d(h, n) * c8;
    b.fwd.u = l * n * c8;
    b.fwd.v = 0;
    b.tape = make_tape(p);
    b.gx = n;
    if (bwd_rows_adjoint(p)) {
      // every octave's first-order gradients at once, the second-order gradients of one j1
      // (all j2 > j1), and the column-transformed output gradients of all K channels
      b.gu = b.ga = 0;
      for (int j = 0; j < h.J; ++j) b.gu += l * (n >> h.res(j));
      for (int j = 1; second && j < h.J; ++j) b.ga += l * (n >> h.res(j));
      b.gh = static_cast<size_t>(h.K) * (n >> h.res(h.J));
    } else {
      b.gu = l * n;
      b.ga = second ? l * (n >> h.res(1)) : 0;
      b.gh = l * (n >> h.res(h.J));
    }
    if (p.padded) b.pad_floats = 2 * n + static_cast<size_t>(h.K) * (n >> h.res(h.J));
    b.per_plane = b.fwd.xh + b.fwd.t + b.fwd.u + (b.tape.total + b.gx + b.gu + b.ga + b.gh) * c8 +
                  b.pad_floats * sizeof(float);
  } else {
    const size_t t1 = l * n, t2 = second ? l * l * (n >> (2 * h.res(1))) : 0;
    if (p.fused) {
      // buffers of the fused forward schedule (see make_layout)
      size_t ft1 = 0, ft2 = 0;
      for (int j = 0; j < h.J; ++j) ft1 += l * (n >> (2 * h.res(j)));
      for (int j = 1; j < h.J; ++j) ft2 += l * l * (n >> (2 * h.res(j)));
      b.fwd.xh = n * c8;
      b.fwd.t = ft1 * c8;
      b.fwd.u = second ? l * n * c8 : 0;
      b.fwd.v = 0;  // the taped pass writes the second-order row-pass outputs into the tape
      (void)ft2;
    } else {
      b.fwd.xh = n * c8;
      b.fwd.t = (t1 > t2 ? t1 : t2) * c8;
      b.fwd.u = second ? l * n * c8 : 0;
    }
    b.tape = make_tape(p);
    b.gx = n;
    // spectra of the output-grid gradient planes of one launch (at most L*L, or L, nodes)
    const size_t mm = static_cast<size_t>(p.n1 >> h.res(h.J)) * (p.n2 >> h.res(h.J));
    b.gh = (second ? l * l : l) * mm;
    // every octave's first-order gradients at once, the second-order gradients of one j1
    // (all j2 > j1); output-grid spectra of x's and of one octave's own channels besides
    b.gu = b.ga = 0;
    for (int j = 0; j < h.J; ++j) b.gu += l * (n >> (2 * h.res(j)));
    for (int j = 1; second && j < h.J; ++j) b.ga += l * l * (n >> (2 * h.res(j)));
    b.gh += (l + 1) * mm;
    if (p.padded)
      b.pad_floats = 2 * n + static_cast<size_t>(h.K) * (p.n1 >> h.res(h.J)) * (p.n2 >> h.res(h.J));
    b.per_plane = b.fwd.xh + b.fwd.t + b.fwd.u + b.fwd.v +
                  (b.tape.total + b.gx + b.gu + b.ga + b.gh) * c8 + b.pad_floats * sizeof(float);
  }
  long c = static_cast<long>(scratch_budget() / b.per_plane);
  if (c < 1) c = 1;
  if (c > batch) c = batch;
  b.chunk = c;
  b.fwd.chunk = c;
  b.fwd.per_plane = b.per_plane;
  return b;
}

// ---- backward pass of the 2-D cascade for one chunk, schedule built on k_rows2d_adj: the
// gradient spectrum of a first-order node is one launch over its own lowpass term and all
// its second-order children, x's over its lowpass term and all first-order nodes; nodes
// that fit one workgroup take the modulus backward step in a single kernel.
scat_status backward_2d_rows_adjoint(scat_plan *p, const float *go, float *gi, long pc, BwdLayout &bl,
                                     float2 *GX, float2 *GU, float2 *GA, float2 *GH, hipStream_t st) {
  const scat::HostPlan &h = p->host;
  const int J = h.J, L = h.LQ, K = h.K;
  const int Nr = p->n1, Nc = p->n2;
  const int rJ = h.res(J);
  const int m_r = Nr >> rJ, m_c = Nc >> rJ;
  const size_t n = static_cast<size_t>(Nr) * Nc, mm = static_cast<size_t>(m_r) * m_c;
  const float *tab = p->d_tables;
  const float2 *tw = p->d_tw;
  const int tw_n = p->tw_n;
  const bool second = h.max_order == 2 && J >= 2;
  auto lg = [](int v) {
    int r = 0;
    while ((1 << r) < v) ++r;
    return r;
  };
  // GH: scratch of the node kernels' launches, then the small transforms of x's and of the
  // current octave's output gradients
  float2 *GHX = GH + (second ? static_cast<size_t>(L) * L : static_cast<size_t>(L)) * mm * pc;
  float2 *GHU = GHX + mm * pc;
  auto low_child = [&](const float2 *ghat, int res, int Mr, int Mc) {
    return scat::Rows2dAdjChild{ghat, tab + p->phi_cols_off[res], tab + p->phi_rows_off[res],
                                lg(Mr / m_r), lg(Mc / m_c), ChanMap{1, 1, 0, 0}, 0};
  };
  SCAT_TRY(scat::launch_small_fft2(go, pc, ChanMap{1, 1, 0, 0}, K, m_r, m_c, GHX, tw, tw_n, st));
  // (rows of 512 points: the row-adjoint kernel leaves the inverse row transform to a pass of
  // its own)
  const bool top_inv = scat::rows2d_adj_supported(Nc, true);
  scat::Rows2dAdjArgs top{};
  top.inverse = top_inv ? 1 : 0;
  top.c[top.n++] = low_child(GHX, 0, Nr, Nc);
  auto flush = [&](float2 *dst, long nodes, int Sr, int Sc, scat::Rows2dAdjArgs &a) -> hipError_t {
    hipError_t e = scat::launch_rows2d_adj(dst, nodes, Sr, Sc, a, tw, tw_n, st);
    a.n = 0;
    a.accumulate = 1;
    return e;
  };
  int s2_base = 1 + J * L;
  float2 *GUj = GU;
  const float2 *Tfwd = reinterpret_cast<const float2 *>(static_cast<const char *>(p->work) +
                                                        bl.fwd.xh * pc);
  size_t t_off = 0;  // as forward_2d_fused lays out T: all octaves, one after the other
  for (int j1 = 0; j1 < J; ++j1) {
    const int r1 = h.res(j1);
    const int M1r = Nr >> r1, M1c = Nc >> r1;
    const bool kids = second && j1 < J - 1;
    const bool node1 = scat::node_modback_supported(M1r, M1c);
    // a full-resolution level that goes through the column kernel leaves its forward row
    // transform to x's row-adjoint launch, which does it in registers on the way in
    const bool pre_rows = !node1 && r1 == 0 && top_inv;
    // the signal before the modulus as its row pass left it: in the tape, or for nodes with
    // children of fused plans still in the forward pass's buffer
    const float2 *y1 = bl.tape.base + bl.tape.y1_off[j1] * pc;
    if (kids && first_order_in_forward_buffer(*p)) y1 = Tfwd + t_off;
    t_off += static_cast<size_t>(pc) * L * M1r * M1c;
    const ChanMap cm1{L, L, 0, 1 + j1 * L};
    if (!kids && node1) {
      SCAT_TRY(scat::launch_node_modback_low(go, pc * L, cm1, K, m_r, m_c, M1r, M1c,
                                             tab + p->phi_rows_off[r1], tab + p->phi_cols_off[r1], GH,
                                             y1, GUj, tw, tw_n, st, true));
    } else if (!kids) {
      SCAT_TRY(scat::launch_lowpass_adj_rows(go, pc * L, cm1, K, m_r, m_c, M1r, M1c,
                                             tab + p->phi_rows_off[r1], tab + p->phi_cols_off[r1], GH,
                                             GUj, tw, tw_n, st));
      SCAT_TRY(scat::launch_cols_modback(GUj, y1, pc * L, M1r, M1c, tw, tw_n, st, 0,
                                         true));
      if (!pre_rows)
        SCAT_TRY(scat::launch_fft_rows_inplace(GUj, pc * L * M1r, M1c, false, tw, tw_n, st));
    } else {
      const int octs = J - 1 - j1;
      const bool fused_inv = !node1 && scat::rows2d_adj_supported(M1c, true);
      scat::Rows2dAdjArgs a{};
      a.inverse = fused_inv ? 1 : 0;
      SCAT_TRY(scat::launch_small_fft2(go, pc * L, cm1, K, m_r, m_c, GHU, tw, tw_n, st));
      a.c[a.n++] = low_child(GHU, r1, M1r, M1c);
      float2 *GAj = GA;
      for (int j2 = j1 + 1; j2 < J; ++j2) {
        const int r2 = h.res(j2);
        const int M2r = Nr >> r2, M2c = Nc >> r2;
        const long nodes = pc * L * L;
        const ChanMap cm2{L * L, L, octs * L, s2_base + (j2 - j1 - 1) * L};
        const float2 *y2 = bl.tape.base + bl.tape.y2_off.at({j1, j2}) * pc;
        if (scat::node_modback_supported(M2r, M2c)) {
          SCAT_TRY(scat::launch_node_modback_low(go, nodes, cm2, K, m_r, m_c, M2r, M2c,
                                                 tab + p->phi_rows_off[r2], tab + p->phi_cols_off[r2],
                                                 GH, y2, GAj, tw, tw_n, st,
                                                 true));
        } else {
          SCAT_TRY(scat::launch_lowpass_adj_rows(go, nodes, cm2, K, m_r, m_c, M2r, M2c,
                                                 tab + p->phi_rows_off[r2], tab + p->phi_cols_off[r2],
                                                 GH, GAj, tw, tw_n, st));
          SCAT_TRY(scat::launch_cols_modback(GAj, y2, nodes, M2r, M2c, tw, tw_n, st, 0,
                                             true));
          SCAT_TRY(scat::launch_fft_rows_inplace(GAj, nodes * M2r, M2c, false, tw, tw_n, st));
        }
        for (int l2 = 0; l2 < L; ++l2) {
          if (a.n == scat::kRows1dMaxChildren) SCAT_TRY(flush(GUj, pc * L, M1r, M1c, a));
          a.c[a.n++] = scat::Rows2dAdjChild{
              GAj, tab + p->psi2_off[{r1, j2}] + static_cast<size_t>(l2) * M1r * M1c, nullptr,
              r2 - r1, r2 - r1, ChanMap{L, 1, 0, l2}, 0};
        }
        GAj += static_cast<size_t>(nodes) * M2r * M2c;
      }
      s2_base += L * L * octs;
      SCAT_TRY(flush(GUj, pc * L, M1r, M1c, a));
      if (node1) {
        SCAT_TRY(scat::launch_node_modback(GUj, y1, pc * L, M1r, M1c, tw, tw_n, st,
                                           true));
      } else {
        if (!fused_inv)
          SCAT_TRY(scat::launch_fft_rows_inplace(GUj, pc * L * M1r, M1c, true, tw, tw_n, st));
        SCAT_TRY(scat::launch_cols_modback(GUj, y1, pc * L, M1r, M1c, tw, tw_n, st, 0,
                                           true));
        if (!pre_rows)
          SCAT_TRY(scat::launch_fft_rows_inplace(GUj, pc * L * M1r, M1c, false, tw, tw_n, st));
      }
    }
    for (int l = 0; l < L; ++l) {
      if (top.n == scat::kRows1dMaxChildren) SCAT_TRY(flush(GX, pc, Nr, Nc, top));
      top.c[top.n++] = scat::Rows2dAdjChild{GUj, tab + p->psi1_off[j1] + static_cast<size_t>(l) * n,
                                            nullptr, r1, r1, ChanMap{L, 1, 0, l}, 0, pre_rows ? 1 : 0};
    }
    GUj += static_cast<size_t>(pc) * L * M1r * M1c;
  }
  SCAT_TRY(flush(GX, pc, Nr, Nc, top));
  // g_x = Re(inverse transform): the rows are done (or follow here), then the columns
  if (!top_inv) SCAT_TRY(scat::launch_fft_rows_inplace(GX, pc * Nr, Nc, true, tw, tw_n, st));
  SCAT_TRY(scat::launch_fft_cols_inplace(GX, pc, Nr, Nc, true, tw, tw_n, st));
  SCAT_TRY(scat::launch_take_real(GX, gi, pc * static_cast<long>(n), st));
  return SCAT_OK;
}

scat_status backward_2d(scat_plan *p, const float *in, const float *gout, float *gin, long p0,
                        long pc, BwdLayout &bl, hipStream_t st) {
  const scat::HostPlan &h = p->host;
  const int J = h.J, L = h.LQ, K = h.K;
  const int Nr = p->n1, Nc = p->n2;
  const int rJ = h.res(J);
  const int m_r = Nr >> rJ, m_c = Nc >> rJ;
  const size_t n = static_cast<size_t>(Nr) * Nc;
  char *base = static_cast<char *>(p->work);
  float2 *after_fwd =
      reinterpret_cast<float2 *>(base + (bl.fwd.xh + bl.fwd.t + bl.fwd.u + bl.fwd.v) * pc);
  bl.tape.base = after_fwd;
  float2 *GX = after_fwd + bl.tape.total * pc;
  float2 *GU = GX + bl.gx * pc;
  float2 *GA = GU + bl.gu * pc;
  float2 *GH = GA + bl.ga * pc;
  const float *go = gout + static_cast<size_t>(p0) * K * m_r * m_c;
  float *gi = gin + static_cast<size_t>(p0) * n;

  scat_status fs = p->fused ? forward_2d_fused(p, in, nullptr, p0, pc, bl.fwd, st, &bl.tape)
                            : forward_2d(p, in, nullptr, p0, pc, bl.fwd, st, &bl.tape);
  if (fs != SCAT_OK) return fs;
  // (every plan scat_backward accepts keeps at least 4 points per row at every octave, which
  // is all the row-adjoint schedule asks for)
  return backward_2d_rows_adjoint(p, go, gi, pc, bl, GX, GU, GA, GH, st);
}

scat_status forward_1d(scat_plan *p, const float *in, float *out, long p0, long pc,
                       const Layout &lay, hipStream_t st, const Tape *tape = nullptr);

// ---- backward pass of the 1-D cascade for one chunk (signals as n1 x n2 matrices, spectra
// in four-step order): the same chain of adjoints as backward_2d with four-step transforms
// (row pass, twiddle, column pass) and folds / tiles along the second digit only.
scat_status backward_1d(scat_plan *p, const float *in, const float *gout, float *gin, long p0,
                        long pc, BwdLayout &bl, hipStream_t st) {
  const scat::HostPlan &h = p->host;
  const int J = h.J, Q = h.LQ, K = h.K;
  const int N1 = p->n1, N2 = p->n2;
  const int N = N1 * N2;
  const int rJ = h.res(J);
  const int mc_out = N2 >> rJ, m = N >> rJ;
  char *base = static_cast<char *>(p->work);
  float2 *after_fwd = reinterpret_cast<float2 *>(base + (bl.fwd.xh + bl.fwd.t + bl.fwd.u) * pc);
  bl.tape.base = after_fwd;
  float2 *GX = after_fwd + bl.tape.total * pc;
  float2 *GU = GX + bl.gx * pc;
  float2 *GA = GU + bl.gu * pc;
  float2 *GH = GA + bl.ga * pc;
  const float *tab = p->d_tables;
  const float2 *tw = p->d_tw;
  const int tw_n = p->tw_n;
  const float *go = gout + static_cast<size_t>(p0) * K * m;
  float *gi = gin + static_cast<size_t>(p0) * N;

  scat_status fs = forward_1d(p, in, nullptr, p0, pc, bl.fwd, st, &bl.tape);
  if (fs != SCAT_OK) return fs;

  // dst [nodes][N1][Mc] = adjoint lowpass of the nodes' output gradients: forward four-step
  // transform of the m-sample gradient, tiled along k2, times phi^ at resolution `res`
  auto lowpass_adj = [&](long nodes, ChanMap cm, int res, int Mc, float2 *dst) -> hipError_t {
    hipError_t e = scat::launch_gather_real(go, nodes, cm, K, m, GH, st);
    if (e != hipSuccess) return e;
    e = scat::launch_fft_cols_inplace(GH, nodes, N1, mc_out, false, tw, tw_n, st);
    if (e != hipSuccess) return e;
    e = scat::launch_twiddle(GH, nodes, N1, mc_out, false, tw, tw_n, st);
    if (e != hipSuccess) return e;
    e = scat::launch_fft_rows_inplace(GH, nodes * N1, mc_out, false, tw, tw_n, st);
    if (e != hipSuccess) return e;
    return scat::launch_tile_filter(GH, tab + p->phi_off[res], dst, nodes, N1, Mc, mc_out, st);
  };
  // spectrum -> signal, modulus backward against the taped y, signal -> spectrum
  // (y is the taped row-pass output of the node, see forward_1d)
  auto through_modulus = [&](float2 *g, const float2 *y, long nodes, int Mc) -> hipError_t {
    hipError_t e = scat::launch_fft_rows_inplace(g, nodes * N1, Mc, true, tw, tw_n, st);
    if (e != hipSuccess) return e;
    e = scat::launch_cols_modback(g, y, nodes, N1, Mc, tw, tw_n, st, Mc > 1 ? N1 * Mc : 0, true);
    if (e != hipSuccess) return e;
    return scat::launch_fft_rows_inplace(g, nodes * N1, Mc, false, tw, tw_n, st);
  };

  if (bwd_rows_adjoint(*p)) {
    // Adjoint row kernel: a node's gradient (column spectra, ready for the modulus backward)
    // is one launch over the list of its children -- its own lowpass output and the
    // second-order nodes below it -- and x's over the first-order nodes of all octaves.
    auto lg = [](int v) {
      int r = 0;
      while ((1 << r) < v) ++r;
      return r;
    };
    // column half of the forward four-step transform of all K output gradients at once
    SCAT_TRY(scat::launch_gather_real(go, pc * K, ChanMap{K, K, 0, 0}, K, m, GH, st));
    SCAT_TRY(scat::launch_fft_cols_inplace(GH, pc * K, N1, mc_out, false, tw, tw_n, st));
    SCAT_TRY(scat::launch_twiddle(GH, pc * K, N1, mc_out, false, tw, tw_n, st));
    auto low_child = [&](ChanMap cm, int res, int Mc) {
      return scat::Rows1dAdjChild{GH, tab + p->phi_off[res], lg(Mc / mc_out), cm, K};
    };
    scat::Rows1dAdjArgs top{};
    top.c[top.n++] = low_child(ChanMap{1, 1, 0, 0}, 0, N2);
    auto flush_top = [&]() -> hipError_t {
      hipError_t e = scat::launch_rows1d_adj(GX, pc, N1, N2, top, tw, tw_n, st);
      top.n = 0;
      top.accumulate = 1;
      return e;
    };
    int s2 = 1 + J * Q;
    float2 *GUj = GU;
    for (int j1 = 0; j1 < J; ++j1) {
      const int r1 = h.res(j1);
      const int Mc1 = N2 >> r1;
      const bool kids = h.max_order == 2 && j1 < J - 1;
      const int octs = J - 1 - j1;
      scat::Rows1dAdjArgs a{};
      a.c[a.n++] = low_child(ChanMap{Q, Q, 0, 1 + j1 * Q}, r1, Mc1);
      float2 *GAj = GA;
      for (int j2 = j1 + 1; kids && j2 < J; ++j2) {
        const int r2 = h.res(j2);
        const int Mc2 = N2 >> r2;
        scat::Rows1dAdjArgs a2{};
        a2.c[a2.n++] = low_child(ChanMap{Q, 1, octs, s2 + (j2 - j1 - 1)}, r2, Mc2);
        SCAT_TRY(scat::launch_rows1d_adj(GAj, pc * Q, N1, Mc2, a2, tw, tw_n, st));
        SCAT_TRY(scat::launch_cols_modback(GAj, bl.tape.base + bl.tape.y2_off.at({j1, j2}) * pc,
                                           pc * Q, N1, Mc2, tw, tw_n, st, Mc2 > 1 ? N1 * Mc2 : 0, true));
        if (a.n == scat::kRows1dMaxChildren) return SCAT_ERR_ARG;  // J <= 12: at most 12 children
        a.c[a.n++] = scat::Rows1dAdjChild{GAj, tab + p->psi2_off[{r1, j2}], r2 - r1,
                                          ChanMap{1, 1, 0, 0}, 0};
        GAj += static_cast<size_t>(pc) * Q * N1 * Mc2;
      }
      if (kids) s2 += Q * octs;
      SCAT_TRY(scat::launch_rows1d_adj(GUj, pc * Q, N1, Mc1, a, tw, tw_n, st));
      SCAT_TRY(scat::launch_cols_modback(GUj, bl.tape.base + bl.tape.y1_off[j1] * pc, pc * Q, N1, Mc1,
                                         tw, tw_n, st, Mc1 > 1 ? N1 * Mc1 : 0, true));
      for (int q = 0; q < Q; ++q) {
        if (top.n == scat::kRows1dMaxChildren) SCAT_TRY(flush_top());
        top.c[top.n++] = scat::Rows1dAdjChild{
            GUj, tab + p->psi1_off[j1] + static_cast<size_t>(q) * N, r1, ChanMap{Q, 1, 0, q}, 0};
      }
      GUj += static_cast<size_t>(pc) * Q * N1 * Mc1;
    }
    SCAT_TRY(flush_top());
    // g_x = Re(inverse four-step transform): the row half is done, twiddle and columns remain
    SCAT_TRY(scat::launch_twiddle(GX, pc, N1, N2, true, tw, tw_n, st));
    SCAT_TRY(scat::launch_fft_cols_inplace(GX, pc, N1, N2, true, tw, tw_n, st));
    SCAT_TRY(scat::launch_take_real(GX, gi, pc * static_cast<long>(N), st));
    return SCAT_OK;
  }

  SCAT_TRY(lowpass_adj(pc, ChanMap{1, 1, 0, 0}, 0, N2, GX));
  int s2_base = 1 + J * Q;
  for (int j1 = 0; j1 < J; ++j1) {
    const int r1 = h.res(j1);
    const int Mc1 = N2 >> r1;
    const bool kids = h.max_order == 2 && j1 < J - 1;
    const int octs = J - 1 - j1;
    SCAT_TRY(lowpass_adj(pc * Q, ChanMap{Q, Q, 0, 1 + j1 * Q}, r1, Mc1, GU));
    for (int j2 = j1 + 1; kids && j2 < J; ++j2) {
      const int r2 = h.res(j2);
      const int Mc2 = N2 >> r2;
      SCAT_TRY(lowpass_adj(pc * Q, ChanMap{Q, 1, octs, s2_base + (j2 - j1 - 1)}, r2, Mc2, GA));
      SCAT_TRY(through_modulus(GA, bl.tape.base + bl.tape.y2_off.at({j1, j2}) * pc, pc * Q, Mc2));
      SCAT_TRY(scat::launch_tile_accum(GU, tab + p->psi2_off[{r1, j2}], GA, pc * Q, 1, N1, Mc1, N1,
                                       Mc2, st));
    }
    if (kids) s2_base += Q * octs;
    SCAT_TRY(through_modulus(GU, bl.tape.base + bl.tape.y1_off[j1] * pc, pc * Q, Mc1));
    SCAT_TRY(scat::launch_tile_accum(GX, tab + p->psi1_off[j1], GU, pc, Q, N1, N2, N1, Mc1, st));
  }
  // g_x = Re(inverse four-step transform of g_X^)
  SCAT_TRY(scat::launch_fft_rows_inplace(GX, pc * N1, N2, true, tw, tw_n, st));
  SCAT_TRY(scat::launch_twiddle(GX, pc, N1, N2, true, tw, tw_n, st));
  SCAT_TRY(scat::launch_fft_cols_inplace(GX, pc, N1, N2, true, tw, tw_n, st));
  SCAT_TRY(scat::launch_take_real(GX, gi, pc * static_cast<long>(N), st));
  return SCAT_OK;
}

// ---- 3-D solid harmonic plans: tables (pre-scaled by 1/n for the unnormalised inverse
// transforms), twiddles, and the schedule of the definition at full resolution
scat_status upload_3d(scat_plan *p) {
  const scat::HostPlan3D &h = p->h3;
  const size_t n = h.points();
  const double scale = 1.0 / static_cast<double>(n);
  std::vector<float> pool;
  p->psi3_off.clear();
  for (size_t jl = 0; jl < h.psi.size(); ++jl) {
    const std::vector<double> &tab = h.psi[jl];
    p->psi3_off.push_back(pool.size());
    if (!p->fused3) {
      for (double d : tab) pool.push_back(static_cast<float>(d * scale));
      continue;
    }
    // fused passes: tables interleaved in pairs (g_2p, g_2p+1) as complex numbers, the
    // unpaired last one with a zero partner (pool.size() stays even: 8-byte aligned)
    const int M = static_cast<int>(tab.size() / n);
    for (int m = 0; m < M; m += 2)
      for (size_t e = 0; e < n; ++e) {
        pool.push_back(static_cast<float>(tab[m * n + e] * scale));
        pool.push_back(m + 1 < M ? static_cast<float>(tab[(m + 1) * n + e] * scale) : 0.f);
      }
  }
  p->phi3_off = pool.size();
  for (double d : h.phi) pool.push_back(static_cast<float>(d * scale));
  int side = h.shape[0];
  if (h.shape[1] > side) side = h.shape[1];
  if (h.shape[2] > side) side = h.shape[2];
  p->tw_n = side;
  std::vector<float2> tw(p->tw_n);
  const double two_pi = 6.283185307179586476925286766559;
  for (int j = 0; j < p->tw_n; ++j) {
    double a = -two_pi * j / p->tw_n;
    tw[j] = make_float2(static_cast<float>(std::cos(a)), static_cast<float>(std::sin(a)));
  }
  if (hipGetDevice(&p->device) != hipSuccess) return SCAT_ERR_DEVICE;
  if (hipMalloc(&p->d_tables, pool.size() * sizeof(float)) != hipSuccess) return SCAT_ERR_ALLOC;
  if (hipMalloc(&p->d_tw, tw.size() * sizeof(float2)) != hipSuccess) return SCAT_ERR_ALLOC;
  if (hipMemcpy(p->d_tables, pool.data(), pool.size() * sizeof(float), hipMemcpyHostToDevice) !=
      hipSuccess)
    return SCAT_ERR_DEVICE;
  if (hipMemcpy(p->d_tw, tw.data(), tw.size() * sizeof(float2), hipMemcpyHostToDevice) != hipSuccess)
    return SCAT_ERR_DEVICE;
  p->has_device = true;
  return note_static_scratch(p);
}

// scratch per volume.  General path: X^, U^ (and V^ at order 2), work buffer, all complex;
// |.|^2 sums, real.  Fused path: X^, U^, the axis-0 stage T, the 2L+1 filtered signals W_m,
// the slab-folded lowpass spectra P of all K channels and their fully folded form Q.
size_t bytes_per_volume_3d(const scat_plan &p) {
  const scat::HostPlan3D &h = p.h3;
  const size_t n = h.points();
  if (!p.fused3)
    return n * sizeof(float2) * (p.host.max_order == 2 && p.host.J >= 2 ? 4 : 3) + n * sizeof(float);
  const int Jo = h.out_shift();
  const size_t folded12 = static_cast<size_t>(h.shape[0]) * (h.shape[1] >> Jo) * (h.shape[2] >> Jo);
  return (n * (3 + h.L + 1) + static_cast<size_t>(h.K) * (folded12 + (n >> (3 * Jo)))) *
         sizeof(float2);
}

scat_status forward_3d_fused(scat_plan *p, const float *in, float *out, long p0, long pc,
                             hipStream_t st) {
  const scat::HostPlan3D &h = p->h3;
  const int n0 = h.shape[0], n1 = h.shape[1], n2 = h.shape[2];
  const int J = h.J, L = h.L, K = h.K;
  const int Jo = h.out_shift();  // the outputs are read at the samples 2^Jo n
  const size_t n = h.points();
  const size_t tot = static_cast<size_t>(pc) * n;
  const bool second = h.max_order == 2 && J >= 2;
  const int m0 = n0 >> Jo, m1 = n1 >> Jo, m2 = n2 >> Jo;
  float2 *XH = static_cast<float2 *>(p->work);
  float2 *UH = XH + tot;
  float2 *T = UH + tot;
  float2 *W = T + tot;
  float2 *P = W + tot * (L + 1);
  float2 *Q = P + static_cast<size_t>(pc) * K * n0 * m1 * m2;
  const float *tab = p->d_tables;
  const float2 *tw = p->d_tw;
  const int tw_n = p->tw_n;
  const float *x = in + static_cast<size_t>(p0) * n;
  const size_t mout = static_cast<size_t>(m0) * m1 * m2;
  float *o = out + static_cast<size_t>(p0) * K * mout;
  const float *phi = tab + p->phi3_off;
  // dst^ (may be null) and channel c from the real signal with spectrum Fh; its 2l+1
  // filtered versions travel as l+1 complex signals
  auto node = [&](const float2 *Fh, int j, int l, float2 *dst, int c) -> hipError_t {
    const float2 *ps = reinterpret_cast<const float2 *>(
        tab + p->psi3_off[static_cast<size_t>(j) * (L + 1) + l]);
    hipError_t e = scat::launch3_slab_mul_inv(Fh, ps, W, pc, n0, n1, n2, l + 1, tw, tw_n, st);
    if (e != hipSuccess) return e;
    e = scat::launch3_axis0_rho(W, nullptr, T, pc, n0, n1 * n2, l + 1, tw, tw_n, st);
    if (e != hipSuccess) return e;
    return scat::launch3_slab_fwd_low(T, dst, phi, P, pc, n0, n1, n2, Jo, K, c, tw, tw_n, st);
  };
  SCAT_TRY(scat::launch3_axis0_rho(nullptr, x, T, pc, n0, n1 * n2, 0, tw, tw_n, st));
  SCAT_TRY(scat::launch3_slab_fwd_low(T, XH, phi, P, pc, n0, n1, n2, Jo, K, 0, tw, tw_n, st));
  int c1 = 1, c2 = 1 + J * (L + 1);
  for (int j1 = 0; j1 < J; ++j1)
    for (int l = 0; l <= L; ++l) {
      const bool kids = second && j1 < J - 1;
      SCAT_TRY(node(XH, j1, l, kids ? UH : nullptr, c1++));
      if (!kids) continue;
      for (int j2 = j1 + 1; j2 < J; ++j2) SCAT_TRY(node(UH, j2, l, nullptr, c2++));
    }
  // aliases of axis 0, small inverse transforms, real parts: all channels at once
  SCAT_TRY(scat::launch3_fold0(P, Q, pc * K, n0, m0, m1 * m2, st));
  SCAT_TRY(scat::launch3_fft(Q, pc * K, m0, m1, m2, true, tw, tw_n, st));
  SCAT_TRY(scat::launch3_real_part(Q, o, pc * K * static_cast<long>(mout), st));
  return SCAT_OK;
}

scat_status forward_3d(scat_plan *p, const float *in, float *out, long p0, long pc, hipStream_t st) {
  const scat::HostPlan3D &h = p->h3;
  const int n0 = h.shape[0], n1 = h.shape[1], n2 = h.shape[2];
  const int J = h.J, L = h.L, K = h.K;
  const int Jo = h.out_shift();  // the outputs are read at the samples 2^Jo n
  const size_t n = h.points();
  const long tot = pc * static_cast<long>(n);
  const bool second = h.max_order == 2 && J >= 2;
  float2 *XH = static_cast<float2 *>(p->work);
  float2 *UH = XH + tot;
  float2 *Wk = UH + tot;
  float2 *VH = second ? Wk + tot : nullptr;
  float *acc = reinterpret_cast<float *>((second ? VH : Wk) + tot);
  const float *tab = p->d_tables;
  const float2 *tw = p->d_tw;
  const int tw_n = p->tw_n;
  const float *x = in + static_cast<size_t>(p0) * n;
  const size_t mout = static_cast<size_t>(n0 >> Jo) * (n1 >> Jo) * (n2 >> Jo);
  float *o = out + static_cast<size_t>(p0) * K * mout;
  // lowpass of the signal with spectrum Fh, read at the samples 2^J n, to channel c
  auto lowpass = [&](const float2 *Fh, int c) -> hipError_t {
    hipError_t e = scat::launch3_mul_table(Fh, tab + p->phi3_off, Wk, pc, static_cast<long>(n), st);
    if (e != hipSuccess) return e;
    e = scat::launch3_fft(Wk, pc, n0, n1, n2, true, tw, tw_n, st);
    if (e != hipSuccess) return e;
    return scat::launch3_sample(Wk, o, pc, K, c, n0, n1, n2, Jo, st);
  };
  // dst^ = FFT3( sqrt( sum_m |IFFT3(Fh psi_{j,l,m})|^2 ) )
  auto rho = [&](const float2 *Fh, int j, int l, float2 *dst) -> hipError_t {
    const float *ps = tab + p->psi3_off[static_cast<size_t>(j) * (L + 1) + l];
    for (int m = 0; m < 2 * l + 1; ++m) {
      hipError_t e = scat::launch3_mul_table(Fh, ps + static_cast<size_t>(m) * n, Wk, pc,
                                             static_cast<long>(n), st);
      if (e != hipSuccess) return e;
      e = scat::launch3_fft(Wk, pc, n0, n1, n2, true, tw, tw_n, st);
      if (e != hipSuccess) return e;
      e = scat::launch3_accum_abs2(Wk, acc, tot, m == 0, st);
      if (e != hipSuccess) return e;
    }
    hipError_t e = scat::launch3_sqrt(acc, dst, tot, st);
    if (e != hipSuccess) return e;
    return scat::launch3_fft(dst, pc, n0, n1, n2, false, tw, tw_n, st);
  };
  SCAT_TRY(scat::launch3_real_to_complex(x, XH, tot, st));
  SCAT_TRY(scat::launch3_fft(XH, pc, n0, n1, n2, false, tw, tw_n, st));
  SCAT_TRY(lowpass(XH, 0));
  int c1 = 1, c2 = 1 + J * (L + 1);
  for (int j1 = 0; j1 < J; ++j1)
    for (int l = 0; l <= L; ++l) {
      SCAT_TRY(rho(XH, j1, l, UH));
      SCAT_TRY(lowpass(UH, c1++));
      if (!second) continue;
      for (int j2 = j1 + 1; j2 < J; ++j2) {
        SCAT_TRY(rho(UH, j2, l, VH));
        SCAT_TRY(lowpass(VH, c2++));
      }
    }
  return SCAT_OK;
}

// ---- backward pass of a 3-D plan (every shape: the full-grid schedule, transforms by the
// plain passes).  With spectra A accumulated in the Fourier domain, S = sample(F conv phi)
// gives A_F += phi^ FFT(upsample(g_S)); rho = sqrt(sum_m |y_m|^2), y_m = IFFT(F^ g_m) gives
// A_F += sum_m g_m FFT(g_rho y_m / rho); g_F = Re IFFT(A_F).  The filtered signals y_m of the
// node at hand (and of its child) are recomputed and kept while their gradients are formed.
size_t bytes_per_volume_3d_bwd(const scat_plan &p) {
  const size_t n = p.h3.points(), M = 2 * static_cast<size_t>(p.h3.L) + 1;
  // X^, A_X, U^, A_U, work; two sets of filtered signals; two sums of squares; the small
  // spectra of the output gradient, all channels
  return n * sizeof(float2) * (5 + 2 * M) + n * sizeof(float) * 2 +
         static_cast<size_t>(p.h3.K) * (n >> (3 * p.h3.out_shift())) * sizeof(float2);
}

scat_status backward_3d(scat_plan *p, const float *in, const float *gout, float *gin, long p0, long pc,
                        hipStream_t st) {
  const scat::HostPlan3D &h = p->h3;
  const int n0 = h.shape[0], n1 = h.shape[1], n2 = h.shape[2];
  const int J = h.J, L = h.L, K = h.K, M = 2 * L + 1;
  const int Jo = h.out_shift();  // the outputs were read at the samples 2^Jo n
  const size_t n = h.points();
  const long tot = pc * static_cast<long>(n);
  const bool second = h.max_order == 2 && J >= 2;
  float2 *XH = static_cast<float2 *>(p->work);
  float2 *AX = XH + tot, *UH = AX + tot, *AU = UH + tot, *Wk = AU + tot;
  float2 *W1 = Wk + tot, *W2 = W1 + static_cast<size_t>(M) * tot;
  float *acc1 = reinterpret_cast<float *>(W2 + static_cast<size_t>(M) * tot), *acc2 = acc1 + tot;
  float2 *Gs = reinterpret_cast<float2 *>(acc2 + tot);
  const float *tab = p->d_tables;
  const float2 *tw = p->d_tw;
  const int tw_n = p->tw_n;
  const float *x = in + static_cast<size_t>(p0) * n;
  const size_t mout = static_cast<size_t>(n0 >> Jo) * (n1 >> Jo) * (n2 >> Jo);
  const float *go = gout + static_cast<size_t>(p0) * K * mout;
  float *gi = gin + static_cast<size_t>(p0) * n;
  const float *phi = tab + p->phi3_off;
  // table m of (j, l): fused plans keep them as interleaved pairs
  auto table = [&](int j, int l, int m, int *stride) -> const float * {
    const float *base = tab + p->psi3_off[static_cast<size_t>(j) * (L + 1) + l];
    *stride = p->fused3 ? 2 : 1;
    return p->fused3 ? base + static_cast<size_t>(m / 2) * 2 * n + (m & 1)
                     : base + static_cast<size_t>(m) * n;
  };
  auto fft3 = [&](float2 *d, bool inv) {
    return scat::launch3_fft(d, pc, n0, n1, n2, inv, tw, tw_n, st);
  };
  // dst (=|+=) phi^ FFT(upsample(g[chan])): the spectrum of the zero-inserted gradient is
  // the small spectrum of g tiled over the grid
  auto lowpass_adj = [&](int chan, float2 *dst, bool accumulate) -> hipError_t {
    return scat::launch3_tile_phi(Gs, phi, dst, pc, K, chan, n0, n1, n2, Jo, accumulate, st);
  };
  // member p of the pair tables of (j, l) (fused plans)
  auto pair_table = [&](int j, int l, int pr) -> const float2 * {
    return reinterpret_cast<const float2 *>(tab + p->psi3_off[static_cast<size_t>(j) * (L + 1) + l]) +
           static_cast<size_t>(pr) * n;
  };
  // W[m] = IFFT(Fh g_{j,l,m}), acc = sum_m |W[m]|^2.  Fused plans: the tables come in pairs
  // c = g_2p + i g_2p+1 and W[p] = IFFT(Fh c) carries both members (|W[p]|^2 is the sum of
  // their squares, and the adjoint of the product is the product with conj(c)).
  auto filtered = [&](const float2 *Fh, int j, int l, float2 *W, float *acc) -> hipError_t {
    if (p->fused3) {
      // every pair of the node at once: product + inverse slab transform, then axis 0
      hipError_t e = scat::launch3_slab_mul_inv(Fh, pair_table(j, l, 0), W, pc, n0, n1, n2, l + 1, tw,
                                                tw_n, st);
      if (e != hipSuccess) return e;
      return scat::launch3_axis0_back(0, W, acc, nullptr, pc, n0, n1 * n2, l + 1, tw, tw_n, st);
    }
    const int cnt = p->fused3 ? l + 1 : 2 * l + 1;
    for (int m = 0; m < cnt; ++m) {
      float2 *w = W + static_cast<size_t>(m) * tot;
      hipError_t e;
      if (p->fused3) {
        e = scat::launch3_mul_ctable(Fh, pair_table(j, l, m), w, pc, static_cast<long>(n), false, false, st);
      } else {
        int fs;
        const float *t = table(j, l, m, &fs);
        e = scat::launch3_mul_table(Fh, t, w, pc, static_cast<long>(n), st, fs, false);
      }
      if (e != hipSuccess) return e;
      e = fft3(w, true);
      if (e != hipSuccess) return e;
      e = scat::launch3_accum_abs2(w, acc, tot, m == 0, st);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  };
  // A += sum_m g_m FFT(Re(gu) W[m] / sqrt(acc)); W is overwritten
  auto rho_adj = [&](const float2 *gu, int j, int l, float2 *W, const float *acc,
                     float2 *A) -> hipError_t {
    if (p->fused3) {
      hipError_t e = scat::launch3_axis0_back(1, W, const_cast<float *>(acc), gu, pc, n0, n1 * n2,
                                              l + 1, tw, tw_n, st);
      if (e != hipSuccess) return e;
      return scat::launch3_slab_fwd_mulacc(W, pair_table(j, l, 0), A, pc, n0, n1, n2, l + 1, tw, tw_n,
                                           st);
    }
    const int cnt = p->fused3 ? l + 1 : 2 * l + 1;
    for (int m = 0; m < cnt; ++m) {
      float2 *w = W + static_cast<size_t>(m) * tot;
      hipError_t e = scat::launch3_rho_back(gu, acc, w, tot, st);
      if (e != hipSuccess) return e;
      e = fft3(w, false);
      if (e != hipSuccess) return e;
      if (p->fused3) {
        e = scat::launch3_mul_ctable(w, pair_table(j, l, m), A, pc, static_cast<long>(n), true, true, st);
      } else {
        int fs;
        const float *t = table(j, l, m, &fs);
        e = scat::launch3_mul_table(w, t, A, pc, static_cast<long>(n), st, fs, true);
      }
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  };
  // small spectra of the output gradient, all channels of the chunk at once
  SCAT_TRY(scat::launch3_real_to_complex(go, Gs, pc * K * static_cast<long>(mout), st));
  SCAT_TRY(scat::launch3_fft(Gs, pc * K, n0 >> Jo, n1 >> Jo, n2 >> Jo, false, tw, tw_n, st));
  SCAT_TRY(scat::launch3_real_to_complex(x, XH, tot, st));
  SCAT_TRY(fft3(XH, false));
  SCAT_TRY(lowpass_adj(0, AX, false));
  int c1 = 1, c2 = 1 + J * (L + 1);
  for (int j1 = 0; j1 < J; ++j1)
    for (int l = 0; l <= L; ++l) {
      SCAT_TRY(filtered(XH, j1, l, W1, acc1));
      SCAT_TRY(lowpass_adj(c1++, AU, false));
      if (second && j1 < J - 1) {
        SCAT_TRY(scat::launch3_sqrt(acc1, UH, tot, st));
        SCAT_TRY(fft3(UH, false));
        for (int j2 = j1 + 1; j2 < J; ++j2) {
          SCAT_TRY(filtered(UH, j2, l, W2, acc2));
          // gradient of the child's modulus signal: Re IFFT(phi^ FFT(upsample(g)))
          SCAT_TRY(lowpass_adj(c2++, Wk, false));
          SCAT_TRY(fft3(Wk, true));
          SCAT_TRY(rho_adj(Wk, j2, l, W2, acc2, AU));
        }
      }
      SCAT_TRY(fft3(AU, true));
      SCAT_TRY(rho_adj(AU, j1, l, W1, acc1, AX));
    }
  SCAT_TRY(fft3(AX, true));
  SCAT_TRY(scat::launch3_real_part(AX, gi, tot, st));
  return SCAT_OK;
}

// ---- 1-D schedule (four-step transforms: the signal is an n1 x n2 matrix)
scat_status forward_1d(scat_plan *p, const float *in, float *out, long p0, long pc,
                       const Layout &lay, hipStream_t st, const Tape *tape) {
  const scat::HostPlan &h = p->host;
  const int J = h.J, Q = h.LQ, K = h.K;
  const int N1 = p->n1, N2 = p->n2;
  const int N = N1 * N2;
  const int rJ = h.res(J);
  const int mc_out = N2 >> rJ;
  char *base = static_cast<char *>(p->work);
  float2 *XH = reinterpret_cast<float2 *>(base);
  float2 *T = reinterpret_cast<float2 *>(base + lay.xh * pc);
  float2 *U = reinterpret_cast<float2 *>(base + (lay.xh + lay.t) * pc);
  float2 *V = reinterpret_cast<float2 *>(base + (lay.xh + lay.t + lay.u) * pc);
  const float *tab = p->d_tables;
  const float2 *tw = p->d_tw;
  const int tw_n = p->tw_n;
  const float *x = in + static_cast<size_t>(p0) * N;
  float *o = out ? out + static_cast<size_t>(p0) * K * (N >> rJ) : nullptr;
  const bool lp = tape == nullptr;  // form the lowpassed outputs
  const ChanMap none{1, 1, 0, 0};

  // row-pass outputs of the lowpass: channels 1 .. K-1 of every signal, channel-major, for
  // one column pass at the end; then channel 0
  float2 *TL = reinterpret_cast<float2 *>(base + (lay.xh + lay.t + lay.u + lay.v) * pc);
  const int m_out = N >> rJ;
  float2 *TL0 = TL + static_cast<size_t>(pc) * (K - 1) * m_out;
  // lowpass child of nodes at resolution r whose output channels are cm: phi at r, fold to rJ
  auto low_child = [&](int r, ChanMap cm) {
    return scat::Rows1dChild{tab + p->phi_off[r], TL, rJ - r, m_out,
                             ChanMap{cm.G, cm.inner, cm.outer_stride, cm.base - 1}, K - 1};
  };

  SCAT_TRY(scat::launch_col(0, x, pc, N1, N2, XH, N, nullptr, 0, nullptr, nullptr, none, K, tw,
                            tw_n, st));
  // the row transform of x's column spectra: alone, or (plain pass, row lengths the register
  // row kernel takes) by that kernel in place, with the lowpass of S0 as its one child
  const bool s0_rides = lp && scat::rows1d_half_supported(N1, N2);
  if (s0_rides) {
    scat::Rows1dArgs xa;
    xa.n = 1;
    xa.c[0] = scat::Rows1dChild{tab + p->phi_off[0], TL0, rJ, m_out, ChanMap{1, 1, 0, 0}, 0};
    xa.spec_out = XH;
    SCAT_TRY(scat::launch_rows1d(XH, pc, N1, N2, xa, tw, tw_n, st));
  } else {
    SCAT_TRY(scat::launch_row_fwd(XH, pc * N1, N2, tw, tw_n, st));
  }
  // S0
  if (lp) {
    if (!s0_rides) {
      const unsigned long long *m0 = nullptr;
      auto it = p->mask64_off.find({-1, J});
      if (p->d_masks64 != nullptr && it != p->mask64_off.end() && rJ == J) m0 = p->d_masks64 + it->second;
      SCAT_TRY(scat::launch_mulfold_invrow(XH, tab + p->phi_off[0], TL0, pc, 1, N1, N2, 0, rJ, m_out,
                                           tw, tw_n, st, m0));
    }
    // (its column pass: with the other channels' at the end where that launch takes it along)
    if (!(K > 1 && scat::col_out_tail_supported(N1, mc_out, tw_n)))
      SCAT_TRY(scat::launch_col(2, TL0, pc, N1, mc_out, nullptr, 0, nullptr, 0, nullptr, o,
                                ChanMap{1, 1, 0, 0}, K, tw, tw_n, st));
  }
  if (tape == nullptr) {
    // Plain forward pass, breadth first: the row passes of all first-order octaves, ONE column
    // pass over all of them (arrays that differ in their number of columns are segments of one
    // launch), per octave one row pass over its spectra (lowpass + the wavelets of every coarser
    // octave; the children are stored grouped by their own octave j2, node (signal, j1, k)),
    // one column pass over all second-order nodes and one lowpass row pass per child octave.
    size_t off1[scat::kRows1dMaxChildren + 1] = {0}, t2_off[scat::kRows1dMaxChildren + 1] = {0};
    size_t tot1 = 0, tot2 = 0;
    for (int j = 0; j < J; ++j) {
      off1[j] = tot1;
      tot1 += static_cast<size_t>(Q) * (N >> h.res(j));
    }
    for (int j2 = 1; h.max_order == 2 && j2 < J; ++j2) {
      t2_off[j2] = tot2;
      tot2 += static_cast<size_t>(j2) * Q * (N >> h.res(j2));
    }
    float2 *T2 = T + tot1 * pc;
    // The columns are real after the modulus: where every octave's shape allows it, the column
    // passes write rows 0 .. N1/2 of each spectrum only (compactly, at the start of the node's
    // place) and the row passes derive the other rows from them.
    bool half = N1 == 32 || N1 == 64 || N1 == 128 || N1 == 256;
    for (int j = 0; half && j < J; ++j) half = (N2 >> h.res(j)) >= 4 && scat::rows1d_half_supported(N1, N2 >> h.res(j));
    // column passes (mode 1 with the four-step twiddle) over a list of arrays
    auto cols_pass = [&](const float2 *src, float2 *dst, const std::vector<scat::ColSeg> &all) -> scat_status {
      // (half spectra: two columns per thread in the merged launch, which also takes narrow arrays)
      const int least = half ? 4 : 16;
      std::vector<scat::ColSeg> together;
      for (const scat::ColSeg &sg : all)
        if (N1 == 256 && sg.Mc >= least && static_cast<int>(together.size()) < scat::kColMaxSegs) together.push_back(sg);
      const bool merged = together.size() >= 2;
      if (merged)
        SCAT_TRY(scat::launch_col_segs(src, dst, N1, together.data(), static_cast<int>(together.size()), half, tw,
                                       tw_n, st));
      size_t taken = 0;
      for (const scat::ColSeg &sg : all) {
        if (merged && N1 == 256 && sg.Mc >= least && taken < together.size()) {
          ++taken;
          continue;
        }
        SCAT_TRY(scat::launch_col(1, src + sg.src_off, sg.nodes, N1, sg.Mc, dst + sg.uc_off, N1 * sg.Mc, nullptr, 0,
                                  nullptr, nullptr, none, K, tw, tw_n, st, half));
      }
      return SCAT_OK;
    };
    std::vector<scat::ColSeg> segs;
    for (int j1 = 0; j1 < J; ++j1) {
      const int r1 = h.res(j1);
      const unsigned long long *m1 = nullptr;
      {
        auto it = p->mask64_off.find({0, j1});
        if (p->d_masks64 != nullptr && it != p->mask64_off.end() && r1 == j1) m1 = p->d_masks64 + it->second;
      }
      SCAT_TRY(scat::launch_mulfold_invrow(XH, tab + p->psi1_off[j1], T + off1[j1] * pc, pc, Q, N1, N2, 0, r1,
                                           N >> r1, tw, tw_n, st, m1));
      segs.push_back(scat::ColSeg{pc * Q, N2 >> r1, static_cast<long long>(off1[j1] * pc),
                                  static_cast<long long>(off1[j1] * pc)});
    }
    SCAT_TRY(cols_pass(T, U, segs));
    for (int j1 = 0; j1 < J; ++j1) {
      const int r1 = h.res(j1);
      scat::Rows1dArgs ch;
      ch.n = 0;
      ch.c[ch.n++] = low_child(r1, ChanMap{Q, Q, 0, 1 + j1 * Q});
      for (int j2 = j1 + 1; h.max_order == 2 && j2 < J; ++j2) {
        const int r2 = h.res(j2);
        // node (signal, k) of this octave is signal number (signal * j2 + j1) * Q + k of group j2
        ch.c[ch.n++] = scat::Rows1dChild{tab + p->psi2_off[{r1, j2}], T2 + t2_off[j2] * pc, r2 - r1, N >> r2,
                                         ChanMap{Q, Q, 0, j1 * Q}, j2 * Q};
      }
      SCAT_TRY(scat::launch_rows1d(U + off1[j1] * pc, pc * Q, N1, N2 >> r1, ch, tw, tw_n, st, half));
    }
    if (h.max_order == 2 && J >= 2) {
      segs.clear();
      for (int j2 = 1; j2 < J; ++j2)
        segs.push_back(scat::ColSeg{pc * j2 * Q, N2 >> h.res(j2), static_cast<long long>(t2_off[j2] * pc),
                                    static_cast<long long>(t2_off[j2] * pc)});
      SCAT_TRY(cols_pass(T2, V, segs));
      for (int j2 = 1; j2 < J; ++j2) {
        const int r2 = h.res(j2);
        scat::Rows1dArgs lc;
        lc.n = 1;
        lc.c[0] = low_child(r2, ChanMap{j2 * Q, 1, 0, 1});
        lc.c[0].chan_tab = p->d_chan1d + p->chan1d_off[j2];
        SCAT_TRY(scat::launch_rows1d(V + t2_off[j2] * pc, pc * j2 * Q, N1, N2 >> r2, lc, tw, tw_n, st, half));
      }
    }
    if (K > 1) {
      if (scat::col_out_tail_supported(N1, mc_out, tw_n))
        SCAT_TRY(scat::launch_col_out_tail(TL, pc * (K - 1), pc, mc_out, o, ChanMap{K - 1, K - 1, 0, 1}, K, tw, tw_n,
                                           st));
      else
        SCAT_TRY(scat::launch_col(2, TL, pc * (K - 1), N1, mc_out, nullptr, 0, nullptr, 0, nullptr, o,
                                  ChanMap{K - 1, K - 1, 0, 1}, K, tw, tw_n, st));
    }
    return SCAT_OK;
  }
  // Taped pass: every node is taped as its row pass leaves it, before the inverse column
  // transform, which the backward pass's column kernel does itself: the row pass writes
  // straight into the tape, a leaf (no children below it) needs no column kernel here, and
  // the column kernel of a node with children writes their spectra only.
  for (int j1 = 0; j1 < J; ++j1) {
    const int r1 = h.res(j1);
    const int Mc1 = N2 >> r1;
    const int M1 = N >> r1;
    const bool kids = h.max_order == 2 && j1 < J - 1;
    float2 *t1 = tape->base + tape->y1_off[j1] * pc;
    const unsigned long long *m1 = nullptr;
    {
      auto it = p->mask64_off.find({0, j1});
      if (p->d_masks64 != nullptr && it != p->mask64_off.end() && r1 == j1) m1 = p->d_masks64 + it->second;
    }
    SCAT_TRY(scat::launch_mulfold_invrow(XH, tab + p->psi1_off[j1], t1, pc, Q, N1, N2, 0, r1, M1,
                                         tw, tw_n, st, m1));
    if (!kids) continue;
    // (half spectra between the two passes where the shapes allow it, as in the plain pass)
    const bool half_t = (N1 == 32 || N1 == 64 || N1 == 128 || N1 == 256) && Mc1 >= 4 &&
                        scat::rows1d_half_supported(N1, Mc1);
    SCAT_TRY(scat::launch_col(1, t1, pc * Q, N1, Mc1, U, M1, nullptr, 0, nullptr, nullptr, none, K,
                              tw, tw_n, st, half_t));
    scat::Rows1dArgs ch;
    ch.n = 0;
    for (int j2 = j1 + 1; j2 < J; ++j2) {
      const int r2 = h.res(j2);
      ch.c[ch.n++] = scat::Rows1dChild{tab + p->psi2_off[{r1, j2}], tape->base + tape->y2_off.at({j1, j2}) * pc,
                                       r2 - r1, N >> r2, ChanMap{1, 1, 0, 0}, 0};
    }
    SCAT_TRY(scat::launch_rows1d(U, pc * Q, N1, Mc1, ch, tw, tw_n, st, half_t));
  }
  return SCAT_OK;
}

// Makes the plan's scratch buffer at least `need` bytes (growing it synchronises the device).
scat_status ensure_scratch(scat_plan *plan, size_t need) {
  plan->work = plan->d_scratch;
  if (need <= plan->scratch_bytes) return SCAT_OK;
  if (hipDeviceSynchronize() != hipSuccess) return SCAT_ERR_DEVICE;
  if (plan->d_scratch) (void)hipFree(plan->d_scratch);
  plan->d_scratch = nullptr;
  plan->work = nullptr;
  plan->scratch_bytes = 0;
  if (hipMalloc(&plan->d_scratch, need) != hipSuccess) return SCAT_ERR_ALLOC;
  plan->scratch_bytes = need;
  plan->work = plan->d_scratch;
  return SCAT_OK;
}

// Routes the launches of one call to the plan's timer while it records.
struct ObserverScope {
  explicit ObserverScope(scat_plan *plan) {
    scat::set_launch_observer(plan->timer.enabled ? &plan->timer : nullptr);
  }
  ~ObserverScope() { scat::set_launch_observer(nullptr); }
};

// The chunk loop of a forward call: `lay.chunk` planes at a time through the schedule of the
// plan, all on `st`, using the scratch plan->work points at (lay.per_plane * lay.chunk bytes).
scat_status forward_chunks(scat_plan *plan, const float *in, float *out, long batch, const Layout &lay,
                           hipStream_t st, bool observe = true) {
  struct NoObserver {
    scat_plan *p;
    bool was;
    explicit NoObserver(scat_plan *q, bool off) : p(q), was(q->timer.enabled) {
      if (off) p->timer.enabled = false;
    }
    ~NoObserver() { p->timer.enabled = was; }
  } no_observer(plan, !observe);  // (the timer creates HIP events on demand)
  ObserverScope observer_scope(plan);
  const scat::HostPlan &h = plan->host;
  for (long p0 = 0; p0 < batch; p0 += lay.chunk) {
    long pc = batch - p0 < lay.chunk ? batch - p0 : lay.chunk;
    const float *cin = in;
    float *cout = out;
    long cp0 = p0;
    float *xp = nullptr, *op = nullptr;
    if (plan->padded) {
      // extend this chunk's signals into scratch and transform them as planes 0..pc-1
      char *tail = static_cast<char *>(plan->work) +
                   (lay.xh + lay.t + lay.u + lay.v + lay.w) * static_cast<size_t>(lay.chunk);
      xp = reinterpret_cast<float *>(tail);
      op = reinterpret_cast<float *>(tail + lay.pad_in * static_cast<size_t>(lay.chunk));
      if (h.dims == 3) {
        const int *u = plan->user_shape3, *g = plan->h3.shape;
        hipLaunchKernelGGL(k_pad_symmetric3, dim3(stream_blocks(pc * static_cast<long>(plan->h3.points()))),
                           dim3(256), 0, st, in + static_cast<size_t>(p0) * u[0] * u[1] * u[2], xp, pc,
                           u[0], u[1], u[2], g[0], g[1], g[2]);
      } else {
        const int ur = plan->user_shape[0], uc = plan->user_shape[1];
        hipLaunchKernelGGL(k_pad_symmetric, dim3(stream_blocks(pc * h.shape[0] * h.shape[1])),
                           dim3(256), 0, st, in + static_cast<size_t>(p0) * ur * uc, xp, pc, ur, uc,
                           h.shape[0], h.shape[1]);
      }
      if (hipGetLastError() != hipSuccess) return SCAT_ERR_DEVICE;
      cin = xp;
      cout = op;
      cp0 = 0;
    }
    scat_status s = h.dims == 3   ? (plan->fused3 ? forward_3d_fused(plan, cin, cout, cp0, pc, st)
                                                  : forward_3d(plan, cin, cout, cp0, pc, st))
                    : h.dims == 1 ? forward_1d(plan, cin, cout, cp0, pc, lay, st)
                    : plan->tree  ? forward_2d_tree(plan, cin, cout, cp0, pc, lay, st)
                    : plan->node  ? forward_2d_node(plan, cin, cout, cp0, pc, lay, st)
                    : plan->fused ? forward_2d_fused(plan, cin, cout, cp0, pc, lay, st)
                                  : forward_2d(plan, cin, cout, cp0, pc, lay, st);
    if (s != SCAT_OK) return s;
    if (plan->padded && h.dims == 3) {
      const int Jo = plan->h3.out_shift();
      const int *g = plan->h3.shape, *o = plan->user_out3;
      const long maps = pc * h.K;
      hipLaunchKernelGGL(k_crop3, dim3(stream_blocks(maps * o[0] * o[1] * o[2])), dim3(256), 0, st, op,
                         out + static_cast<size_t>(p0) * h.K * o[0] * o[1] * o[2], maps, g[0] >> Jo,
                         g[1] >> Jo, g[2] >> Jo, o[0], o[1], o[2]);
      if (hipGetLastError() != hipSuccess) return SCAT_ERR_DEVICE;
    } else if (plan->padded) {
      const int m_r = h.dims == 2 ? h.shape[0] >> h.res(h.J) : 1, m_c = h.shape[1] >> h.res(h.J);
      const int o_r = plan->user_out[0], o_c = plan->user_out[1];
      hipLaunchKernelGGL(k_crop, dim3(stream_blocks(pc * h.K * o_r * o_c)), dim3(256), 0, st, op,
                         out + static_cast<size_t>(p0) * h.K * o_r * o_c, pc * h.K, m_r, m_c, o_r,
                         o_c);
      if (hipGetLastError() != hipSuccess) return SCAT_ERR_DEVICE;
    }
  }
  return SCAT_OK;
}

}  // namespace

extern "C" {

scat_status scat_plan_create(scat_plan **out_plan, int dims, const int *shape, int J, int LQ,
                             int max_order) {
  return create_common(out_plan, dims, shape, J, LQ, max_order, true);
}

scat_status scat_plan_create_padded(scat_plan **out_plan, int dims, const int *shape, int J,
                                    int LQ, int max_order) {
  return create_common(out_plan, dims, shape, J, LQ, max_order, true, true);
}

scat_status scat_plan_create_padded_host(scat_plan **out_plan, int dims, const int *shape, int J,
                                         int LQ, int max_order) {
  return create_common(out_plan, dims, shape, J, LQ, max_order, false, true);
}

scat_status scat_plan_create_ex(scat_plan **out_plan, int dims, const int *shape, int J, int LQ,
                                int max_order, int oversampling, int flags) {
  if (flags & ~15) {
    if (out_plan != nullptr) *out_plan = nullptr;
    return SCAT_ERR_ARG;
  }
  return create_common(out_plan, dims, shape, J, LQ, max_order, (flags & SCAT_PLAN_HOST_ONLY) == 0,
                       (flags & SCAT_PLAN_PADDED) != 0, oversampling,
                       (flags & SCAT_PLAN_PASS_KERNELS) == 0);
}

scat_status scat_plan_grid_shape(const scat_plan *plan, int *shape_out) {
  if (plan == nullptr || shape_out == nullptr) return SCAT_ERR_NULL;
  const scat::HostPlan &h = plan->host;
  if (h.dims == 3) {
    for (int d = 0; d < 3; ++d) shape_out[d] = plan->h3.shape[d];
    return SCAT_OK;
  }
  if (h.dims == 2) shape_out[0] = h.shape[0];
  shape_out[h.dims == 2 ? 1 : 0] = h.shape[1];
  return SCAT_OK;
}

scat_status scat_plan_create_host(scat_plan **out_plan, int dims, const int *shape, int J, int LQ,
                                  int max_order) {
  return create_common(out_plan, dims, shape, J, LQ, max_order, false);
}

scat_status scat_forward(scat_plan *plan, const float *in, float *out, long batch, void *stream) {
  if (plan == nullptr) return SCAT_ERR_NULL;
  if (batch < 0) return SCAT_ERR_ARG;
  if (batch == 0) return SCAT_OK;
  if (in == nullptr || out == nullptr) return SCAT_ERR_NULL;
  if (!plan->has_device) return SCAT_ERR_DEVICE;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != plan->device) return SCAT_ERR_DEVICE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const Layout lay = make_layout(*plan, batch);
  const size_t need = lay.per_plane * static_cast<size_t>(lay.chunk);
  {
    const scat_status grown = ensure_scratch(plan, need);
    if (grown != SCAT_OK) return grown;
  }
  return forward_chunks(plan, in, out, batch, lay, st);
}

scat_status scat_plan_reserve(scat_plan *plan, long batch, int with_backward) {
  if (plan == nullptr) return SCAT_ERR_NULL;
  if (batch < 1) return SCAT_ERR_ARG;
  if (!plan->has_device) return SCAT_ERR_DEVICE;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != plan->device) return SCAT_ERR_DEVICE;
  size_t need = scat_plan_workspace_bytes(plan, batch);
  if (with_backward) need = std::max(need, scat_plan_backward_workspace_bytes(plan, batch));
  if (need <= plan->scratch_bytes) return SCAT_OK;
  return ensure_scratch(plan, need);
}

scat_status scat_forward_static(scat_plan *plan, const float *in, float *out, long batch,
                                void *stream) {
  if (plan == nullptr) return SCAT_ERR_NULL;
  if (batch < 0) return SCAT_ERR_ARG;
  if (batch == 0) return SCAT_OK;
  if (in == nullptr || out == nullptr) return SCAT_ERR_NULL;
  if (!plan->has_device || plan->static_scratch == nullptr) return SCAT_ERR_DEVICE;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != plan->device) return SCAT_ERR_DEVICE;
  const Layout lay = make_layout(*plan, batch, kStaticScratchBytes);
  if (lay.per_plane > kStaticScratchBytes) return SCAT_ERR_WORKSPACE;
  plan->work = plan->static_scratch;
  return forward_chunks(plan, in, out, batch, lay, static_cast<hipStream_t>(stream), false);
}

scat_status scat_backward(scat_plan *plan, const float *in, const float *grad_out, float *grad_in,
                          long batch, void *stream) {
  if (plan == nullptr) return SCAT_ERR_NULL;
  if (batch < 0) return SCAT_ERR_ARG;
  const scat::HostPlan &h = plan->host;
  if (h.dims == 3) {
    if (batch == 0) return SCAT_OK;
    if (in == nullptr || grad_out == nullptr || grad_in == nullptr) return SCAT_ERR_NULL;
    if (!plan->has_device) return SCAT_ERR_DEVICE;
    int dev3 = -1;
    if (hipGetDevice(&dev3) != hipSuccess || dev3 != plan->device) return SCAT_ERR_DEVICE;
    hipStream_t st3 = static_cast<hipStream_t>(stream);
    // padded plans: extended input, its gradient and the zero-extended output gradient
    // sit behind the periodic pass's buffers
    const size_t n3 = plan->h3.points(), mout3 = n3 >> (3 * plan->h3.out_shift());
    const size_t core = bytes_per_volume_3d_bwd(*plan);
    const size_t per = core + (plan->padded ? (2 * n3 + h.K * mout3) * sizeof(float) : 0);
    long chunk = static_cast<long>(scratch_budget() / per);
    if (chunk < 1) chunk = 1;
    if (chunk > batch) chunk = batch;
    const size_t need3 = per * static_cast<size_t>(chunk);
    {
    const scat_status grown = ensure_scratch(plan, need3);
    if (grown != SCAT_OK) return grown;
  }
  ObserverScope observer_scope(plan);
    for (long p0 = 0; p0 < batch; p0 += chunk) {
      const long pc = batch - p0 < chunk ? batch - p0 : chunk;
      if (!plan->padded) {
        scat_status s3 = backward_3d(plan, in, grad_out, grad_in, p0, pc, st3);
        if (s3 != SCAT_OK) return s3;
        continue;
      }
      const int *u = plan->user_shape3, *g = plan->h3.shape, *o = plan->user_out3;
      const int Jo = plan->h3.out_shift();
      const size_t un = static_cast<size_t>(u[0]) * u[1] * u[2];
      const size_t on = static_cast<size_t>(o[0]) * o[1] * o[2];
      float *xp = reinterpret_cast<float *>(static_cast<char *>(plan->work) +
                                            core * static_cast<size_t>(chunk));
      float *gxp = xp + n3 * chunk;
      float *gop = gxp + n3 * chunk;
      hipLaunchKernelGGL(k_pad_symmetric3, dim3(stream_blocks(pc * static_cast<long>(n3))), dim3(256), 0,
                         st3, in + static_cast<size_t>(p0) * un, xp, pc, u[0], u[1], u[2], g[0], g[1],
                         g[2]);
      hipLaunchKernelGGL(k_uncrop3, dim3(stream_blocks(pc * h.K * static_cast<long>(mout3))), dim3(256),
                         0, st3, grad_out + static_cast<size_t>(p0) * h.K * on, gop, pc * h.K,
                         g[0] >> Jo, g[1] >> Jo, g[2] >> Jo, o[0], o[1], o[2]);
      if (hipGetLastError() != hipSuccess) return SCAT_ERR_DEVICE;
      scat_status s3 = backward_3d(plan, xp, gop, gxp, 0, pc, st3);
      if (s3 != SCAT_OK) return s3;
      hipLaunchKernelGGL(k_unpad_symmetric3, dim3(stream_blocks(pc * static_cast<long>(un))), dim3(256),
                         0, st3, gxp, grad_in + static_cast<size_t>(p0) * un, pc, u[0], u[1], u[2], g[0],
                         g[1], g[2]);
      if (hipGetLastError() != hipSuccess) return SCAT_ERR_DEVICE;
    }
    return SCAT_OK;
  }
  if (h.dims == 1) {
    // signals are n1 x n2 matrices: n1-point column transforms, row transforms of n2 >> r
    if (!scat::backward_side_supported(plan->n1) || plan->n2 > 512) return SCAT_ERR_SHAPE;
  } else {
    // every grid of the cascade must have sides the plain transforms handle, and the
    // output grid must fit the adjoint lowpass kernel's LDS stage
    const int small_r = plan->n1 >> h.res(h.J - 1), small_c = plan->n2 >> h.res(h.J - 1);
    const int m_r = plan->n1 >> h.res(h.J), m_c = plan->n2 >> h.res(h.J);
    const bool grid_ok = scat::small_fft2_supported(m_r, m_c);
    if (!scat::backward_side_supported(plan->n1) || !scat::backward_side_supported(plan->n2) ||
        !scat::backward_side_supported(small_r) || !scat::backward_side_supported(small_c) || !grid_ok)
      return SCAT_ERR_SHAPE;
  }
  if (batch == 0) return SCAT_OK;
  if (in == nullptr || grad_out == nullptr || grad_in == nullptr) return SCAT_ERR_NULL;
  if (!plan->has_device) return SCAT_ERR_DEVICE;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != plan->device) return SCAT_ERR_DEVICE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  BwdLayout bl = make_bwd_layout(*plan, batch);
  const size_t need = bl.per_plane * static_cast<size_t>(bl.chunk);
  {
    const scat_status grown = ensure_scratch(plan, need);
    if (grown != SCAT_OK) return grown;
  }
  ObserverScope observer_scope(plan);
  for (long p0 = 0; p0 < batch; p0 += bl.chunk) {
    long pc = batch - p0 < bl.chunk ? batch - p0 : bl.chunk;
    if (!plan->padded) {
      scat_status s = h.dims == 1 ? backward_1d(plan, in, grad_out, grad_in, p0, pc, bl, st)
                                  : backward_2d(plan, in, grad_out, grad_in, p0, pc, bl, st);
      if (s != SCAT_OK) return s;
      continue;
    }
    // padded plan: extend the input and (with zeros) the output gradient to the periodic
    // grid, run the periodic backward pass there, fold the extended gradient back
    // (a 1-D signal is one row of n1 * n2 samples here, whatever its matrix form inside)
    const size_t n = static_cast<size_t>(plan->n1) * plan->n2;
    const int P_r = h.dims == 1 ? 1 : plan->n1, P_c = h.dims == 1 ? static_cast<int>(n) : plan->n2;
    const int m_r = P_r >> (h.dims == 1 ? 0 : h.res(h.J)), m_c = P_c >> h.res(h.J);
    const int ur = plan->user_shape[0], uc = plan->user_shape[1];
    const int o_r = plan->user_out[0], o_c = plan->user_out[1];
    float *xp = reinterpret_cast<float *>(static_cast<char *>(plan->work) +
                                          (bl.per_plane - bl.pad_floats * sizeof(float)) *
                                              static_cast<size_t>(bl.chunk));
    float *gxp = xp + n * bl.chunk;
    float *gop = gxp + n * bl.chunk;
    hipLaunchKernelGGL(k_pad_symmetric, dim3(stream_blocks(pc * static_cast<long>(n))), dim3(256), 0,
                       st, in + static_cast<size_t>(p0) * ur * uc, xp, pc, ur, uc, P_r, P_c);
    hipLaunchKernelGGL(k_uncrop, dim3(stream_blocks(pc * h.K * m_r * m_c)), dim3(256), 0, st,
                       grad_out + static_cast<size_t>(p0) * h.K * o_r * o_c, gop, pc * h.K, m_r, m_c,
                       o_r, o_c);
    if (hipGetLastError() != hipSuccess) return SCAT_ERR_DEVICE;
    scat_status s = h.dims == 1 ? backward_1d(plan, xp, gop, gxp, 0, pc, bl, st)
                                : backward_2d(plan, xp, gop, gxp, 0, pc, bl, st);
    if (s != SCAT_OK) return s;
    hipLaunchKernelGGL(k_unpad_symmetric, dim3(stream_blocks(pc * ur * uc)), dim3(256), 0, st, gxp,
                       grad_in + static_cast<size_t>(p0) * ur * uc, pc, ur, uc, P_r, P_c);
    if (hipGetLastError() != hipSuccess) return SCAT_ERR_DEVICE;
  }
  return SCAT_OK;
}

size_t scat_plan_backward_workspace_bytes(const scat_plan *plan, long batch) {
  if (plan == nullptr || batch <= 0) return 0;
  if (plan->host.dims == 3) {
    const size_t n3 = plan->h3.points(), mout3 = n3 >> (3 * plan->h3.out_shift());
    const size_t per = bytes_per_volume_3d_bwd(*plan) +
                       (plan->padded ? (2 * n3 + plan->host.K * mout3) * sizeof(float) : 0);
    long chunk = static_cast<long>(scratch_budget() / per);
    if (chunk < 1) chunk = 1;
    return per * static_cast<size_t>(chunk > batch ? batch : chunk);
  }
  const BwdLayout bl = make_bwd_layout(*plan, batch);
  return bl.per_plane * static_cast<size_t>(bl.chunk);
}

scat_status scat_plan_destroy(scat_plan *plan) {
  if (plan == nullptr) return SCAT_OK;
  if (plan->has_device) {
    int cur = -1;
    bool sw = hipGetDevice(&cur) == hipSuccess && cur != plan->device;
    if (sw) (void)hipSetDevice(plan->device);
    (void)hipDeviceSynchronize();
    plan->timer.release();
    free_device(plan);
    if (sw) (void)hipSetDevice(cur);
  }
  delete plan;
  return SCAT_OK;
}

int scat_plan_num_coeffs(const scat_plan *plan) { return plan ? plan->host.K : -1; }

scat_status scat_plan_out_shape(const scat_plan *plan, int *shape_out) {
  if (plan == nullptr || shape_out == nullptr) return SCAT_ERR_NULL;
  const scat::HostPlan &h = plan->host;
  if (h.dims == 3) {
    for (int d = 0; d < 3; ++d)
      shape_out[d] = plan->padded ? plan->user_out3[d] : plan->h3.shape[d] >> plan->h3.out_shift();
    return SCAT_OK;
  }
  if (plan->padded) {
    if (h.dims == 2) shape_out[0] = plan->user_out[0];
    shape_out[h.dims == 2 ? 1 : 0] = plan->user_out[1];
  } else if (h.dims == 2) {
    shape_out[0] = h.shape[0] >> h.res(h.J);
    shape_out[1] = h.shape[1] >> h.res(h.J);
  } else {
    shape_out[0] = h.shape[1] >> h.res(h.J);
  }
  return SCAT_OK;
}

scat_status scat_plan_coeff_index(const scat_plan *plan, int c, int idx[5]) {
  if (plan == nullptr || idx == nullptr) return SCAT_ERR_NULL;
  if (c < 0 || c >= plan->host.K) return SCAT_ERR_ARG;
  if (plan->host.dims == 3) {
    const scat::Coeff3D &r3 = plan->h3.index[c];
    idx[0] = r3.order;
    idx[1] = r3.j1;
    idx[2] = r3.l;
    idx[3] = r3.j2;
    idx[4] = -1;
    return SCAT_OK;
  }
  const scat::CoeffRow &r = plan->host.index[c];
  idx[0] = r.order;
  idx[1] = r.j1;
  idx[2] = r.t1;
  idx[3] = r.j2;
  idx[4] = r.t2;
  return SCAT_OK;
}

size_t scat_plan_workspace_bytes(const scat_plan *plan, long batch) {
  if (plan == nullptr || batch <= 0) return 0;
  const Layout lay = make_layout(*plan, batch);
  return lay.per_plane * static_cast<size_t>(lay.chunk);
}

scat_status scat_plan_filter(const scat_plan *plan, int kind, int index, int res,
                             double *out_host) {
  if (plan == nullptr || out_host == nullptr) return SCAT_ERR_NULL;
  if (plan->host.dims == 3) {
    // kind 0: the lowpass; kind 1: index = j (L+1) + l gives that pair's 2l+1 real tables
    const scat::HostPlan3D &h3 = plan->h3;
    if (res != 0) return SCAT_ERR_ARG;
    const std::vector<double> *v = nullptr;
    if (kind == 0 && index == 0) v = &h3.phi;
    if (kind == 1 && index >= 0 && index < static_cast<int>(h3.psi.size())) v = &h3.psi[index];
    if (v == nullptr) return SCAT_ERR_ARG;
    std::memcpy(out_host, v->data(), v->size() * sizeof(double));
    return SCAT_OK;
  }
  const FilterTable *t = plan->host.find(kind, index, res);
  if (t == nullptr) return SCAT_ERR_ARG;
  std::memcpy(out_host, t->v.data(), t->v.size() * sizeof(double));
  return SCAT_OK;
}

scat_status scat_plan_timing_begin(scat_plan *plan, const char *kernel_name) {
  if (plan == nullptr) return SCAT_ERR_NULL;
  if (!plan->has_device) return SCAT_ERR_DEVICE;
  LaunchTimer &t = plan->timer;
  t.rows.clear();
  t.pair_row.clear();
  t.failed = false;
  t.only = kernel_name ? kernel_name : "";
  t.enabled = true;
  return SCAT_OK;
}

int scat_plan_timing_end(scat_plan *plan) {
  if (plan == nullptr || !plan->timer.enabled) return -1;
  plan->timer.enabled = false;
  if (!plan->timer.collect()) return -1;
  return static_cast<int>(plan->timer.rows.size());
}

scat_status scat_plan_timing_row(const scat_plan *plan, int row, char *name, size_t name_len,
                                 long *launches, double *ms, double *alg_bytes,
                                 double *model_flops) {
  if (plan == nullptr) return SCAT_ERR_NULL;
  if (row < 0 || row >= static_cast<int>(plan->timer.rows.size())) return SCAT_ERR_ARG;
  const LaunchTimer::Row &r = plan->timer.rows[row];
  if (name != nullptr && name_len > 0) {
    std::strncpy(name, r.name.c_str(), name_len - 1);
    name[name_len - 1] = 0;
  }
  if (launches) *launches = r.launches;
  if (ms) *ms = r.ms;
  if (alg_bytes) *alg_bytes = r.bytes;
  if (model_flops) *model_flops = r.flops;
  return SCAT_OK;
}

const char *scat_status_string(scat_status s) {
  switch (s) {
    case SCAT_OK: return "ok";
    case SCAT_ERR_ARG: return "invalid argument";
    case SCAT_ERR_SHAPE: return "shape must be powers of two, each at least 2^J";
    case SCAT_ERR_ALLOC: return "allocation failed";
    case SCAT_ERR_DEVICE: return "GPU error or plan has no device state";
    case SCAT_ERR_NULL: return "null pointer";
    case SCAT_ERR_WORKSPACE: return "one plane needs more scratch than the static buffer holds";
  }
  return "unknown status";
}

}  // extern "C"
