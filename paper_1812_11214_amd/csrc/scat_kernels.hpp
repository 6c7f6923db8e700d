// Launch wrappers of the generic scattering kernels (see scat_kernels.hip).
#pragma once

#include <hip/hip_runtime.h>

namespace scat {

// Where a kernel's node number g (within one input plane p) lands in the output:
// channel = base + (g / inner) * outer_stride + (g % inner), node = p * G + g.
struct ChanMap {
  int G, inner, outer_stride, base;
};

hipError_t launch_mulfold_invrow(const float2 *src, const float *filt, float2 *dst, long S, int F,
                                 int Sr, int Sc, int fr, int fc, int post_tw_m, const float2 *tw,
                                 int tw_n, hipStream_t st);

hipError_t launch_col(int mode, const void *src, long nodes, int Mr, int Mc, float2 *uc,
                      int post_tw_m, const float *phi_rows, int m_r, float *w_out, float *out,
                      ChanMap cm, int K, const float2 *tw, int tw_n, hipStream_t st);

hipError_t launch_row_fwd(float2 *data, long rows, int Mc, const float2 *tw, int tw_n,
                          hipStream_t st);

hipError_t launch_row_lowpass(const float *w, long nodes, int m_r, int Mc, int m_c,
                              const float *phi_cols, float *out, ChanMap cm, int K,
                              const float2 *tw, int tw_n, hipStream_t st);

}  // namespace scat
