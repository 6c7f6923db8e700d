/*
 * scat.h -- C ABI of the MI355X wavelet scattering library (order <= 2; 1-D and 2-D Morlet
 * cascades, 3-D solid harmonic scattering).
 *
 * The operation is the scattering transform of the Kymatio paper (arXiv 1812.11214),
 * section 2: with a lowpass phi_J and wavelet banks psi_lambda on a periodic grid,
 *
 *     S0 x[n]                = (x (*) phi_J)[n]
 *     S1 x[n, l1]            = (|x (*) psi_l1| (*) phi_J)[n]
 *     S2 x[n, l1, l2]        = (||x (*) psi_l1| (*) psi_l2| (*) phi_J)[n],  |l2| > |l1|
 *
 * ((*) = periodic convolution), computed as that section's "Implementation" paragraph
 * describes: products in the Fourier domain, every filtered signal downsampled, the
 * tree walked one first-order branch after the other.  Downsampling schedule (the
 * paper names none): a signal filtered by a wavelet of octave j lives on the grid
 * subsampled by 2^j, the output on the grid subsampled by 2^J, sample phase 0.
 *
 * Filters (the paper names Morlet wavelets and gives no constants): sigma_j = 0.8*2^j,
 * xi_j = (3 pi/4) 2^-j, 2-D slant 4/L and angles pi*l/L, phi_J a Gaussian with
 * sigma = 0.8*2^J; 1-D first order has Q wavelets per octave, xi_k = (3 pi/4) 2^(-k/Q),
 * sigma_k = 0.3 pi / (xi_k (1 - 2^(-1/Q))) (0.8*2^k when Q = 1), second order one
 * wavelet per octave.
 *
 * All pointers named `in`/`out`/`grad_*` are DEVICE pointers; everything else is host
 * memory.  Every function returns a status and never throws or aborts.  The library needs
 * a GPU for the plan constructors without "host" in their name (or flag), scat_forward and
 * scat_backward only.
 */
#ifndef SCAT_H
#define SCAT_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct scat_plan scat_plan; /* opaque, owned by the library */

typedef enum {
  SCAT_OK = 0,
  SCAT_ERR_ARG = 1,    /* bad dims / J / L / Q / max_order / batch / index */
  SCAT_ERR_SHAPE = 2,  /* a side is not a power of two, is smaller than 2^J, or is outside the
                          range the called function supports */
  SCAT_ERR_ALLOC = 3,  /* host or device allocation failed */
  SCAT_ERR_DEVICE = 4, /* a HIP call failed (no device, launch error, ...) */
  SCAT_ERR_NULL = 5,   /* a required pointer is NULL */
  SCAT_ERR_WORKSPACE = 6 /* scat_forward_static: one plane of this plan needs more scratch than
                            the library's static buffer holds */
} scat_status;

/*
 * Build a plan: coefficient index table, filter bank (evaluated in fp64 from the
 * analytic Fourier transforms, summed over 2 pi aliases, folded to every resolution the
 * cascade uses, pre-scaled by the inverse-transform normalisation, stored as fp32) and
 * FFT twiddle tables, uploaded to the current HIP device.
 *
 *   dims       1 or 2 (3: see below)
 *   shape      host array of `dims` ints; each a power of two and >= 2^J (2-D: rows, cols)
 *   J          number of octaves, >= 1; the output grid is shape >> J
 *   LQ         2-D: number of angles L >= 1;  1-D: first-order wavelets per octave Q >= 1
 *   max_order  1 or 2
 *
 * dims = 3 makes a plan for the paper's 3-D transform (section 2: solid harmonic wavelets
 * psi_{j,l,m}, non-linearity rho(x (*) psi_{j,l}) = sqrt(sum_m |x (*) psi_{j,l,m}|^2) in
 * place of the modulus):
 *
 *   shape      3 ints (slowest axis first), each a power of two in 4...256 and >= 2^J
 *   J          number of scales 1...8, j = 0...J-1;  LQ = L, the largest degree, 0...8
 *   channels   K = 1 + J(L+1) + (L+1) J(J-1)/2: S0; S1 by (j, l); S2 by (j1, l, j2) with the
 *              same degree l in both layers and j2 > j1
 *
 * The paper prints no 3-D formulas; the reading: psi_{l,m}(u) = (2 pi)^(-3/2) e^(-|u|^2/2)
 * |u|^l Y_l^m(u/|u|) dilated by 2^j with unit L1 scaling, phi_J a unit-mass Gaussian of
 * standard deviation 2^J, both sampled at the integers and periodised; every convolution is
 * evaluated on the full grid and the lowpassed result read at the samples 2^J n.  Since rho
 * does not depend on the orthonormal basis of the degree-l harmonics, the tables hold the
 * real harmonics.  scat_plan_create_padded / SCAT_PLAN_PADDED: volumes of any size up to
 * 256 - 2^J per side, extended symmetrically as described below (SCAT_ERR_SHAPE beyond).
 * Oversampling o: only the output grid changes, the samples 2^max(J-o,0) n.  scat_backward
 * works on every 3-D plan.
 *
 * On success *out_plan is a new plan the caller must release with scat_plan_destroy.
 * On failure *out_plan is NULL and nothing is leaked.
 */
scat_status scat_plan_create(scat_plan **out_plan, int dims, const int *shape, int J, int LQ,
                             int max_order);

/*
 * Same as scat_plan_create but touches no GPU: the plan holds the host copies of the
 * tables only (for inspection with the scat_plan_* getters below); scat_forward on such a
 * plan returns SCAT_ERR_DEVICE.
 */
scat_status scat_plan_create_host(scat_plan **out_plan, int dims, const int *shape, int J,
                                  int LQ, int max_order);

/*
 * Plans for signals of ANY size (each side >= 1).  The paper's usage example (section 4,
 * "Interface") applies the transform to a 28 x 28 array without saying how the boundary is
 * handled; the reading taken here: every signal is extended symmetrically to the periodic
 * grid whose sides are the smallest powers of two >= side + 2^J (the margin's first half
 * mirrors the far edge, x[n-1], x[n-2], ..., the second half leads up to the near edge of
 * the next period, ..., x[1], x[0]; reflections repeat with period 2n), the periodic
 * transform runs on that grid, and the output keeps the samples 2^J k that lie inside the
 * signal: side ceil(n / 2^J).  scat_forward then takes inputs of `shape` and writes outputs
 * of scat_plan_out_shape; scat_plan_grid_shape tells the periodic grid; scat_plan_filter
 * refers to that grid.  scat_backward works on these plans too: it applies the
 * adjoints of the crop (zero extension) and of the symmetric extension (every sample
 * collects the gradients of its mirror images) around the periodic backward pass.
 * SCAT_ERR_SHAPE if the periodic grid exceeds what scat_plan_create accepts.
 */
scat_status scat_plan_create_padded(scat_plan **out_plan, int dims, const int *shape, int J,
                                    int LQ, int max_order);
scat_status scat_plan_create_padded_host(scat_plan **out_plan, int dims, const int *shape, int J,
                                         int LQ, int max_order);

/*
 * General form of plan creation.  `oversampling` = o >= 0 keeps every signal 2^o times finer
 * than the default schedule (the paper, section 2 "Implementation", only says that
 * intermediate signals are downsampled; o is the knob for how much): after a wavelet of
 * octave j the grid is subsampled by 2^max(j-o, 0) and the output by 2^max(J-o, 0), so the
 * output has sides shape >> max(J-o, 0).  With o >= J nothing is subsampled and the output,
 * read at the samples 2^J k, is the section-2 definition itself.  flags: bitwise OR of
 * SCAT_PLAN_PADDED (signals of any size, see scat_plan_create_padded),
 * SCAT_PLAN_HOST_ONLY (no GPU, see scat_plan_create_host), SCAT_PLAN_NODE_KERNELS and
 * SCAT_PLAN_PASS_KERNELS (below).  scat_backward limits the size of
 * the output grid in 2-D (see there), which limits o.
 */
#define SCAT_PLAN_PADDED 1
#define SCAT_PLAN_HOST_ONLY 2
/* 2-D plans of 256 x 256 at J = 3 or 128 x 128 at J = 2 (without oversampling): scat_forward
 * walks the tree with one workgroup per node (the "Implementation" paragraph's depth-first
 * walk: a node's inverse transform, modulus, lowpass and, for parents, spectrum never leave
 * the compute unit; only the spectra of the input and of first-order moduli with children are
 * kept in scratch).  This is what these plans do by default; SCAT_PLAN_NODE_KERNELS is kept
 * for callers that ask for it by name and changes nothing.  SCAT_PLAN_PASS_KERNELS selects
 * the row and column passes over the whole batch instead (the schedule of every other 2-D
 * shape), for comparison: same results to rounding.  Both are ignored by other shapes and by
 * scat_backward. */
#define SCAT_PLAN_NODE_KERNELS 4
#define SCAT_PLAN_PASS_KERNELS 8
scat_status scat_plan_create_ex(scat_plan **out_plan, int dims, const int *shape, int J, int LQ,
                                int max_order, int oversampling, int flags);

/* Writes the `dims` side lengths of the periodic grid the plan transforms on (equal to
 * `shape` for plans made by scat_plan_create). */
scat_status scat_plan_grid_shape(const scat_plan *plan, int *shape_out);

/*
 * Enqueue the transform of `batch` planes on `stream` (a hipStream_t passed as void*,
 * NULL = the default stream).  Does not synchronise.
 *
 *   in   device, float32, batch x shape[0] (x shape[1] (x shape[2])), C-contiguous.  Read only.
 *   out  device, float32, batch x K x (shape[0]>>J) (x (shape[1]>>J) ...), C-contiguous, where
 *        K = scat_plan_num_coeffs: channel 0 is S0, then S1 in order (j1, theta1) [1-D: by
 *        first-order wavelet index], then S2 in order (j1, theta1, j2, theta2) [1-D: (k1, j2)];
 *        3-D: S0, then S1 by (j, l), then S2 by (j1, l, j2).
 *
 * Image channels are the caller's business: a (B, C, H, W) tensor is batch = B*C planes.
 * `in` and `out` must not overlap and must stay valid until the stream has run the work.
 * The plan owns a scratch buffer that is (re)allocated when a call needs a larger one, so
 * at most one scat_forward per plan may be in flight at a time, and a call that grows
 * the buffer synchronises the device first.  batch == 0 is a no-op.
 */
scat_status scat_forward(scat_plan *plan, const float *in, float *out, long batch,
                         void *stream);

/*
 * Grow the plan's scratch buffer now to what scat_forward (and, with with_backward != 0,
 * scat_backward) needs for calls of up to `batch` planes, so that those calls neither
 * allocate nor synchronise (paper, section 2 "Implementation": the transform is meant to sit
 * inside a training or serving loop).  Synchronises the device if the buffer has to grow;
 * must run on the plan's device with no call of this plan in flight.  The buffer never
 * shrinks.  Errors: SCAT_ERR_NULL, SCAT_ERR_ARG (batch < 1), SCAT_ERR_DEVICE (host-only plan
 * or wrong device), SCAT_ERR_ALLOC.
 */
scat_status scat_plan_reserve(scat_plan *plan, long batch, int with_backward);

/*
 * scat_forward for callers that cannot allocate device memory (code under HIP graph capture,
 * serving loops and harnesses that forbid hipMalloc): same arguments, same result, but the
 * intermediate arrays live in a buffer of SCAT_STATIC_SCRATCH_MB MiB that is part of the
 * library's device image (each GPU the library runs on holds one copy until the process
 * ends) instead of the plan's own scratch.  The call allocates and frees nothing and records
 * no kernel timing (scat_plan_timing_* is ignored for it).  A batch whose intermediates exceed
 * the buffer is run in consecutive chunks on `stream`.
 * Errors: as scat_forward, and SCAT_ERR_WORKSPACE if a single plane of this plan needs more
 * than the buffer (scat_plan_workspace_bytes(plan, 1) > SCAT_STATIC_SCRATCH_MB MiB); then
 * nothing is enqueued.
 * Every call on a GPU shares that GPU's buffer, whatever the plan or stream: calls whose work
 * overlaps in time on one GPU race; the caller orders them (one stream, or events).  The
 * buffer keeps the last call's contents between calls; the schedules write every element
 * before reading it, so nothing needs clearing.
 */
#define SCAT_STATIC_SCRATCH_MB 64
scat_status scat_forward_static(scat_plan *plan, const float *in, float *out, long batch,
                                void *stream);

/*
 * Backward pass: the gradient of  sum(grad_out * S(in))  with respect to `in`,
 * i.e. the transposed Jacobian of scat_forward applied to grad_out.  The paper lists
 * differentiability as a feature of its package (section 3, "Relation to previous
 * software") without formulas; the cascade is a chain of real-linear maps and complex
 * moduli, and this call applies the adjoints in reverse order, with d|y| = Re(conj(y) dy)/|y|
 * and the convention that the modulus passes no gradient where y = 0.
 *
 *   in        device, float32, batch x shape, as given to scat_forward.  Read only.
 *   grad_out  device, float32, batch x K x out_shape (the layout of scat_forward's `out`).
 *             Read only.
 *   grad_in   device, float32, batch x shape.  Overwritten with the gradient.
 *
 * The forward cascade is recomputed inside the call (its outputs S are not formed) and the
 * complex signals before every modulus are kept in the plan's scratch buffer until the
 * call's work has run; the same one-call-in-flight rule as scat_forward applies, and the
 * two share the scratch buffer.  Enqueues on `stream`, does not synchronise.
 * 3-D plans: rho = sqrt(sum_m |y_m|^2) passes g y_m / rho to y_m (nothing where rho = 0); the
 * degree-0 signal y is real, so there the factor is sign(y), decided by rounding where |y| is
 * below fp32 resolution.
 * Errors: SCAT_ERR_ARG for batch < 0.  SCAT_ERR_SHAPE, 2-D: unless every
 * side and every side subsampled for the last octave lies in 4...512 and the output grid
 * has at most 1024 points or is one of 16 x 16 ... 128 x 128, square or 2 : 1 (the latter
 * only if the rows keep at least 4 points at every octave); 1-D: unless the signal, seen as the n1 x n2 matrix of the
 * four-step transform (n2 = 2^max(ceil(log2(n)/2), J), n1 = n / n2), has n1 in 4...512 and
 * n2 <= 512 (so n <= 2^18 at most).
 */
scat_status scat_backward(scat_plan *plan, const float *in, const float *grad_out,
                          float *grad_in, long batch, void *stream);

/* Bytes of device scratch a scat_backward call with this batch size uses (0 if unsupported). */
size_t scat_plan_backward_workspace_bytes(const scat_plan *plan, long batch);

/* Release a plan and its device memory.  NULL is a no-op returning SCAT_OK. */
scat_status scat_plan_destroy(scat_plan *plan);

/* ---- introspection: host only, never touches the GPU ------------------------------ */

/* Number of output channels K (1 + J*L + L^2 J(J-1)/2 in 2-D at max_order 2); -1 on NULL. */
int scat_plan_num_coeffs(const scat_plan *plan);

/* Writes the `dims` output side lengths: shape >> max(J - oversampling, 0), rounded up for
 * padded plans. */
scat_status scat_plan_out_shape(const scat_plan *plan, int *shape_out);

/* Row c of the index table: idx = {order, j1, t1, j2, t2}, unused fields -1.
 * 2-D: t = angle index.  1-D: t1 = first-order wavelet index k (octave j1 = k / Q),
 * t2 = second-order wavelet index (= j2).  3-D: t1 = degree l, t2 unused. */
scat_status scat_plan_coeff_index(const scat_plan *plan, int c, int idx[5]);

/* Bytes of device scratch a scat_forward call with this batch size uses. */
size_t scat_plan_workspace_bytes(const scat_plan *plan, long batch);

/*
 * Copy one filter's Fourier samples, as the kernels read them but WITHOUT the
 * normalisation pre-scale, into host memory as float64, natural frequency order
 * (2-D: rows x cols of the grid at resolution `res`, i.e. shape >> res; 1-D: length
 * shape[0] >> res).
 *   kind 0: lowpass phi_J folded to resolution res        (index ignored)
 *   kind 1: first-order wavelet `index` (2-D: j*L + theta; 1-D: k), res must be 0
 *   kind 2: second-order wavelet `index` (2-D: j*L + theta; 1-D: j) folded to res < j
 * 3-D plans (res must be 0): kind 0 index 0 is the lowpass (shape[0] x shape[1] x shape[2]);
 * kind 1 with index j*(L+1) + l gives the 2l+1 real tables of that scale and degree,
 * (2l+1) x shape: r^l e^(-r^2/2) times the real orthonormal harmonics of degree l at
 * w = 2^j (omega + 2 pi a), r = |w|, summed over the aliases a (the factor (-i)^l of the
 * Fourier transform has modulus 1 and is dropped).
 * Returns SCAT_ERR_ARG if that table is not part of the plan.
 */
scat_status scat_plan_filter(const scat_plan *plan, int kind, int index, int res,
                             double *out_host);

/* ---- per-kernel timing, for benchmarks ---------------------------------------------- */

/*
 * From now on scat_forward brackets kernel launches with HIP events on the stream it is
 * given: every launch if kernel_name is NULL, else only launches of the kernel with that
 * name (as a profiler prints it without namespaces and arguments, e.g.
 * "k_rows_fused<256>").  Discards earlier records.  Costs two event records per timed
 * launch; leave it off otherwise.
 */
scat_status scat_plan_timing_begin(scat_plan *plan, const char *kernel_name);

/* Stops recording, waits for the recorded launches and sums them per kernel name.
 * Returns the number of distinct kernels recorded, or -1 on error / if not recording. */
int scat_plan_timing_end(scat_plan *plan);

/*
 * Row `row` of the last scat_plan_timing_end: kernel name (copied, NUL-terminated, into
 * name[name_len]), number of launches, their summed duration in milliseconds, the bytes
 * those launches had to move at the least (each input and filter table read once, each
 * output written once) and their model flops (5 n log2 n per n-point transform plus
 * 4 per filter multiply-accumulate and modulus).  Any out pointer may be NULL.
 */
scat_status scat_plan_timing_row(const scat_plan *plan, int row, char *name, size_t name_len,
                                 long *launches, double *ms, double *alg_bytes,
                                 double *model_flops);

const char *scat_status_string(scat_status s);

#ifdef __cplusplus
}
#endif
#endif /* SCAT_H */
