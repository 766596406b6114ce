/*
 * dft3d -- 3-D complex DFT on a tensor-product grid as mode-wise dense contractions,
 *          for one AMD MI355X (gfx950).  C ABI; no C++ or torch types cross this boundary.
 *
 * Two formulations of the same transform (paper, Section III):
 *   KDFT  every tensor mode is contracted with an N x N Vandermonde matrix (Eq. 10 / Eq. 11);
 *         a nonuniform axis only changes the matrix.
 *   FFT   per axis a split N = A*B (Eq. 13 with P = B): an A-point transform over the slow
 *         sub-index (Eq. 16), a twiddle factor, a B-point transform over the fast sub-index
 *         (the "phase adjustment" of Eq. 15 factored into a diagonal and a matrix product),
 *         and a re-ordering so the result is in natural order.
 *
 * Data layout.  Tensors are nx x ny x nz, C order (z fastest), complex64 stored as interleaved
 * (re, im) floats -- the memory of a contiguous numpy/torch complex64 array.  `in`, `out` and
 * the workspace are DEVICE pointers owned by the caller, 16-byte aligned, non-overlapping.
 * Coordinate arrays are HOST pointers, copied during plan creation.
 *
 * Conventions.  FORWARD uses exp(-2 pi i ...) and is unscaled (Eq. 1, Eq. 12).  BACKWARD uses
 * exp(+2 pi i ...) and multiplies by 1/(nx ny nz), so BACKWARD(FORWARD(x)) = x on uniform axes;
 * it is not offered for nonuniform axes (there the inverse is a linear solve, Section III-A).
 * A nonuniform axis has matrix entries M[k, n] = exp(-2 pi i k c[n]), k = 0..N-1, with c[n] the
 * sample coordinate in cycles (period 1).
 *
 * Errors.  Every call returns a status; nothing throws or aborts across the boundary.
 * dft3d_last_error() returns a thread-local, human-readable message for the last failure.
 * Execution calls only enqueue work on the given HIP stream and never synchronise; calls that
 * use one plan must be ordered on a stream because they share the plan's workspace.
 */
#ifndef DFT3D_H
#define DFT3D_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dft3d_plan_s* dft3d_plan;

typedef enum {
    DFT3D_OK = 0,
    DFT3D_ERR_INVALID_ARG = 1,
    DFT3D_ERR_UNSUPPORTED = 2,
    DFT3D_ERR_ALLOC = 3,
    DFT3D_ERR_HIP = 4
} dft3d_status;

typedef enum { DFT3D_KDFT = 0, DFT3D_FFT = 1 } dft3d_formulation;

/* value = sign of the exponent */
typedef enum { DFT3D_FORWARD = -1, DFT3D_BACKWARD = 1 } dft3d_direction;

/* plan flags */
#define DFT3D_FLAG_CLOBBER_INPUT 1u /* exec may overwrite `in`; then no workspace is needed */
#define DFT3D_FLAG_UNFUSED 2u       /* FFT: run the twiddle and the re-ordering as separate
                                       kernels instead of fusing them into the contractions */
#define DFT3D_FLAG_BF16X3 8u        /* KDFT: float32 accuracy on the bf16 matrix cores -- every fp32
                                       number is decomposed into three bf16 numbers and six cross
                                       products are accumulated in fp32 (Section II-A of the paper),
                                       with three real products per complex product;
                                       used for modes whose shape is a whole number of 128x128 tiles,
                                       other modes fall back to the fp32 kernels (which take three
                                       real products only with DFT3D_FLAG_3M) */
#define DFT3D_FLAG_COMPLEX128 16u   /* tensors are complex128 (interleaved doubles), matrices and twiddles are
                                       kept in fp64 and the contractions run on the fp64 matrix cores (the
                                       float64 precision the paper leaves as future work, Section VI).
                                       Every byte count below doubles (16 bytes per element).  KDFT plans,
                                       and FFT plans as staged passes (first stage with the twiddle in its
                                       epilogue, second stage, re-ordering: no fused axis kernels, no
                                       dft3d_fft_phase / dft3d_fft_axis), and point plans.  Not combined with
                                       3M / BF16X3 / UNFUSED */
#define DFT3D_FLAG_ADJOINT 32u      /* KDFT: the plan applies the conjugate transpose of the transform its
                                       other arguments describe, out = (M_x (x) M_y (x) M_z)^H in: from
                                       integer frequencies back to the (nonuniform) samples, the operation
                                       an iterative solve of the inverse problem of Section III-A needs
                                       next to the forward one.  Shapes are unchanged for
                                       dft3d_plan_create(_ex); a dft3d_plan_create_points plan then takes
                                       a kx x ky x kz tensor and returns an nx x ny x nz one.  On uniform
                                       axes it equals BACKWARD without the 1/N factor */
#define DFT3D_FLAG_3M 4u            /* KDFT: three real products per complex product
                                       (Vr*Xr, Vi*Xi, (Vr+Vi)*(Xr+Xi)) instead of four: 25 % fewer
                                       MFMA operations, slightly larger rounding error in Im */

/*
 * Plan creation (Eq. 3 / Eq. 12 matrices, Eq. 13 split).  Generates the per-axis matrices
 * (and, for FFT, the stage matrices and twiddle tables) in fp64 on the host, rounds them once
 * to fp32 and uploads them; this call allocates device memory and synchronises.
 *   plan      receives the handle, or NULL on failure
 *   nx,ny,nz  axis lengths, each >= 1
 *   f         DFT3D_KDFT or DFT3D_FFT
 *   cx,cy,cz  NULL for a uniform axis, else HOST array of n? doubles (sample coordinates in
 *             cycles).  FFT requires all three NULL (Section III-B: uniform sampling).
 * dft3d_plan_create_ex additionally takes
 *   split     NULL, or three first-stage lengths A (0 = choose); A must divide the axis length.
 *             Default: A = 2^floor(log2(N)/2) for powers of two, else the divisor pair closest
 *             to sqrt(N) with A <= B (512 -> 16*32), except 1024 -> 16*64, 2048 -> 16*128 and, on
 *             complex64 plans without DFT3D_FLAG_UNFUSED, 4096 -> 4*1024, 8192 -> 4*2048,
 *             16384 -> 8*2048 (see dft3d_fft_first_stage; a strided axis only when the extent inside
 *             it is a multiple of 16, the z axis at 4096 points only when the axis transformed next
 *             takes such a split too: otherwise 64*64, 64*128, 128*128).
 *   flags     DFT3D_FLAG_* bits
 * Errors: INVALID_ARG (NULL plan pointer, size < 1 or > 2^24, bad split, unknown formulation or flag,
 * a coordinate that is not finite),
 * UNSUPPORTED (FFT with coordinates, ADJOINT / 3M / BF16X3 on an FFT plan, COMPLEX128 together with
 * 3M / BF16X3 / UNFUSED, ny*nz or nx*ny of 2^31 or more: the kernels index the extents inside and
 * outside an axis with 32 bits),
 * ALLOC / HIP (device allocation or copy failed).
 */
dft3d_status dft3d_plan_create(dft3d_plan* plan, int64_t nx, int64_t ny, int64_t nz,
                               dft3d_formulation f, const double* cx, const double* cy,
                               const double* cz);
dft3d_status dft3d_plan_create_ex(dft3d_plan* plan, int64_t nx, int64_t ny, int64_t nz,
                                  dft3d_formulation f, const double* cx, const double* cy,
                                  const double* cz, const int64_t* split, uint32_t flags);

/*
 * Plan for the general form of Eq. 1 - Eq. 3: arbitrary evaluation points on the z-plane.
 * Axis j of the output has k_j entries, X(z_j0..z_j,k-1), with the K x N Vandermonde matrix
 * V_j[r, n] = z_jr^{-n} (Eq. 3); the transform is V_x (x) V_y (x) V_z applied to the nx x ny x nz
 * input (Eq. 11), giving a kx x ky x kz output.  KDFT only, FORWARD only (the inverse is a
 * linear solve, Section III-A).
 *   zx,zy,zz  HOST arrays of 2*k? doubles, (re, im) of each point; points must be non-zero.  NULL =
 *             that axis uses the N-th roots of unity (then k? must equal n?).
 *   flags     DFT3D_FLAG_3M and / or DFT3D_FLAG_ADJOINT (then the roles of n? and k? swap: input
 *             kx x ky x kz, output nx x ny x nz, matrices V_j^H), DFT3D_FLAG_COMPLEX128 (complex128
 *             tensors, the Vandermonde matrices kept in fp64; not together with 3M), or 0
 * exec needs a workspace of dft3d_plan_workspace_bytes = 8*(nx*ny*kz + nx*ky*kz) bytes (the two
 * intermediates; ADJOINT: 8*(kx*ky*nz + kx*ny*nz)).  dft3d_mode_contract on such a plan reads a tensor whose axes after `axis`
 * already have their output length and writes one whose `axis` has length k (order z, y, x).
 * Errors: INVALID_ARG (sizes, a zero / non-finite point, an entry that overflows fp32), UNSUPPORTED
 * (ky*kz or nx*ny of 2^31 or more; with ADJOINT also ny*nz and kx*ky).
 */
dft3d_status dft3d_plan_create_points(dft3d_plan* plan, int64_t nx, int64_t ny, int64_t nz,
                                      int64_t kx, int64_t ky, int64_t kz, const double* zx,
                                      const double* zy, const double* zz, uint32_t flags);

/* Output lengths of a plan (equal to the input lengths except for evaluation-point plans). */
dft3d_status dft3d_plan_get_output_shape(dft3d_plan plan, int64_t* kx, int64_t* ky, int64_t* kz);

/* Frees the plan and the device memory it owns (not the workspace).  NULL is accepted. */
dft3d_status dft3d_plan_destroy(dft3d_plan plan);

/* Bytes of caller-provided device workspace dft3d_exec needs: 0 with CLOBBER_INPUT and for KDFT
 * plans on complex64 tensors whose axes (input and output) are all at most 32 long -- those run
 * all three modes in one launch of plain fp32 vector arithmetic, whatever arithmetic flags the
 * plan carries (at that size the transform is launch latency: Eq. 10 on 32^3 is 2.5e7 flop) -- else the
 * size of one tensor (8 * nx*ny*nz; 16 * nx*ny*nz for a COMPLEX128 plan) or, for FFT plans that
 * keep their intermediate with a padded row pitch, 8 * nx*ny*(nz+16).  Always query; the step
 * calls below need none. */
size_t dft3d_plan_workspace_bytes(dft3d_plan plan);

/* Hands the plan a DEVICE buffer of at least dft3d_plan_workspace_bytes bytes.  The caller
 * keeps ownership and must keep it alive while exec calls are in flight. */
dft3d_status dft3d_plan_set_workspace(dft3d_plan plan, void* dev, size_t bytes);

/* Which kernel family contracts mode `axis` (0, 1 or 2) of a KDFT plan in dft3d_exec and
 * dft3d_mode_contract (Eq. 11, one mode product): writes a NUL-terminated name such as
 * "k_contract_s", "k_contract_c (3M)", "k_contract_bf16x3", "k_contract_sr", "k_contract_f64" or
 * "k_kdft_small" (the single launch that runs all three modes) into name[len].  Lets a caller see
 * whether a flag such as DFT3D_FLAG_BF16X3 takes effect for a shape.  Host only, launches nothing.
 * On an FFT plan the name says how dft3d_exec transforms the axis (Eq. 13 - 16): "fused" (one pass),
 * "butterflies + fused second stage" (first factor 2, 4 or 8: two passes), "butterflies + second stage",
 * "first stage + second stage" (matrix stages: two passes), "first stage, twiddle pass, second stage"
 * (DFT3D_FLAG_UNFUSED) or "identity" (length 1); a z axis that is not "fused" also needs its re-ordering, a pass
 * of its own unless the pass after it is a butterfly pass and reads through it. */
dft3d_status dft3d_plan_mode_kernel(dft3d_plan plan, int axis, char* name, size_t len);

/* First-stage / second-stage lengths chosen for an axis (0, 1 or 2) of an FFT plan. */
dft3d_status dft3d_plan_get_split(dft3d_plan plan, int axis, int64_t* A, int64_t* B);

/* Order in which dft3d_exec transforms the axes (Eq. 10: the three modes commute): order[0..2] receives
 * the axis of the first, second and third mode.  2, 1, 0 (z, y, x) for every plan except FFT plans that
 * run the x pass first (all three axes on fused kernels, 2048 points or more along x, a workspace: 0, 1, 2).
 * The single-pass entry points below are not affected.  Host only.  INVALID_ARG for NULL arguments. */
dft3d_status dft3d_plan_axis_order(dft3d_plan plan, int order[3]);

/*
 * The whole transform (Eq. 10): out = transform(in).  Out of place: in != out, and neither may
 * overlap the workspace.  `in` is left intact unless the plan has CLOBBER_INPUT.
 * direction: DFT3D_FORWARD or DFT3D_BACKWARD.  stream: a hipStream_t passed as void* (NULL =
 * the null stream).  Errors: INVALID_ARG (NULL / misaligned / aliased pointers, bad direction,
 * workspace missing or too small), UNSUPPORTED (BACKWARD on a nonuniform plan), HIP (launch).
 * The call only launches kernels on `stream` (no allocation, copy, memset or synchronisation), so
 * with per-pass timing off it may be captured into a HIP graph; replaying the graph is what pays
 * for small tensors, where launch latency exceeds kernel time.
 */
dft3d_status dft3d_exec(dft3d_plan plan, const void* in, void* out, int direction,
                        void* stream);

/*
 * dft3d_exec for callers that cannot allocate device memory or hand over a workspace: code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels and bit-identical results; the intermediate tensor that dft3d_exec keeps in the
 * caller's workspace lives in a static device array of DFT3D_NOALLOC_MAX_BYTES inside the library
 * (one per GPU, held from the first plan created on that GPU until the process ends), and any
 * workspace set on the plan is ignored.  The call allocates and frees nothing; the array's address
 * is looked up once per GPU, during plan creation.
 * Errors: as dft3d_exec, and UNSUPPORTED when dft3d_plan_workspace_bytes(plan) exceeds
 * DFT3D_NOALLOC_MAX_BYTES (one complex64 tensor of 128 x 128 x 256, say).
 * Every pass overwrites the part of the array it uses before reading it, so nothing needs clearing
 * between calls; but all calls on one GPU share the one array: two calls whose kernels may overlap
 * in time (different streams, different plans, different threads) race.  Order them on one stream.
 */
#define DFT3D_NOALLOC_MAX_BYTES (32u << 20)
dft3d_status dft3d_exec_noalloc(dft3d_plan plan, const void* in, void* out, int direction,
                                void* stream);

/*
 * Per-pass timing of dft3d_exec (measurement aid; the analogue of the per-operation breakdown
 * the paper reads from its profiler in Section V).  After enable_profiling(plan, max_execs)
 * the next max_execs calls of dft3d_exec record a HIP event before and after every kernel on
 * the exec stream (no synchronisation is added).  read_profile, called after the caller has
 * synchronised the stream, returns the milliseconds of each pass of exec number exec_index
 * (0-based since enabling): ms must hold DFT3D_MAX_PASSES floats, *npass receives the count.
 * enable_profiling(plan, 0) switches it off and frees the events.
 */
#define DFT3D_MAX_PASSES 16
dft3d_status dft3d_plan_enable_profiling(dft3d_plan plan, int max_execs);
dft3d_status dft3d_plan_read_profile(dft3d_plan plan, int exec_index, float* ms, int* npass);

/* ---- single steps of the path; each is one kernel launch, out of place, same layout ------- */

/* KDFT, one mode product (Eq. 2 along `axis` of the tensor; steps of Eq. 11):
 *   out[.., k, ..] = sum_n M_axis[k, n] in[.., n, ..].   axis = 0, 1 or 2.
 * BACKWARD conjugates the matrix and scales by 1/N_axis.  Valid on KDFT plans. */
dft3d_status dft3d_mode_contract(dft3d_plan plan, int axis, const void* in, void* out,
                                 int direction, void* stream);

/* FFT, first stage on `axis` (Eq. 16, then the twiddle if fuse_twiddle != 0):
 *   out[k_a*B + beta] = T * sum_l exp(-+2 pi i k_a l / A) in[B*l + beta],
 *   T = exp(-+2 pi i beta k_a / N) if fuse_twiddle else 1.  Valid on FFT plans.
 * A first factor of 2, 4 or 8 is evaluated as butterflies in vector arithmetic (an element-wise,
 * memory-bound pass) on complex64 plans without DFT3D_FLAG_UNFUSED; every other one as a contraction
 * with the A x A matrix on the matrix cores. */
dft3d_status dft3d_fft_first_stage(dft3d_plan plan, int axis, const void* in, void* out,
                                   int direction, int fuse_twiddle, void* stream);

/* FFT, the twiddle alone (the diagonal part of Eq. 15's phase adjustment):
 *   out[k_a*B + beta] = exp(-+2 pi i beta k_a / N) in[k_a*B + beta].  Memory-bound pass. */
dft3d_status dft3d_fft_phase(dft3d_plan plan, int axis, const void* in, void* out,
                             int direction, void* stream);

/* FFT, second stage on `axis` (the matrix part of Eq. 15's phase adjustment):
 *   W[k_a, k_b] = sum_beta exp(-+2 pi i k_b beta / B) in[k_a*B + beta]
 * stored at slot k_a*B + k_b, or, if reorder != 0, in natural order at k_a + A*k_b.
 * BACKWARD also scales by 1/N_axis.
 * With A = 2, 4 or 8 and B = 512, 1024 or 2048 (complex64, no DFT3D_FLAG_UNFUSED; x and y: extent inside
 * the axis a multiple of 16; z: reorder = 0) the B-point sums are evaluated by the fused kernel of
 * dft3d_fft_axis for B = 16 x (B/16), i.e. Eq. 13 - 16 applied to the second stage once more; otherwise as a
 * contraction with the B x B matrix.  dft3d_exec runs such an axis in two passes, and where the z axis and
 * the axis transformed after it both have such a split, the first stage of the second one reads its input
 * through the z re-ordering, which then takes no pass of its own. */
dft3d_status dft3d_fft_second_stage(dft3d_plan plan, int axis, const void* in, void* out,
                                    int direction, int reorder, void* stream);

/* FFT, one whole axis in a single fused kernel: first stage, twiddle, second stage and natural
 * order (Eq. 13 - Eq. 16 for that axis), one read and one write of the tensor.  Offered for
 * axis 2 (z) with splits 16x16, 16x32, 16x64, 16x128, 32x32, 32x64, 64x64 and for axes 0, 1 (x, y)
 * with splits 16x16, 16x32, 16x64, 16x128, 32x32, 32x64 when the extent inside the axis is a multiple
 * of 16; UNSUPPORTED otherwise.  For A x (C*16) with A = 16 or 32 the kernels evaluate the second stage of
 * Eq. 16 with its own factor split once more (C-point butterflies and a 16-point matrix stage): the same
 * sums in another order of evaluation.  dft3d_exec uses the fused kernel whenever it applies (unless the plan has
 * DFT3D_FLAG_UNFUSED).  The default split of 1024 and 2048 points is 16 x 64 and 16 x 128. */
dft3d_status dft3d_fft_axis(dft3d_plan plan, int axis, const void* in, void* out, int direction,
                            void* stream);

/* FFT, the re-ordering alone (Section IV, in-order transform): for every axis whose bit is set
 * in axes_mask (bit 0 = x, 1 = y, 2 = z), out[k_a + A*k_b] = in[k_a*B + k_b].  Pure data
 * movement through LDS; memory-bound pass. */
dft3d_status dft3d_fft_reorder(dft3d_plan plan, int axes_mask, const void* in, void* out,
                               void* stream);

/* Plain device-to-device copy of `bytes` (multiple of 16) with the library's own copy kernel:
 * the achievable-HBM-bandwidth reference for the memory-bound passes and the calibration
 * kernel for hardware byte counters (its traffic is exactly 2*bytes).  variant selects the
 * launch shape (0 = default; +100 = loads and stores with the streaming hint the memory-bound
 * passes use).  in/out: DEVICE, 16-byte aligned, non-overlapping. */
dft3d_status dft3d_device_copy(const void* in, void* out, size_t bytes, int variant, void* stream);

/* ---- host-side generator, exposed so its rounding can be tested without a GPU -------------- */

/* Writes the n x n transform matrix of one axis as the library rounds it (fp64 evaluation with
 * exact argument reduction, one rounding to fp32): re[k*n + j], im[k*n + j] = M[k, j].
 * coords: NULL (uniform) or HOST array of n doubles.  HOST output arrays of n*n floats. */
dft3d_status dft3d_generate_matrix(int64_t n, const double* coords, int direction, float* re,
                                   float* im);

/* Writes the k x n Vandermonde matrix V[r*n + j] = z_r^{-j} (Eq. 3) for k points given as HOST
 * (re, im) pairs, as the library rounds it, to HOST arrays of k*n floats. */
dft3d_status dft3d_generate_points_matrix(int64_t k, int64_t n, const double* z, float* re, float* im);

/* Writes the A x B twiddle table T[k_a*B + beta] = exp(-+2 pi i beta k_a / (A*B)) to HOST arrays. */
dft3d_status dft3d_generate_twiddle(int64_t A, int64_t B, int direction, float* re, float* im);

const char* dft3d_status_string(dft3d_status s);
const char* dft3d_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DFT3D_H */
