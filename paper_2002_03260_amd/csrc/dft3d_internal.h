// Internal declarations shared by the host side (plan, generator) and the HIP kernels of the
// dft3d library.  Not part of the public boundary (include/dft3d.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "dft3d.h"

namespace dft3d {

// ---- device matrices --------------------------------------------------------------------
// A K x N complex matrix M is kept on the device as two fp32 planes stored TRANSPOSED,
// plane[n * ld + k] = Re/Im M[k, n], zero-padded to `rows` x `ld` with ld a multiple of
// kPlaneLdAlign and rows a multiple of kPlaneRowAlign, so kernels stage tiles of it without
// bounds checks.  (Lanes of an MFMA operand walk k at fixed n: unit stride in this layout.)
constexpr int kPlaneLdAlign = 128;
constexpr int kPlaneRowAlign = 64;

struct DeviceMatrix {
    float* re = nullptr;
    float* im = nullptr;
    int K = 0;     // output length (rows of M)
    int N = 0;     // contracted length (columns of M)
    int ld = 0;    // padded K
    int rows = 0;  // padded N
    // Optional bf16 decomposition of the same matrix for the bf16-split contraction: nine planes
    // (Re, Im, Re + Im) x (hi, mid, lo), zero padded to split_rows x split_ld, stored tile by tile as
    // [k tile of 128][chunk of 16 n][plane][128 k][16 n] (n contiguous: a bf16 MFMA operand lane
    // holds 8 consecutive n; the piece one kernel iteration needs is contiguous).
    unsigned short* split = nullptr;
    int split_ld = 0;     // padded N (multiple of 16)
    int split_rows = 0;   // padded K (multiple of 128)
    int split_planes = 0; // 9: three levels each of Re, Im and Re + Im (three-product scheme)
    // Optional fp64 copy for complex128 plans: planes re, im (rows64 * ld64 doubles apart), transposed
    // like the fp32 planes, plane[n * ld64 + k].
    double* f64 = nullptr;
    int ld64 = 0;         // padded K (multiple of 64)
    int rows64 = 0;       // padded N (multiple of 16)
};

// ---- one mode contraction ---------------------------------------------------------------
// in  viewed as [O][N][I] (contiguous),  out element (o, k, i) at
//   (o / Olo) * sYohi + (o % Olo) * sYolo + k * sYk + i
// out = scale * tw * sum_n M[k, n] in[o, n, i], with M conjugated if conj != 0 and
// tw = Tw[k * twB + i / twInner] if Tw != nullptr else 1.
struct ContractArgs {
    const float2* X;
    float2* Y;
    DeviceMatrix M;
    int64_t O;
    int64_t I;
    int64_t Olo, sYohi, sYolo, sYk;
    const float2* Tw;
    int twB;
    int64_t twInner;
    float scale;
    int conj;
    int three_m;   // use the three-real-product complex scheme where a kernel for it exists
    int bf16x3;    // use the bf16-split kernel (M.split must be set) where the shape allows
};

hipError_t launch_contract(const ContractArgs& a, hipStream_t stream);
// The kernel family launch_contract picks for these arguments (nothing is launched).
const char* contract_kernel_name(const ContractArgs& a);

// Streaming variant for strided modes with a small square matrix (16, 32 or 64) and an inner
// extent that is a multiple of 16: one wavefront per 16-column tile, no staging of the data in LDS.
bool contract_sr_supported(const ContractArgs& a);
hipError_t launch_contract_sr(const ContractArgs& a, hipStream_t stream);

// bf16-split variant (three bf16 levels per fp32 number, six cross products on bf16 MFMA, three
// real products per complex product); only whole 128 x 128 tiles, no fused twiddle.
bool contract_bf16x3_supported(const ContractArgs& a);
hipError_t launch_contract_bf16x3(const ContractArgs& a, hipStream_t stream);

// ---- double-precision mode contraction (complex128 tensors) ----------------------------------
// Same operation and output addressing as ContractArgs, on interleaved (re, im) doubles.  The
// matrix is two fp64 planes (re, then im, `rows * ld` doubles apart) stored transposed and zero
// padded like the fp32 planes: plane[n * ld + k], ld a multiple of 64, rows a multiple of 16.
struct ContractArgs64 {
    const void* X;
    void* Y;
    const double* M;
    int K, N, ld, rows;
    int64_t O;
    int64_t I;
    int64_t Olo, sYohi, sYolo, sYk;
    double scale;
    int conj;
    // optional twiddle fused into the epilogue: out *= Tw[k * twB + (i / twInner)] (conjugated when conj);
    // (re, im) pairs of doubles, NULL = none
    const double* Tw;
    int twB;
    int64_t twInner;
};
hipError_t launch_contract_f64(const ContractArgs64& a, hipStream_t stream);

// Sub-index swap of a complex128 tensor (same meaning as ReorderArgs, 16-byte elements).
hipError_t launch_reorder_c128(const void* in, void* out, const int n[3], const int A[3], const int B[3],
                               const int swap[3], hipStream_t stream);

// ---- twiddle (phase) multiply -------------------------------------------------------------
// Tensor viewed as [outer][A][B][inner]; out = in * Tw[k_a * B + beta] (conjugated if conj).
hipError_t launch_phase(const float2* in, float2* out, int64_t outer, int A, int B, int64_t inner,
                        const float2* Tw, int conj, hipStream_t stream);

// ---- sub-index swap (in-order re-ordering) ------------------------------------------------
// For each axis j with swap[j] != 0, the element at slot ka*B[j] + kb moves to ka + A[j]*kb.
struct ReorderArgs {
    const float2* in;
    float2* out;
    int n[3];
    int A[3];
    int B[3];
    int swap[3];
};
hipError_t launch_reorder(const ReorderArgs& a, hipStream_t stream);

// ---- fused contiguous-axis FFT-formulation pass ---------------------------------------------
// One launch = first stage + twiddle + second stage + in-order placement of the z axis of a
// tensor with `nrows` rows of A*B complex numbers.  Available for a fixed set of (A, B).
bool fft_z_supported(int A, int B);
hipError_t launch_fft_z(const float2* in, float2* out, int64_t nrows, int A, int B,
                        const DeviceMatrix& FA, const DeviceMatrix& FB, const float2* Tw, float scale,
                        int conj, hipStream_t stream);

// Register-resident variant of the same pass (one wavefront per row, no LDS); launch_fft_z uses it
// for the splits it covers.
bool fft_zr_supported(int A, int B);
hipError_t launch_fft_zr(const float2* in, float2* out, int64_t nrows, int A, int B,
                         const DeviceMatrix& FA, const DeviceMatrix& FB, const float2* Tw, float scale,
                         int conj, hipStream_t stream);

// The same pass with the second factor split once more (16 x (C*16): two 16-point matrix stages around
// C-point butterflies), one wavefront per row; launch_fft_z uses it for the splits it covers.
bool fft_zn_supported(int A, int B);
hipError_t launch_fft_zn(const float2* in, float2* out, int64_t nrows, int A, int B,
                         const DeviceMatrix& FA, const DeviceMatrix& FB, const float2* Tw, float scale,
                         int conj, hipStream_t stream);

// First stage (+ twiddle unless Tw is null) of a split whose first factor R is 2, 4 or 8, on the view
// [O][R][B][inner]: butterflies in vector arithmetic, one element-wise memory-bound pass.  With pA > 1 the
// rows of the innermost tensor axis (nz = pA * pB points, inner a multiple of nz) are read through that axis'
// re-ordering [k_a][k_b] -> k_a + pA * k_b, which then needs no pass of its own.
bool radix_stage_supported(int R, int64_t B, int64_t inner);
hipError_t launch_radix_twiddle(const float2* in, float2* out, int64_t O, int R, int64_t B, int64_t inner,
                                const float2* Tw, int conj, int64_t nz, int pA, int pB, hipStream_t stream);

// ---- fused strided-axis FFT-formulation pass ------------------------------------------------
// Tensor viewed as [O][A*B][I]; one launch = both stages, twiddle and natural order along the
// middle index.  I must be a multiple of 16; available for a fixed set of (A, B).
bool fft_s_supported(int A, int B, int64_t I);
hipError_t launch_fft_s(const float2* in, float2* out, int64_t O, int64_t I, int A, int B,
                        const DeviceMatrix& FA, const DeviceMatrix& FB, const float2* Tw, float scale,
                        int conj, hipStream_t stream);

// Variant of the strided-axis pass with the data as MFMA operands straight from global memory
// (only the intermediate of the two stages passes through LDS); launch_fft_s uses it for the
// splits it covers.
// General addressing of that kernel: the tensor is [O][N = A*B][Yn][16 * Zt] with separate element
// strides on the input and the output side (o: inO / outO, n: inN / outN, y: inY / outY; the last
// index is contiguous).  Lets an intermediate tensor carry a padded row pitch.
struct FftStridedArgs {
    const float2* X;
    float2* Y;
    int64_t O, Yn, Zt;
    int64_t inO, inN, inY;
    int64_t outO, outN, outY;
};
hipError_t launch_fft_sr_ex(const FftStridedArgs& a, int A, int B, const DeviceMatrix& FA,
                            const DeviceMatrix& FB, const float2* Tw, float scale, int conj, hipStream_t stream);
bool fft_sr_supported(int A, int B, int64_t I);
// One-time set-up of the strided-axis kernels that use more LDS than a launch gets by default
// (idempotent; called at plan creation).
hipError_t configure_fft_kernels();
// Strided-axis pass with the second factor split once more (16 x 128); launch_fft_sr_ex uses it for the
// split it covers.
bool fft_sn_supported(int A, int B, int64_t I);
hipError_t launch_fft_sn(const FftStridedArgs& a, int A, int B, const DeviceMatrix& FA, const DeviceMatrix& FB,
                         const float2* Tw, float scale, int conj, hipStream_t stream);
hipError_t configure_fft_nested_kernels();
hipError_t launch_fft_sr(const float2* in, float2* out, int64_t O, int64_t I, int A, int B,
                         const DeviceMatrix& FA, const DeviceMatrix& FB, const float2* Tw, float scale,
                         int conj, hipStream_t stream);

// ---- plain copy (bandwidth reference / counter calibration) -------------------------------
// variant: units digit = accesses in flight per thread (1, 2, else 4); tens digit t > 0 caps the
// grid at 256*t workgroups (grid-stride), 0 launches one chunk per workgroup.
// Whole KDFT transform of a tensor whose axes are all at most 32 long (input and output) in one
// launch: in[Mx.N][My.N][Mz.N] -> out[Mx.K][My.K][Mz.K], scaled, matrices conjugated when conj != 0.
bool kdft_small_supported(const DeviceMatrix& Mx, const DeviceMatrix& My, const DeviceMatrix& Mz);
hipError_t launch_kdft_small(const float2* in, float2* out, const DeviceMatrix& Mx, const DeviceMatrix& My,
                             const DeviceMatrix& Mz, float scale, int conj, hipStream_t stream);

hipError_t launch_copy(const void* in, void* out, size_t bytes, int variant, hipStream_t stream);

// ---- host generator -----------------------------------------------------------------------
// exp(sign * 2 pi i * t) for t = p/q reduced exactly (uniform) or a real number of turns.
void unit_root_ratio(int64_t p, int64_t q, int sign, double* re, double* im);
void unit_root_turns(double t, int sign, double* re, double* im);
// K x N matrix of Eq. 3 as printed for K evaluation points z (re, im pairs), in fp64.
dft3d_status generate_points_matrix_f64(int64_t k, int64_t n, const double* z, double* re, double* im);

void set_error(const char* fmt, ...);

// dft3d_exec with the intermediate storage given explicitly instead of taken from the plan.
dft3d_status exec_with_workspace(dft3d_plan p, const void* in, void* out, int direction, void* stream,
                                 void* workspace, size_t workspace_bytes, const char* who);

// Device address, on the current device, of the library's static scratch array (resolved once per
// device); nullptr with the error text set on failure.
void* noalloc_scratch_for_current_device();

}  // namespace dft3d
