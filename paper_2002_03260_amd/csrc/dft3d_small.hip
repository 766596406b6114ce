// Whole KDFT transform of a small tensor (every axis at most 32 long, on input and on output) in ONE
// launch.  At these sizes (paper Eq. 10 on a 32^3 tensor is 256 KiB and 2.5e7 flop) three mode
// kernels are pure launch latency, so one workgroup per output index k_x does all three modes:
//
//   1. S[b, c]   = sum_a  Mx[k_x, a] * in[a, b, c]       (mode x, for this workgroup's k_x only;
//                                                         the input is read by every workgroup, from L2;
//                                                         all of a thread's loads are in flight at once)
//   2. T[b, k_z] = sum_c  S[b, c] * Mz[k_z, c]            (mode z, in LDS)
//   3. out[k_x, k_y, k_z] = scale * sum_b My[k_y, b] * T[b, k_z]      (mode y, in LDS)
//
// which is Eq. 11's Kronecker factorisation applied in the order x, z, y.  Mode x is plain fp32 vector
// arithmetic on data streamed from L2; modes z and y are 32 x 32 x 32 products in LDS and run on the
// matrix cores (as vector code they were bound by LDS bandwidth: 2 us each of a 12 us kernel).  The
// matrices may be rectangular (evaluation-point plans) and are conjugated for BACKWARD.
#include <hip/hip_runtime.h>

#include "dft3d_internal.h"

namespace dft3d {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kSmallMax = 32;              // longest axis served
constexpr int kPitch = kSmallMax + 1;      // odd pitch (in complex numbers): rows land on distinct banks
constexpr int kSmallThreads = 1024;        // one thread per element of a 32 x 32 slab

__device__ __forceinline__ float2 cmul_add(float2 acc, float2 a, float2 b)
{
    acc.x = fmaf(a.x, b.x, acc.x);
    acc.x = fmaf(-a.y, b.y, acc.x);
    acc.y = fmaf(a.x, b.y, acc.y);
    acc.y = fmaf(a.y, b.x, acc.y);
    return acc;
}

// Matrix planes are stored transposed, plane[n * ld + k]; sgn = -1 conjugates.
__device__ __forceinline__ float2 entry(const DeviceMatrix& M, int k, int n, float sgn)
{
    const int idx = n * M.ld + k;
    return make_float2(M.re[idx], sgn * M.im[idx]);
}

__global__ __launch_bounds__(kSmallThreads) void k_kdft_small(const float2* __restrict__ in, float2* __restrict__ out,
                                                    DeviceMatrix Mx, DeviceMatrix My, DeviceMatrix Mz,
                                                    float scale, int conj)
{
    __shared__ float2 mx[kSmallMax];                    // Mx[k_x, a] of this workgroup
    __shared__ float2 my[kSmallMax * kPitch];           // My[k_y, b]
    __shared__ float2 mz[kSmallMax * kPitch];           // Mz[k_z, c]
    __shared__ float2 S[kSmallMax * kPitch];            // [b][c]
    __shared__ float2 T[kSmallMax * kPitch];            // [b][k_z]

    const int nx = Mx.N, ny = My.N, nz = Mz.N;          // input lengths
    const int ky = My.K, kz = Mz.K;                     // output lengths (kx = gridDim.x)
    const int kx_i = blockIdx.x;
    const int tid = threadIdx.x;
    const float sgn = conj ? -1.0f : 1.0f;

    // The kernel is a chain of memory latencies, so everything it reads from global memory is
    // requested first, in one go: this thread's entry of My and of Mz, its entry of the Mx row and the
    // whole column in[:, b, c] of its slab element (b, c) -- up to 32 independent loads in flight.
    // Thread t is element (b, c) = (t / 32, t % 32) of the zero-padded 32 x 32 slab and entry
    // (k, n) = (t % 32, t / 32) of the zero-padded matrices (consecutive threads, consecutive k: the
    // planes are contiguous along k).
    const int b = tid >> 5, c = tid & 31;
    const bool live = b < ny && c < nz;
    const int64_t plane = (int64_t)ny * nz;
    const float2* col = in + (live ? (int64_t)b * nz + c : 0);
    float2 xin[kSmallMax];
#pragma unroll
    for (int a = 0; a < kSmallMax; ++a) xin[a] = col[(int64_t)(a < nx ? a : nx - 1) * plane];     // (rows past nx: re-read, weight 0)
    const int mk = tid & 31, mn = tid >> 5;
    const float2 ey = (mk < ky && mn < ny) ? entry(My, mk, mn, sgn) : make_float2(0.f, 0.f);
    const float2 ez = (mk < kz && mn < nz) ? entry(Mz, mk, mn, sgn) : make_float2(0.f, 0.f);
    if (tid < kSmallMax) mx[tid] = tid < nx ? entry(Mx, kx_i, tid, sgn) : make_float2(0.f, 0.f);
    my[mk * kPitch + mn] = ey;
    mz[mk * kPitch + mn] = ez;
    __syncthreads();

    // 1. mode x for this k_x, from the registers; elements outside the tensor are the zero padding that
    // the 32 x 32 x 32 products below rely on
    {
        float2 acc = make_float2(0.f, 0.f);
#pragma unroll
        for (int a = 0; a < kSmallMax; ++a) acc = cmul_add(acc, mx[a], xin[a]);
        S[b * kPitch + c] = live ? acc : make_float2(0.f, 0.f);
    }
    __syncthreads();

    // 2. mode z and 3. mode y on the matrix cores: 32 x 32 x 32 complex products (the arrays are zero
    // beyond the actual lengths), one 16 x 16 output block per wave for the first four waves.
    // MFMA 16x16x4 operand layout: lane l supplies A[l % 16][l / 16] and B[l / 16][l % 16]; accumulator
    // register v is D[4 * (l / 16) + v][l % 16].
    const int wave = tid >> 6, lane = tid & 63;
    const int l16 = lane & 15, lq = lane >> 4;
    const int bi = (wave >> 1) * 16, bj = (wave & 1) * 16;      // block origin (rows, columns)
    if (wave < 4) {
        // T[b, k_z] = sum_c S[b, c] * Mz[k_z, c]:  A = S (rows b), B[c][k_z] = mz[k_z][c]
        f32x4 pr = {0.f, 0.f, 0.f, 0.f}, pi = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int st = 0; st < kSmallMax / 4; ++st) {
            const float2 av = S[(bi + l16) * kPitch + 4 * st + lq];
            const float2 bv = mz[(bj + l16) * kPitch + 4 * st + lq];
            pr = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, bv.x, pr, 0, 0, 0);
            pi = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, bv.y, pi, 0, 0, 0);
            pr = __builtin_amdgcn_mfma_f32_16x16x4f32(-av.y, bv.y, pr, 0, 0, 0);
            pi = __builtin_amdgcn_mfma_f32_16x16x4f32(av.y, bv.x, pi, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) T[(bi + 4 * lq + v) * kPitch + bj + l16] = make_float2(pr[v], pi[v]);
    }
    __syncthreads();
    if (wave < 4) {
        // out[k_y, k_z] = sum_b My[k_y, b] * T[b, k_z]:  A = my (rows k_y), B[b][k_z] = T[b][k_z]
        f32x4 pr = {0.f, 0.f, 0.f, 0.f}, pi = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int st = 0; st < kSmallMax / 4; ++st) {
            const float2 av = my[(bi + l16) * kPitch + 4 * st + lq];
            const float2 bv = T[(4 * st + lq) * kPitch + bj + l16];
            pr = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, bv.x, pr, 0, 0, 0);
            pi = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, bv.y, pi, 0, 0, 0);
            pr = __builtin_amdgcn_mfma_f32_16x16x4f32(-av.y, bv.y, pr, 0, 0, 0);
            pi = __builtin_amdgcn_mfma_f32_16x16x4f32(av.y, bv.x, pi, 0, 0, 0);
        }
        const int k3 = bj + l16;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int k2 = bi + 4 * lq + v;
            if (k2 < ky && k3 < kz)
                out[((int64_t)kx_i * ky + k2) * kz + k3] = make_float2(pr[v] * scale, pi[v] * scale);
        }
    }
}

}  // namespace

bool kdft_small_supported(const DeviceMatrix& Mx, const DeviceMatrix& My, const DeviceMatrix& Mz)
{
    const DeviceMatrix* m[3] = {&Mx, &My, &Mz};
    for (const DeviceMatrix* q : m)
        if (!q->re || q->N < 1 || q->K < 1 || q->N > kSmallMax || q->K > kSmallMax) return false;
    return true;
}

hipError_t launch_kdft_small(const float2* in, float2* out, const DeviceMatrix& Mx, const DeviceMatrix& My,
                             const DeviceMatrix& Mz, float scale, int conj, hipStream_t stream)
{
    if (!kdft_small_supported(Mx, My, Mz)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_kdft_small, dim3((unsigned)Mx.K), dim3(kSmallThreads), 0, stream, in, out, Mx, My, Mz, scale, conj);
    return hipGetLastError();
}

}  // namespace dft3d
