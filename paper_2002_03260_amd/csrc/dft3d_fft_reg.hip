// FFT formulation of the contiguous (z) axis with the whole axis pass in registers: first stage,
// twiddle, second stage and natural-order stores of one row of N = A*B points by ONE wavefront,
// without LDS and without barriers (paper Eq. 13 - Eq. 16 for one axis; n = B*l + beta,
// k = k_a + A*k_b).
//
// The trick is in the operand layouts of v_mfma_f32_16x16x4_f32 (A[i = lane % 16][k = lane / 16],
// B[k = lane / 16][j = lane % 16], D register v of a lane = row 4*(lane/16) + v, column lane % 16):
//
//   stage 1 is computed transposed,  Zt[beta, k_a] = sum_l Xt[beta, l] FA[l, k_a]:
//     A operand = data straight from global memory (lane: beta = 16*bb + lane%16, l = 4*s + lane/16,
//                 i.e. four 128-byte segments per load),  B operand = FA (constant registers),
//     D holds rows beta = 16*bb + 4*(lane/16) + v and columns k_a = 16*ab + lane%16;
//   the twiddle multiplies D element by element (its table is pre-arranged in the D layout);
//   stage 2,  Wt[k_b, k_a] = sum_beta FB[k_b, beta] Zt[beta, k_a],  contracts over the ROW index of
//     D.  A sum does not care about the order of its terms, so D register v is used directly as
//     the B operand of k-step (bb, v) -- lane group g then stands for beta = 16*bb + 4*g + v -- and
//     the A operand FB[k_b, beta] is loaded once in that permuted order (constant registers);
//   D of stage 2 has rows k_b = 16*kbb + 4*(lane/16) + v and columns k_a: the output index
//     k = k_a + A*k_b runs along the lanes, so the stores are 128-byte segments as well.
//
// Every row costs (A + B) * (A*B / 256) MFMAs with four real products per complex product (96 for
// 16 x 32), three quarters of that with three (the M3 variant), and nothing else but a few VALU
// operations per point for the twiddle and the sums.  With no LDS and no barriers, three to eight
// waves per SIMD overlap each other's loads, stores and MFMAs.
#include <hip/hip_runtime.h>

#include "dft3d_internal.h"

namespace dft3d {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ f32x4 mfma(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

template <int A, int B, int MINW, bool M3>
__global__ __launch_bounds__(256, MINW) void k_fft_zr(const float2* __restrict__ in, float2* __restrict__ out,
                                                       int64_t nrows, DeviceMatrix FA, DeviceMatrix FB,
                                                       const float2* __restrict__ Tw, float scale, int conj)
{
    constexpr int N = A * B;
    constexpr int NAB = A / 16;      // blocks of k_a
    constexpr int NBB = B / 16;      // blocks of beta (and of k_b)
    constexpr int NS1 = A / 4;       // k-steps of stage 1 (over l)

    const int lane = threadIdx.x & 63;
    const int l16 = lane & 15, lq = lane >> 4;
    const int64_t wave = ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * gridDim.y * 4;
    if (wave >= nrows) return;

    const float isign = conj ? -1.0f : 1.0f;

    // ---- constants, loaded once per wave ---------------------------------------------------
    // stage-1 B operand: FA[k_a = 16*ab + l16][l = 4*s + lq]   (matrix planes are plane[n * ld + k])
    float fa_r[NAB][NS1], fa_i[NAB][NS1], fa_s[NAB][NS1];       // fa_s = re + im, for the three-product scheme
#pragma unroll
    for (int ab = 0; ab < NAB; ++ab)
#pragma unroll
        for (int s = 0; s < NS1; ++s) {
            const int idx = (4 * s + lq) * FA.ld + 16 * ab + l16;
            fa_r[ab][s] = FA.re[idx];
            fa_i[ab][s] = FA.im[idx] * isign;
            fa_s[ab][s] = fa_r[ab][s] + fa_i[ab][s];
        }
    // stage-2 A operand: scale * FB[k_b = 16*kbb + l16][beta = 16*bb + 4*lq + v]
    float fb_r[NBB][NBB][4], fb_i[NBB][NBB][4], fb_s[NBB][NBB][4];
#pragma unroll
    for (int kbb = 0; kbb < NBB; ++kbb)
#pragma unroll
        for (int bb = 0; bb < NBB; ++bb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int idx = (16 * bb + 4 * lq + v) * FB.ld + 16 * kbb + l16;
                fb_r[kbb][bb][v] = FB.re[idx] * scale;
                fb_i[kbb][bb][v] = FB.im[idx] * (scale * isign);
                fb_s[kbb][bb][v] = fb_r[kbb][bb][v] + fb_i[kbb][bb][v];
            }
    // twiddle in the D layout of stage 1: T[k_a = 16*ab + l16][beta = 16*bb + 4*lq + v]
    float tw_r[NBB][NAB][4], tw_i[NBB][NAB][4];
#pragma unroll
    for (int bb = 0; bb < NBB; ++bb)
#pragma unroll
        for (int ab = 0; ab < NAB; ++ab)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float2 t = Tw[(16 * ab + l16) * B + 16 * bb + 4 * lq + v];
                tw_r[bb][ab][v] = t.x;
                tw_i[bb][ab][v] = t.y * isign;
            }

    // ---- rows ------------------------------------------------------------------------------
    // Two register sets take turns: while one row is transformed the loads of the wave's next row
    // are already in flight into the other set (requested first thing in the iteration, so the
    // wait for a row never includes the stores issued after its request).
    const int ld_off = B * lq + l16;     // + B*4*s + 16*bb
    auto load_row = [&](f32x2 (&x)[NBB][NS1], int64_t row) {
        const f32x2* src = reinterpret_cast<const f32x2*>(in) + row * N + ld_off;
#pragma unroll
        for (int bb = 0; bb < NBB; ++bb)
#pragma unroll
            for (int s = 0; s < NS1; ++s) x[bb][s] = src[4 * B * s + 16 * bb];
    };
    // Three real products per complex product: with P1 = sum a_r b_r, P2 = sum a_i b_i and
    // P3 = sum (a_r + a_i)(b_r + b_i), Re = P1 - P2 and Im = P3 - P1 - P2: 72 instead of 96 MFMAs per
    // row for 16 x 32, paid with a few additions per point.
    auto transform_row_3m = [&](const f32x2 (&x)[NBB][NS1], int64_t row) {
        f32x4 p1[NBB][NAB], p2[NBB][NAB], p3[NBB][NAB];
#pragma unroll
        for (int bb = 0; bb < NBB; ++bb)
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab) {
                p1[bb][ab] = f32x4{0.f, 0.f, 0.f, 0.f};
                p2[bb][ab] = f32x4{0.f, 0.f, 0.f, 0.f};
                p3[bb][ab] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
        for (int s = 0; s < NS1; ++s)
#pragma unroll
            for (int bb = 0; bb < NBB; ++bb) {
                const float xs = x[bb][s].x + x[bb][s].y;
#pragma unroll
                for (int ab = 0; ab < NAB; ++ab) {
                    p1[bb][ab] = mfma(x[bb][s].x, fa_r[ab][s], p1[bb][ab]);
                    p2[bb][ab] = mfma(x[bb][s].y, fa_i[ab][s], p2[bb][ab]);
                    p3[bb][ab] = mfma(xs, fa_s[ab][s], p3[bb][ab]);
                }
            }
        // combine, twiddle, and the sum stage 2 needs
        f32x4 zr[NBB][NAB], zi[NBB][NAB], zs[NBB][NAB];
#pragma unroll
        for (int bb = 0; bb < NBB; ++bb)
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float a = p1[bb][ab][v] - p2[bb][ab][v];
                    const float b = p3[bb][ab][v] - p1[bb][ab][v] - p2[bb][ab][v];
                    zr[bb][ab][v] = a * tw_r[bb][ab][v] - b * tw_i[bb][ab][v];
                    zi[bb][ab][v] = a * tw_i[bb][ab][v] + b * tw_r[bb][ab][v];
                    zs[bb][ab][v] = zr[bb][ab][v] + zi[bb][ab][v];
                }
        f32x4 q1[NBB][NAB], q2[NBB][NAB], q3[NBB][NAB];
#pragma unroll
        for (int kbb = 0; kbb < NBB; ++kbb)
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab) {
                q1[kbb][ab] = f32x4{0.f, 0.f, 0.f, 0.f};
                q2[kbb][ab] = f32x4{0.f, 0.f, 0.f, 0.f};
                q3[kbb][ab] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
        for (int bb = 0; bb < NBB; ++bb)
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int kbb = 0; kbb < NBB; ++kbb)
#pragma unroll
                    for (int ab = 0; ab < NAB; ++ab) {
                        q1[kbb][ab] = mfma(fb_r[kbb][bb][v], zr[bb][ab][v], q1[kbb][ab]);
                        q2[kbb][ab] = mfma(fb_i[kbb][bb][v], zi[bb][ab][v], q2[kbb][ab]);
                        q3[kbb][ab] = mfma(fb_s[kbb][bb][v], zs[bb][ab][v], q3[kbb][ab]);
                    }
        f32x2* dst = reinterpret_cast<f32x2*>(out) + row * N + l16 + A * 4 * lq;
#pragma unroll
        for (int kbb = 0; kbb < NBB; ++kbb)
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    dst[16 * ab + A * (16 * kbb + v)] = f32x2{q1[kbb][ab][v] - q2[kbb][ab][v],
                                                             q3[kbb][ab][v] - q1[kbb][ab][v] - q2[kbb][ab][v]};
    };
    auto transform_row_4m = [&](const f32x2 (&x)[NBB][NS1], int64_t row) {
        // stage 1
        f32x4 zr[NBB][NAB], zi[NBB][NAB];
#pragma unroll
        for (int bb = 0; bb < NBB; ++bb)
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab) {
                zr[bb][ab] = f32x4{0.f, 0.f, 0.f, 0.f};
                zi[bb][ab] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
        for (int s = 0; s < NS1; ++s) {
#pragma unroll
            for (int bb = 0; bb < NBB; ++bb)
#pragma unroll
                for (int ab = 0; ab < NAB; ++ab) {
                    zr[bb][ab] = mfma(x[bb][s].x, fa_r[ab][s], zr[bb][ab]);
                    zi[bb][ab] = mfma(x[bb][s].x, fa_i[ab][s], zi[bb][ab]);
                }
#pragma unroll
            for (int bb = 0; bb < NBB; ++bb)
#pragma unroll
                for (int ab = 0; ab < NAB; ++ab) {
                    zr[bb][ab] = mfma(-x[bb][s].y, fa_i[ab][s], zr[bb][ab]);
                    zi[bb][ab] = mfma(x[bb][s].y, fa_r[ab][s], zi[bb][ab]);
                }
        }
        // twiddle; zn = -Im is what the real part of stage 2 multiplies
        f32x4 zn[NBB][NAB];
#pragma unroll
        for (int bb = 0; bb < NBB; ++bb)
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float a = zr[bb][ab][v], b = zi[bb][ab][v];
                    zr[bb][ab][v] = a * tw_r[bb][ab][v] - b * tw_i[bb][ab][v];
                    zi[bb][ab][v] = a * tw_i[bb][ab][v] + b * tw_r[bb][ab][v];
                    zn[bb][ab][v] = -zi[bb][ab][v];
                }
        // stage 2
        f32x4 wr[NBB][NAB], wi[NBB][NAB];
#pragma unroll
        for (int kbb = 0; kbb < NBB; ++kbb)
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab) {
                wr[kbb][ab] = f32x4{0.f, 0.f, 0.f, 0.f};
                wi[kbb][ab] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
        for (int bb = 0; bb < NBB; ++bb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
#pragma unroll
                for (int kbb = 0; kbb < NBB; ++kbb)
#pragma unroll
                    for (int ab = 0; ab < NAB; ++ab) {
                        wr[kbb][ab] = mfma(fb_r[kbb][bb][v], zr[bb][ab][v], wr[kbb][ab]);
                        wi[kbb][ab] = mfma(fb_r[kbb][bb][v], zi[bb][ab][v], wi[kbb][ab]);
                    }
#pragma unroll
                for (int kbb = 0; kbb < NBB; ++kbb)
#pragma unroll
                    for (int ab = 0; ab < NAB; ++ab) {
                        wr[kbb][ab] = mfma(fb_i[kbb][bb][v], zn[bb][ab][v], wr[kbb][ab]);
                        wi[kbb][ab] = mfma(fb_i[kbb][bb][v], zr[bb][ab][v], wi[kbb][ab]);
                    }
            }
        // natural order: k = k_a + A * k_b
        f32x2* dst = reinterpret_cast<f32x2*>(out) + row * N + l16 + A * 4 * lq;
#pragma unroll
        for (int kbb = 0; kbb < NBB; ++kbb)
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    dst[16 * ab + A * (16 * kbb + v)] = f32x2{wr[kbb][ab][v], wi[kbb][ab][v]};
    };

    f32x2 xa[NBB][NS1], xb[NBB][NS1];
    load_row(xa, wave);
    for (int64_t row = wave; row < nrows; row += 2 * nwaves) {
        // a request past the end re-reads the wave's current row (in bounds, never used)
        const int64_t row1 = row + nwaves, row2 = row + 2 * nwaves;
        load_row(xb, row1 < nrows ? row1 : row);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (M3) transform_row_3m(xa, row);
        else transform_row_4m(xa, row);
        __builtin_amdgcn_sched_barrier(0);
        if (row1 >= nrows) break;
        load_row(xa, row2 < nrows ? row2 : row);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (M3) transform_row_3m(xb, row1);
        else transform_row_4m(xb, row1);
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int A, int B, int MINW, bool M3>
hipError_t launch_inst(const float2* in, float2* out, int64_t nrows, const DeviceMatrix& FA,
                       const DeviceMatrix& FB, const float2* Tw, float scale, int conj, hipStream_t stream)
{
    // persistent waves: MINW per SIMD on every CU, fewer when there are fewer rows
    const int64_t resident = 256 * MINW;                 // workgroups of 4 waves
    const int64_t want = (nrows + 3) / 4;
    const int64_t blocks = want < resident ? want : resident;
    hipLaunchKernelGGL((k_fft_zr<A, B, MINW, M3>), dim3((unsigned)blocks), dim3(256), 0, stream, in, out, nrows, FA, FB,
                       Tw, scale, conj);
    return hipGetLastError();
}

}  // namespace

bool fft_zr_supported(int A, int B)
{
    return (A == 16 && B == 16) || (A == 16 && B == 32) || (A == 32 && B == 32);
}

hipError_t launch_fft_zr(const float2* in, float2* out, int64_t nrows, int A, int B, const DeviceMatrix& FA,
                         const DeviceMatrix& FB, const float2* Tw, float scale, int conj, hipStream_t stream)
{
    if (nrows <= 0) return hipSuccess;
    // the kernel indexes the stage matrices and the twiddle table without bounds checks
    if (FA.K != A || FA.N != A || FB.K != B || FB.N != B || !Tw) return hipErrorInvalidValue;
    // three-product scheme where its registers still allow three waves per SIMD (measured 15 % faster
    // at 16 x 32); 32 x 32 would spill with it and runs the four-product scheme
    if (A == 16 && B == 16) return launch_inst<16, 16, 6, true>(in, out, nrows, FA, FB, Tw, scale, conj, stream);
    if (A == 16 && B == 32) return launch_inst<16, 32, 3, true>(in, out, nrows, FA, FB, Tw, scale, conj, stream);
    if (A == 32 && B == 32) return launch_inst<32, 32, 2, false>(in, out, nrows, FA, FB, Tw, scale, conj, stream);
    return hipErrorInvalidValue;
}

}  // namespace dft3d
