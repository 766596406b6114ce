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

// The outputs of these passes are not read again by the kernel that writes them: streaming store.
__device__ __forceinline__ void stream_store(f32x2* dst, f32x2 v) { __builtin_nontemporal_store(v, dst); }
__device__ __forceinline__ f32x2 stream_load(const f32x2* src) { return __builtin_nontemporal_load(src); }

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
            for (int s = 0; s < NS1; ++s) x[bb][s] = stream_load(&src[4 * B * s + 16 * bb]);
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
                    stream_store(&dst[16 * ab + A * (16 * kbb + v)],
                                 f32x2{q1[kbb][ab][v] - q2[kbb][ab][v],
                                       q3[kbb][ab][v] - q1[kbb][ab][v] - q2[kbb][ab][v]});
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
                    stream_store(&dst[16 * ab + A * (16 * kbb + v)], f32x2{wr[kbb][ab][v], wi[kbb][ab][v]});
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

// Contiguous axis, larger splits (32 x 64): the same one-wavefront-per-row scheme, but the stage
// matrices and the twiddle table no longer fit the register file next to the row's intermediate,
// so they sit in LDS, pre-arranged in per-lane operand order ([...][lane]: every read is lane
// contiguous and conflict free) and never written after the fill -- still no barrier in the row
// loop.  Stage 1 runs one block of 16 beta at a time (its data requested one block ahead, across
// rows), stage 2 one block of 16 k_b at a time with its results stored at once, so the registers
// hold the intermediate Z of the row (A*B/32 of them) plus one block of accumulators.  Three real
// products per complex product.
template <int A, int B>
__global__ __launch_bounds__(512, 2) void k_fft_zl(const float2* __restrict__ in, float2* __restrict__ out,
                                                    int64_t nrows, DeviceMatrix FA, DeviceMatrix FB,
                                                    const float2* __restrict__ Tw, float scale, int conj)
{
    constexpr int N = A * B;
    constexpr int NAB = A / 16;      // blocks of k_a
    constexpr int NBB = B / 16;      // blocks of beta (and of k_b)
    constexpr int NS1 = A / 4;       // k-steps of stage 1 (over l)

    __shared__ float fa_r[NAB * NS1 * 64], fa_i[NAB * NS1 * 64];             // [ab][s][lane]
    __shared__ float fb_r[NBB * NBB * 4 * 64], fb_i[NBB * NBB * 4 * 64];     // [kbb][bb][v][lane]
    __shared__ float2 tws[NBB * NAB * 4 * 64];                               // [bb][ab][v][lane]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int l16 = lane & 15, lq = lane >> 4;
    const float isign = conj ? -1.0f : 1.0f;

    for (int e = tid; e < NAB * NS1 * 64; e += 512) {
        const int ln = e & 63, s = (e >> 6) % NS1, ab = (e >> 6) / NS1;
        const int idx = (4 * s + (ln >> 4)) * FA.ld + 16 * ab + (ln & 15);       // FA[k_a][l] at plane[l * ld + k_a]
        fa_r[e] = FA.re[idx];
        fa_i[e] = FA.im[idx] * isign;
    }
    for (int e = tid; e < NBB * NBB * 4 * 64; e += 512) {
        const int ln = e & 63, v = (e >> 6) & 3, bb = (e >> 8) % NBB, kbb = (e >> 8) / NBB;
        const int idx = (16 * bb + 4 * (ln >> 4) + v) * FB.ld + 16 * kbb + (ln & 15);   // FB[k_b][beta]
        fb_r[e] = FB.re[idx] * scale;
        fb_i[e] = FB.im[idx] * (scale * isign);
    }
    for (int e = tid; e < NBB * NAB * 4 * 64; e += 512) {
        const int ln = e & 63, v = (e >> 6) & 3, ab = (e >> 8) % NAB, bb = (e >> 8) / NAB;
        float2 t = Tw[(16 * ab + (ln & 15)) * B + 16 * bb + 4 * (ln >> 4) + v];  // T[k_a][beta]
        t.y *= isign;
        tws[e] = t;
    }
    __syncthreads();

    const int64_t wave = (int64_t)blockIdx.x * 8 + (tid >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 8;
    if (wave >= nrows) return;                    // after the only barrier

    const int ld_off = B * lq + l16;              // + B*4*s + 16*bb
    auto load_block = [&](f32x2 (&x)[NS1], int64_t row, int bb) {
        const f32x2* src = reinterpret_cast<const f32x2*>(in) + row * N + ld_off + 16 * bb;
#pragma unroll
        for (int s = 0; s < NS1; ++s) x[s] = stream_load(&src[4 * B * s]);
    };

    f32x4 zr[NBB][NAB], zi[NBB][NAB];
    auto stage1_block = [&](const f32x2 (&x)[NS1], int bb) {
        f32x4 p1[NAB], p2[NAB], p3[NAB];
#pragma unroll
        for (int ab = 0; ab < NAB; ++ab) {
            p1[ab] = f32x4{0.f, 0.f, 0.f, 0.f};
            p2[ab] = f32x4{0.f, 0.f, 0.f, 0.f};
            p3[ab] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int s = 0; s < NS1; ++s) {
            const float xs = x[s].x + x[s].y;
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab) {
                const float fr = fa_r[(ab * NS1 + s) * 64 + lane], fi = fa_i[(ab * NS1 + s) * 64 + lane];
                p1[ab] = mfma(x[s].x, fr, p1[ab]);
                p2[ab] = mfma(x[s].y, fi, p2[ab]);
                p3[ab] = mfma(xs, fr + fi, p3[ab]);
            }
        }
#pragma unroll
        for (int ab = 0; ab < NAB; ++ab)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float2 t = tws[((bb * NAB + ab) * 4 + v) * 64 + lane];
                const float a = p1[ab][v] - p2[ab][v];
                const float b = p3[ab][v] - p1[ab][v] - p2[ab][v];
                zr[bb][ab][v] = a * t.x - b * t.y;
                zi[bb][ab][v] = a * t.y + b * t.x;
            }
    };
    auto stage2_block = [&](int64_t row, int kbb) {
        f32x4 q1[NAB], q2[NAB], q3[NAB];
#pragma unroll
        for (int ab = 0; ab < NAB; ++ab) {
            q1[ab] = f32x4{0.f, 0.f, 0.f, 0.f};
            q2[ab] = f32x4{0.f, 0.f, 0.f, 0.f};
            q3[ab] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int bb = 0; bb < NBB; ++bb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (v == 0 && bb > 0) __builtin_amdgcn_sched_barrier(0);
                const float gr = fb_r[((kbb * NBB + bb) * 4 + v) * 64 + lane];
                const float gi = fb_i[((kbb * NBB + bb) * 4 + v) * 64 + lane];
                const float gs = gr + gi;
#pragma unroll
                for (int ab = 0; ab < NAB; ++ab) {
                    q1[ab] = mfma(gr, zr[bb][ab][v], q1[ab]);
                    q2[ab] = mfma(gi, zi[bb][ab][v], q2[ab]);
                    q3[ab] = mfma(gs, zr[bb][ab][v] + zi[bb][ab][v], q3[ab]);
                }
            }
        // natural order: k = k_a + A * k_b
        f32x2* dst = reinterpret_cast<f32x2*>(out) + row * N + l16 + A * 4 * lq + A * 16 * kbb;
#pragma unroll
        for (int ab = 0; ab < NAB; ++ab)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                stream_store(&dst[16 * ab + A * v], f32x2{q1[ab][v] - q2[ab][v], q3[ab][v] - q1[ab][v] - q2[ab][v]});
    };

    static_assert(NBB % 2 == 0, "the two data register sets alternate block by block");
    f32x2 xa[NS1], xb[NS1];
    load_block(xa, wave, 0);
    for (int64_t row = wave; row < nrows; row += nwaves) {
        const int64_t next = row + nwaves < nrows ? row + nwaves : row;    // past the end: a harmless re-read
        // the tables are loop invariant, but keeping them in registers across rows is exactly what
        // does not fit: make the compiler read them again in every row
        asm volatile("" ::: "memory");
#pragma unroll
        for (int bb = 0; bb < NBB; bb += 2) {
            load_block(xb, row, bb + 1);
            __builtin_amdgcn_sched_barrier(0);
            stage1_block(xa, bb);
            __builtin_amdgcn_sched_barrier(0);
            if (bb + 2 < NBB) load_block(xa, row, bb + 2);
            else load_block(xa, next, 0);
            __builtin_amdgcn_sched_barrier(0);
            stage1_block(xb, bb + 1);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int kbb = 0; kbb < NBB; ++kbb) {
            stage2_block(row, kbb);
            __builtin_amdgcn_sched_barrier(0);      // keeps the table reads of later blocks from being issued early
        }
    }
}

// ---- strided axes ------------------------------------------------------------------------------
// Tensor viewed as [O][N = A*B][I]; a workgroup of four waves transforms one tile of all N positions
// x 16 contiguous columns at a time.  The columns are the MFMA column index (lane % 16), so the
// data is the B operand of both stages and 16 lanes cover one 128-byte segment:
//   stage 1 (wave w takes beta = w, w+4, ..):  D[k_a, i] = sum_l FA[k_a, l] x[B*l + beta, i]
//     with x straight from global memory into the operand registers -- the whole tile sits in
//     registers, requested one tile ahead, each register re-requested right after its last use;
//     twiddle on D; D goes to LDS as Z[k_a][beta][i];
//   stage 2 (wave w takes k_a = w, w+4, ..):   D[k_b, i] = sum_beta FB[k_b, beta] Z[k_a][beta][i]
//     with Z read from LDS in the order of the contraction; D is stored straight to global
//     memory at row k_a + A*k_b.
// Only Z passes through LDS (one write, one read, both conflict free without padding), with two
// barriers per tile; the stage matrices are constant operand registers.  Three real products per
// complex product (see the contiguous-axis kernel).
template <int A, int B, int MINW>
__global__ __launch_bounds__(256, MINW) void k_fft_sr(FftStridedArgs a, DeviceMatrix FA, DeviceMatrix FB,
                                                       const float2* __restrict__ Tw, float scale, int conj)
{
    const float2* __restrict__ X = a.X;
    float2* __restrict__ Y = a.Y;
    constexpr int N = A * B;
    static_assert(A == 16, "one block of k_a per stage-1 product");
    constexpr int NBB = B / 16;      // blocks of k_b
    constexpr int NS1 = A / 4;       // k-steps of stage 1 (over l)
    constexpr int NS2 = B / 4;       // k-steps of stage 2 (over beta)
    constexpr int NG = B / 4;        // beta values per wave
    constexpr int NH = A / 4;        // k_a values per wave

    __shared__ __align__(16) float2 Zs[N * 16];       // [k_a][beta][i]
    __shared__ __align__(16) float2 tws[N];           // T[k_a][beta], conjugated for BACKWARD

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // uniform: addresses built from it stay scalar
    const int l16 = lane & 15, lq = lane >> 4;
    const float isign = conj ? -1.0f : 1.0f;

    for (int e = tid; e < N; e += 256) {
        float2 t = Tw[e];
        t.y *= isign;
        tws[e] = t;
    }
    // stage-1 A operand: FA[k_a = l16][l = 4*s + lq]   (matrix planes are plane[n * ld + k])
    float fa_r[NS1], fa_i[NS1], fa_s[NS1];
#pragma unroll
    for (int s = 0; s < NS1; ++s) {
        const int idx = (4 * s + lq) * FA.ld + l16;
        fa_r[s] = FA.re[idx];
        fa_i[s] = FA.im[idx] * isign;
        fa_s[s] = fa_r[s] + fa_i[s];
    }
    // stage-2 A operand: scale * FB[k_b = 16*kbb + l16][beta = 4*s + lq]
    float fb_r[NBB][NS2], fb_i[NBB][NS2], fb_s[NBB][NS2];
#pragma unroll
    for (int kbb = 0; kbb < NBB; ++kbb)
#pragma unroll
        for (int s = 0; s < NS2; ++s) {
            const int idx = (4 * s + lq) * FB.ld + 16 * kbb + l16;
            fb_r[kbb][s] = FB.re[idx] * scale;
            fb_i[kbb][s] = FB.im[idx] * (scale * isign);
            fb_s[kbb][s] = fb_r[kbb][s] + fb_i[kbb][s];
        }

    // tile -> (o, y, 16-column group); input and output have their own strides (see FftStridedArgs)
    const int64_t per_o = a.Yn * a.Zt;
    const int64_t ntiles = a.O * per_o;
    const int64_t nwg = (int64_t)gridDim.x * gridDim.y;
    // Addresses = uniform 64-bit base (tile, wave, compile-time row) + 32-bit lane offset; the host
    // side guarantees that the lane offsets fit.
    auto in_base = [&](int64_t tile) {
        const int64_t o = tile / per_o, r = tile % per_o;
        return o * a.inO + (r / a.Zt) * a.inY + (r % a.Zt) * 16;
    };
    auto out_base = [&](int64_t tile) {
        const int64_t o = tile / per_o, r = tile % per_o;
        return o * a.outO + (r / a.Zt) * a.outY + (r % a.Zt) * 16;
    };
    const int64_t inN = a.inN, outN = a.outN;
    const unsigned ld_lane = (unsigned)(B * lq) * (unsigned)inN + l16;        // row B*lq, column l16
    const unsigned st_lane = (unsigned)(A * 4 * lq) * (unsigned)outN + l16;   // row A*4*lq, column l16

    // operand registers of the tile: xq[g][s] = x[B*(4*s + lq) + beta_g, i], beta_g = wave + 4*g
    f32x2 xq[NG][NS1];
    auto request = [&](int64_t tile, int g) {
        const f32x2* src = reinterpret_cast<const f32x2*>(X) + in_base(tile) + (int64_t)(wave + 4 * g) * inN;
#pragma unroll
        for (int s = 0; s < NS1; ++s) xq[g][s] = stream_load(&(src + (int64_t)(4 * B * s) * inN)[ld_lane]);
    };

    int64_t tile = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
    if (tile < ntiles) {
#pragma unroll
        for (int g = 0; g < NG; ++g) request(tile, g);
    }
    __syncthreads();                               // twiddle table
    for (; tile < ntiles; tile += nwg) {
        const int64_t next = tile + nwg < ntiles ? tile + nwg : tile;    // past the end: a harmless re-read

        // ---- stage 1: two beta values at a time
#pragma unroll
        for (int g = 0; g < NG; g += 2) {
            f32x4 p1[2], p2[2], p3[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                p1[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                p2[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                p3[u] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int s = 0; s < NS1; ++s)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const f32x2 x = xq[g + u][s];
                    p1[u] = mfma(fa_r[s], x.x, p1[u]);
                    p2[u] = mfma(fa_i[s], x.y, p2[u]);
                    p3[u] = mfma(fa_s[s], x.x + x.y, p3[u]);
                }
            // the registers of these two beta values are free: request them for the next tile
            request(next, g);
            request(next, g + 1);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int beta = wave + 4 * (g + u);
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int ka = 4 * lq + v;
                    const float2 t = tws[ka * B + beta];
                    const float a = p1[u][v] - p2[u][v];
                    const float b = p3[u][v] - p1[u][v] - p2[u][v];
                    *reinterpret_cast<f32x2*>(&Zs[(ka * B + beta) * 16 + l16]) =
                        f32x2{a * t.x - b * t.y, a * t.y + b * t.x};
                }
            }
        }
        __syncthreads();

        // ---- stage 2: one k_a at a time, all blocks of k_b in flight
        f32x2* dst = reinterpret_cast<f32x2*>(Y) + out_base(tile);          // uniform
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            const int ka = wave + 4 * h;
            f32x4 q1[NBB], q2[NBB], q3[NBB];
#pragma unroll
            for (int kbb = 0; kbb < NBB; ++kbb) {
                q1[kbb] = f32x4{0.f, 0.f, 0.f, 0.f};
                q2[kbb] = f32x4{0.f, 0.f, 0.f, 0.f};
                q3[kbb] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int s = 0; s < NS2; ++s) {
                const f32x2 z = *reinterpret_cast<const f32x2*>(&Zs[(ka * B + 4 * s + lq) * 16 + l16]);
                const float zs = z.x + z.y;
#pragma unroll
                for (int kbb = 0; kbb < NBB; ++kbb) {
                    q1[kbb] = mfma(fb_r[kbb][s], z.x, q1[kbb]);
                    q2[kbb] = mfma(fb_i[kbb][s], z.y, q2[kbb]);
                    q3[kbb] = mfma(fb_s[kbb][s], zs, q3[kbb]);
                }
            }
#pragma unroll
            for (int kbb = 0; kbb < NBB; ++kbb)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    // row k_a + A*k_b with k_b = 16*kbb + 4*lq + v: the lq part is in st_lane
                    stream_store(&(dst + (int64_t)(ka + A * (16 * kbb + v)) * outN)[st_lane],
                                 f32x2{q1[kbb][v] - q2[kbb][v], q3[kbb][v] - q1[kbb][v] - q2[kbb][v]});
                }
        }
        __syncthreads();                           // Z is rewritten by the next tile
    }
}

// ---- strided axes, streaming form ------------------------------------------------------------------
// The kernels above keep the whole intermediate Z[k_a][beta][columns] of a tile in LDS, which limits a
// tile to N * columns * 8 bytes <= 128 KiB: 16 or 32 columns at N = 512, nothing at N = 2048.  Here Z
// never exists as a whole.  The second stage is a sum over beta, so its RESULT is what stays resident:
// every wave keeps the accumulators of its share of the output tile W[k_a][k_b][columns] in registers
// (the whole tile, N * columns complex numbers = 256 KiB, is half of the CU's register file) and the
// first stage feeds it a slot of SB consecutive beta at a time through a small double-buffered LDS
// ring:
//   slot t:  stage 1, wave w = (beta = SB*t + w / CH, column group w % CH):
//                D[k_a, c] = twiddle * sum_l FA[k_a, l] x[B*l + beta, c]   (data straight from global
//                memory into the MFMA B operand, requested two slots ahead)  ->  Z ring
//            one barrier
//            stage 2, wave w owns the pairs (k_a, column group) p = w, w + 8, ..:
//                W[k_a, k_b, c] += sum_{beta in slot} FB[k_b, beta] Z[k_a, beta, c]
//   after the last slot the accumulators are stored to rows k_a + A*k_b and cleared.
// Stage 1 uses three real products per complex product (its three accumulators live for one slot);
// stage 2 uses four with two accumulators (re, im), because three resident accumulators per output
// would not fit.  Per element 6*A + 8*B flop instead of 6*(A + B).
// A tile is all N positions x 16*CV*CH columns: CV = complex numbers per lane and access (1 or 2),
// CH = column groups side by side.  N = 512: CV = 2, CH = 2 (64 columns, 512 contiguous bytes per row
// from two neighbouring waves); N = 2048: CV = 1, CH = 1 (16 columns).  Stage matrices and twiddles
// sit in LDS in per-lane operand order.  One workgroup of eight waves per CU, one barrier per slot.
template <int CV>
struct cvec;
template <>
struct cvec<1> { typedef f32x2 type; };
template <>
struct cvec<2> { typedef f32x4 type; };

template <int A, int B, int CV, int CH, int SB>
struct FftSsLayout {
    static constexpr int N = A * B;
    static constexpr int NW = 8;
    static constexpr int NAB = A / 16, NBB = B / 16, NS1 = A / 4, KS = SB / 4, NSLOT = B / SB;
    static constexpr int PPW = A * CH / NW;                     // (k_a, column group) pairs per wave
    static constexpr int VB = 8 * CV;                           // bytes of one lane's element
    static constexpr int PK = CH * SB * 16 + 32 / VB;           // Z ring: elements per k_a (32 bytes of padding)
    static constexpr size_t z_bytes = (size_t)2 * A * PK * VB;
    static constexpr size_t fa_bytes = (size_t)NAB * NS1 * 3 * 64 * 4;
    static constexpr size_t fb_bytes = (size_t)NBB * (B / 4) * 2 * 64 * 4;
    static constexpr size_t tw_bytes = (size_t)N * 8;
    static constexpr size_t lds_bytes = z_bytes + fa_bytes + fb_bytes + tw_bytes;
    static_assert(SB * CH == NW, "one stage-1 unit per wave and slot");
    static_assert(SB % 4 == 0 && NSLOT % 2 == 0 && PPW >= 1 && (A * CH) % NW == 0, "slot structure");
};

template <int A, int B, int CV, int CH, int SB>
__global__ __launch_bounds__(512, 1) void k_fft_ss(FftStridedArgs a, DeviceMatrix FA, DeviceMatrix FB,
                                                    const float2* __restrict__ Tw, float scale, int conj)
{
    typedef FftSsLayout<A, B, CV, CH, SB> L;
    typedef typename cvec<CV>::type vec;
    constexpr int NAB = L::NAB, NBB = L::NBB, NS1 = L::NS1, KS = L::KS, NSLOT = L::NSLOT, PPW = L::PPW, PK = L::PK;
    constexpr int NW = L::NW;

    extern __shared__ __align__(16) unsigned char smem_ss[];
    // Operand tables in per-lane order, four consecutive k-steps (or all blocks of k_b) side by side, so
    // that one 16-byte LDS read feeds many matrix instructions:
    vec* Zs = reinterpret_cast<vec*>(smem_ss);                                   // [2][A][PK]
    f32x4* faT = reinterpret_cast<f32x4*>(smem_ss + L::z_bytes);                // [NAB][NS1/4][re, im, re+im][lane] x (4 k-steps)
    f32x4* fbT = reinterpret_cast<f32x4*>(smem_ss + L::z_bytes + L::fa_bytes);  // [B/4][NBB/2][lane] x (re, im of two blocks of k_b)
    float2* tws = reinterpret_cast<float2*>(smem_ss + L::z_bytes + L::fa_bytes + L::fb_bytes);   // T[beta][k_a]

    const float2* __restrict__ X = a.X;
    float2* __restrict__ Y = a.Y;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lq = lane >> 4;
    const float isign = conj ? -1.0f : 1.0f;

    // ---- tables, once per workgroup ------------------------------------------------------------------
    {
        float* faF = reinterpret_cast<float*>(faT);
        for (int e = tid; e < NAB * NS1 * 64; e += 512) {
            const int ln = e & 63, s = (e >> 6) % NS1, ab = (e >> 6) / NS1;
            const int idx = (4 * s + (ln >> 4)) * FA.ld + 16 * ab + (ln & 15);    // FA[k_a][l] at plane[l * ld + k_a]
            const float r = FA.re[idx], i = FA.im[idx] * isign;
            float* t = faF + (((ab * (NS1 / 4) + s / 4) * 3) * 64 + ln) * 4 + (s & 3);
            t[0] = r;
            t[64 * 4] = i;
            t[128 * 4] = r + i;
        }
        float* fbF = reinterpret_cast<float*>(fbT);
        for (int e = tid; e < NBB * (B / 4) * 64; e += 512) {
            const int ln = e & 63, bq = (e >> 6) % (B / 4), kbb = (e >> 6) / (B / 4);
            const int idx = (4 * bq + (ln >> 4)) * FB.ld + 16 * kbb + (ln & 15);  // FB[k_b][beta]
            float* t = fbF + ((bq * (NBB / 2) + kbb / 2) * 64 + ln) * 4 + 2 * (kbb & 1);
            t[0] = FB.re[idx] * scale;
            t[1] = FB.im[idx] * (scale * isign);
        }
        for (int e = tid; e < A * B; e += 512) {        // Tw is T[k_a][beta]: transposed here
            float2 t = Tw[e];
            t.y *= isign;
            tws[(e % B) * A + e / B] = t;
        }
    }

    // ---- geometry --------------------------------------------------------------------------------------
    // tile -> (o, y, column block): tiles are visited first, first + nwg, ..; the position is advanced
    // with carries instead of being divided out of the tile index every time (64-bit divisions in the
    // loop cost more issue slots than the matrix instructions)
    constexpr int TG = CV * CH;                        // 16-column groups per tile
    const int64_t ztt = a.Zt / TG;
    const int64_t per_o = a.Yn * ztt;
    const int64_t ntiles = a.O * per_o;
    const int64_t nwg = (int64_t)gridDim.x * gridDim.y;
    const int64_t first = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
    struct Pos {
        int o, y, zt;                                  // (the host side keeps all three below 2^31)
    };
    const int ztt32 = (int)ztt, yn32 = (int)a.Yn;
    const Pos step = {(int)(nwg / per_o), (int)((nwg % per_o) / ztt), (int)(nwg % ztt)};
    auto advance = [&](Pos& p) {
        p.zt += step.zt;
        if (p.zt >= ztt32) {
            p.zt -= ztt32;
            p.y += 1;
        }
        p.y += step.y;
        if (p.y >= yn32) {
            p.y -= yn32;
            p.o += 1;
        }
        p.o += step.o;
    };
    Pos rq = {(int)(first / per_o), (int)((first % per_o) / ztt), (int)(first % ztt)};   // tile of the slot requested next
    Pos st = rq;                                                                          // tile being accumulated
    const int64_t inN = a.inN, outN = a.outN;
    // stage-1 unit of this wave: beta = SB*slot + ub, column group ug
    const int ub = wave / CH, ug = wave % CH;
    const unsigned ld_lane = (unsigned)(B * lq) * (unsigned)inN + (unsigned)(16 * CV * ug + CV * l16);
    const unsigned st_lane = (unsigned)(A * 4 * lq) * (unsigned)outN + (unsigned)(CV * l16);

    vec xs[2][NS1];                                    // two register sets: slots alternate
    const int64_t in_step = (int64_t)(4 * B) * inN;     // rows between the k-steps of stage 1
    const int64_t out_stepA = (int64_t)A * outN, out_step16A = 16 * out_stepA;
    auto request = [&](int set, int slot) {            // of the tile at rq
        const float2* src = X + ((int64_t)rq.o * a.inO + (int64_t)rq.y * a.inY + (int64_t)rq.zt * (16 * TG)) +
                            (int64_t)(SB * slot + ub) * inN;
#pragma unroll
        for (int s = 0; s < NS1; ++s) {
            xs[set][s] = __builtin_nontemporal_load(reinterpret_cast<const vec*>(&src[ld_lane]));
            src += in_step;
        }
    };

    // stage-2 accumulators of this wave: pair j = (k_a, column group) of p = wave + NW*j
    f32x4 wr[PPW][CV][NBB], wi[PPW][CV][NBB];
    auto clear_acc = [&]() {
#pragma unroll
        for (int j = 0; j < PPW; ++j)
#pragma unroll
            for (int h = 0; h < CV; ++h)
#pragma unroll
                for (int kbb = 0; kbb < NBB; ++kbb) {
                    wr[j][h][kbb] = f32x4{0.f, 0.f, 0.f, 0.f};
                    wi[j][h][kbb] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
    };

    // ---- one barrier interval: stage 2 of slot g interleaved with stage 1 of slot g + 1 ----------------
    // The two are independent (different accumulators, different ring buffers), and each alone leaves
    // the matrix pipe idle while it waits for LDS operands (stage 1: twelve MFMAs per operand read, then
    // the twiddles and the ring writes without any).  So they are issued as one stream: a group of
    // stage-2 MFMAs, then the stage-1 group whose operands were requested one group earlier, and so on;
    // sched_barrier keeps the compiler from undoing the order.
    constexpr int G1 = NAB * (NS1 / 4);                // stage-1 groups: 12 * CV MFMAs each
    constexpr int G2 = KS * NBB;                       // stage-2 groups: 4 * PPW * CV MFMAs each
    static_assert(G2 >= G1 + 2, "enough stage-2 groups to interleave stage 1 and its tail");
    auto interval = [&](int set, int slot2, int buf2, int slot1, int buf1) {      // set: compile-time constant
        // stage 1 state
        f32x4 p1[NAB][CV], p2[NAB][CV], p3[NAB][CV];
#pragma unroll
        for (int ab = 0; ab < NAB; ++ab)
#pragma unroll
            for (int h = 0; h < CV; ++h) {
                p1[ab][h] = f32x4{0.f, 0.f, 0.f, 0.f};
                p2[ab][h] = f32x4{0.f, 0.f, 0.f, 0.f};
                p3[ab][h] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        f32x4 fr, fi, fs;                              // stage-1 operands of the next group
        auto read_fa = [&](int g1) {
            const int sq = g1 / NAB, ab = g1 % NAB;
            const f32x4* t = faT + ((ab * (NS1 / 4) + sq) * 3) * 64 + lane;
            fr = t[0], fi = t[64], fs = t[128];
        };
        auto group1 = [&](int g1) {
            const int sq = g1 / NAB, ab = g1 % NAB;
            const f32x4 r = fr, i = fi, q = fs;
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                const vec x = xs[set][4 * sq + s4];
#pragma unroll
                for (int h = 0; h < CV; ++h) {
                    p1[ab][h] = mfma(r[s4], x[2 * h], p1[ab][h]);
                    p2[ab][h] = mfma(i[s4], x[2 * h + 1], p2[ab][h]);
                    p3[ab][h] = mfma(q[s4], x[2 * h] + x[2 * h + 1], p3[ab][h]);
                }
            }
        };
        const int beta = SB * slot1 + ub;
        f32x4 tq[NAB][2];                              // twiddles of this lane's k_a: 32 contiguous bytes of T[beta][k_a] per block
        auto read_tw = [&]() {
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab) {
                const f32x4* t = reinterpret_cast<const f32x4*>(tws + beta * A + 16 * ab + 4 * lq);
                tq[ab][0] = t[0];
                tq[ab][1] = t[1];
            }
        };
        vec* zw = Zs + (size_t)buf1 * (A * PK) + (ug * SB + ub) * 16 + l16;
        auto tail1 = [&](int ab) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int ka = 16 * ab + 4 * lq + v;
                const float tx = tq[ab][v / 2][2 * (v & 1)], ty = tq[ab][v / 2][2 * (v & 1) + 1];
                vec z;
#pragma unroll
                for (int h = 0; h < CV; ++h) {
                    const float re = p1[ab][h][v] - p2[ab][h][v];
                    const float im = p3[ab][h][v] - p1[ab][h][v] - p2[ab][h][v];
                    z[2 * h] = re * tx - im * ty;
                    z[2 * h + 1] = re * ty + im * tx;
                }
                zw[ka * PK] = z;
            }
        };
        // stage 2 state
        const vec* zr = Zs + (size_t)buf2 * (A * PK) + lq * 16 + l16;
        vec z[PPW];
        float zn[PPW][CV];
        f32x4 fq[NBB / 2];
        auto read_z = [&](int ks) {
#pragma unroll
            for (int j = 0; j < PPW; ++j) {
                const int p = wave + NW * j;
                z[j] = zr[(p / CH) * PK + ((p % CH) * SB + 4 * ks) * 16];
            }
            const f32x4* t = fbT + (size_t)(slot2 * KS + ks) * (NBB / 2) * 64 + lane;
#pragma unroll
            for (int q = 0; q < NBB / 2; ++q) fq[q] = t[q * 64];
        };
        auto group2 = [&](int g2) {
            const int kbb = g2 % NBB;
            if (kbb == 0) {
#pragma unroll
                for (int j = 0; j < PPW; ++j)
#pragma unroll
                    for (int h = 0; h < CV; ++h) zn[j][h] = -z[j][2 * h + 1];
            }
            const float r = fq[kbb / 2][2 * (kbb & 1)], i = fq[kbb / 2][2 * (kbb & 1) + 1];
#pragma unroll
            for (int j = 0; j < PPW; ++j)
#pragma unroll
                for (int h = 0; h < CV; ++h) wr[j][h][kbb] = mfma(r, z[j][2 * h], wr[j][h][kbb]);
#pragma unroll
            for (int j = 0; j < PPW; ++j)
#pragma unroll
                for (int h = 0; h < CV; ++h) wi[j][h][kbb] = mfma(r, z[j][2 * h + 1], wi[j][h][kbb]);
#pragma unroll
            for (int j = 0; j < PPW; ++j)
#pragma unroll
                for (int h = 0; h < CV; ++h) wr[j][h][kbb] = mfma(i, zn[j][h], wr[j][h][kbb]);
#pragma unroll
            for (int j = 0; j < PPW; ++j)
#pragma unroll
                for (int h = 0; h < CV; ++h) wi[j][h][kbb] = mfma(i, z[j][2 * h], wi[j][h][kbb]);
        };

        read_z(0);
        read_fa(0);
        __builtin_amdgcn_sched_barrier(0);
        // groups of stage 2 in order; after group n (n < G1) the stage-1 group n, whose operands were
        // requested before stage-2 group n; then the twiddle reads, and the tail split over NAB groups
#pragma unroll
        for (int g2 = 0; g2 < G2; ++g2) {
            if (g2 % NBB == 0 && g2 > 0) {
                // (the previous k-step's last group has been issued: its operands may be replaced)
                read_z(g2 / NBB);
                __builtin_amdgcn_sched_barrier(0);
            }
            group2(g2);
            __builtin_amdgcn_sched_barrier(0);
            if (g2 < G1) {
                group1(g2);
                if (g2 + 1 < G1) read_fa(g2 + 1);
                else read_tw();
                __builtin_amdgcn_sched_barrier(0);
            } else if (g2 - G1 < NAB) {
                tail1(g2 - G1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    auto store_tile = [&]() {                          // the tile at st
        float2* dst = Y + ((int64_t)st.o * a.outO + (int64_t)st.y * a.outY + (int64_t)st.zt * (16 * TG));
#pragma unroll
        for (int j = 0; j < PPW; ++j) {
            const int p = wave + NW * j;
            const int ka = p / CH, cg = p % CH;
            float2* blk = dst + (int64_t)ka * outN + 16 * CV * cg;       // row k_a, this pair's columns
#pragma unroll
            for (int kbb = 0; kbb < NBB; ++kbb) {
                // rows k_a + A*k_b with k_b = 16*kbb + 4*lq + v: the lq part is in st_lane
                float2* row = blk;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    vec w;
#pragma unroll
                    for (int h = 0; h < CV; ++h) {
                        w[2 * h] = wr[j][h][kbb][v];
                        w[2 * h + 1] = wi[j][h][kbb][v];
                    }
                    __builtin_nontemporal_store(w, reinterpret_cast<vec*>(&row[st_lane]));
                    row += out_stepA;
                }
                blk += out_step16A;
            }
        }
    };

    // Slots are numbered g = 0, 1, .. across the tiles of this workgroup.  One barrier per slot: before
    // it every wave has written slot g into ring buffer g % 2 (stage 1) and finished reading that buffer
    // for slot g - 2; after it, stage 2 of slot g runs interleaved with stage 1 of slot g + 1.
    const int64_t mine = first < ntiles ? (ntiles - first + nwg - 1) / nwg : 0;      // tiles of this workgroup
    const int64_t G = mine * NSLOT;
    // Requests and the stage-1 step past the last slot are not skipped: they re-read the last tile and
    // write a ring buffer nobody reads (every access in bounds).  With unconditional loads the compiler
    // can count how many younger requests may still be in flight when a register set is used; a
    // conditional request made it wait for all of them, the one issued a moment ago included.
    auto request_slot = [&](int set, int64_t g) {      // called with g = 0, 1, 2, .. in this order
        const int slot = (int)(g % NSLOT);
        if (slot == 0 && g != 0 && g < G) advance(rq);
        request(set, slot);
    };
    if (G == 0) return;                            // (whole workgroup, before any barrier)
    clear_acc();
    request_slot(0, 0);
    request_slot(1, 1);
    __syncthreads();                               // tables
    {
        // slot 0 alone: stage 1 with nothing to interleave (a zero-weight stage 2 on the empty ring would
        // need the ring cleared); the same code as in `interval`, without the stage-2 pieces
        f32x4 p1[NAB][CV], p2[NAB][CV], p3[NAB][CV];
#pragma unroll
        for (int ab = 0; ab < NAB; ++ab)
#pragma unroll
            for (int h = 0; h < CV; ++h) {
                p1[ab][h] = f32x4{0.f, 0.f, 0.f, 0.f};
                p2[ab][h] = f32x4{0.f, 0.f, 0.f, 0.f};
                p3[ab][h] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
        for (int sq = 0; sq < NS1 / 4; ++sq)
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab) {
                const f32x4* t = faT + ((ab * (NS1 / 4) + sq) * 3) * 64 + lane;
                const f32x4 fr = t[0], fi = t[64], fs = t[128];
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4) {
                    const vec x = xs[0][4 * sq + s4];
#pragma unroll
                    for (int h = 0; h < CV; ++h) {
                        p1[ab][h] = mfma(fr[s4], x[2 * h], p1[ab][h]);
                        p2[ab][h] = mfma(fi[s4], x[2 * h + 1], p2[ab][h]);
                        p3[ab][h] = mfma(fs[s4], x[2 * h] + x[2 * h + 1], p3[ab][h]);
                    }
                }
            }
        vec* zw = Zs + (ug * SB + ub) * 16 + l16;
#pragma unroll
        for (int ab = 0; ab < NAB; ++ab) {
            const f32x4* t = reinterpret_cast<const f32x4*>(tws + ub * A + 16 * ab + 4 * lq);
            const f32x4 t01 = t[0], t23 = t[1];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int ka = 16 * ab + 4 * lq + v;
                const float tx = (v < 2 ? t01 : t23)[2 * (v & 1)], ty = (v < 2 ? t01 : t23)[2 * (v & 1) + 1];
                vec z;
#pragma unroll
                for (int h = 0; h < CV; ++h) {
                    const float re = p1[ab][h][v] - p2[ab][h][v];
                    const float im = p3[ab][h][v] - p1[ab][h][v] - p2[ab][h][v];
                    z[2 * h] = re * tx - im * ty;
                    z[2 * h + 1] = re * ty + im * tx;
                }
                zw[ka * PK] = z;
            }
        }
        request_slot(0, 2);
    }
    auto body = [&](int set, int64_t g) {          // set: register set of slot g + 1
        __syncthreads();
        const int64_t g1 = g + 1;
        interval(set, (int)(g % NSLOT), (int)(g & 1), (int)(g1 % NSLOT), (int)(g1 & 1));
        request_slot(set, g1 + 2);
        if (g % NSLOT == NSLOT - 1) {
            store_tile();
            clear_acc();
            advance(st);
        }
    };
    for (int64_t g = 0; g < G; g += 2) {
        body(1, g);
        body(0, g + 1);
    }
}

// ---- strided contraction with a small square matrix ----------------------------------------------
// out[o, k, i] = scale * tw * sum_n M[k, n] in[o, n, i] for NK x NK matrices, NK = 16, 32 or 64 (the
// single stages of the FFT formulation when an axis has no fused kernel, and small KDFT modes).
// Such a pass moves 16 bytes per 8*NK flop: it is bound by HBM, so the kernel is built to stream.
// ONE wavefront owns a tile of all NK rows x 16 contiguous columns: the rows are the MFMA B operand
// straight from global memory (16 lanes = one 128-byte segment), the matrix is the A operand read
// from LDS (filled once per workgroup, never written again: no barrier in the loop), and the
// accumulator rows are stored straight to global memory.  Two register sets alternate so the next
// tile's loads are in flight during the current tile.  Three real products per complex product.
template <int NK, int CT, int MINW>
__global__ __launch_bounds__(256, MINW) void k_contract_sr(ContractArgs a, int64_t ntiles)
{
    constexpr int NB = NK / 16;      // blocks of k
    constexpr int NS = NK / 4;       // k-steps (over n)
    constexpr int TC = 16 * CT;      // columns per tile: CT groups of 16 (CT x 128 contiguous bytes per row)
    constexpr int P = NK + 16;       // LDS pitch: lane groups 0,1 (and 2,3) of a read fall on disjoint halves of the banks
    __shared__ float mr[NK * P], mi[NK * P];      // [n][k]: re, im (scale and conjugation applied)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int l16 = lane & 15, lq = lane >> 4;
    const float isign = a.conj ? -1.0f : 1.0f;
    for (int e = tid; e < NK * NK; e += 256) {
        const int n = e / NK, k = e % NK;
        const float r = a.M.re[(int64_t)n * a.M.ld + k] * a.scale;
        const float i = a.M.im[(int64_t)n * a.M.ld + k] * (a.scale * isign);
        mr[n * P + k] = r;
        mi[n * P + k] = i;
    }
    __syncthreads();

    // tile indices are wave-uniform 32-bit numbers (the host checks the count): the index
    // arithmetic, divisions included, stays cheap
    const unsigned wave = (blockIdx.x * 4u) + (unsigned)__builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned nwaves = gridDim.x * 4u;
    if (wave >= ntiles) return;                   // after the only barrier

    const int64_t I = a.I;
    const unsigned ctiles = (unsigned)(I / TC);   // column tiles per o
    const unsigned olo = (unsigned)a.Olo;
    const int m_rd = lq * P + l16;                // + 4*s*P + 16*kb

    auto load_tile = [&](f32x2 (&x)[CT][NS], unsigned tile) {
        const unsigned o = tile / ctiles, c0 = (tile - o * ctiles) * TC;
        const f32x2* src = reinterpret_cast<const f32x2*>(a.X) + (int64_t)o * NK * I + c0 + l16 + (int64_t)lq * I;
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int g = 0; g < CT; ++g) x[g][s] = stream_load(&src[(int64_t)(4 * s) * I + 16 * g]);
    };
    auto transform_tile = [&](const f32x2 (&x)[CT][NS], unsigned tile) {
        f32x4 p1[CT][NB], p2[CT][NB], p3[CT][NB];
#pragma unroll
        for (int g = 0; g < CT; ++g)
#pragma unroll
            for (int kb = 0; kb < NB; ++kb) {
                p1[g][kb] = f32x4{0.f, 0.f, 0.f, 0.f};
                p2[g][kb] = f32x4{0.f, 0.f, 0.f, 0.f};
                p3[g][kb] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            float fr[NB], fi[NB], fs[NB];
#pragma unroll
            for (int kb = 0; kb < NB; ++kb) {
                fr[kb] = mr[m_rd + 4 * s * P + 16 * kb];
                fi[kb] = mi[m_rd + 4 * s * P + 16 * kb];
                fs[kb] = fr[kb] + fi[kb];
            }
#pragma unroll
            for (int g = 0; g < CT; ++g) {
                const float xs = x[g][s].x + x[g][s].y;
#pragma unroll
                for (int kb = 0; kb < NB; ++kb) {
                    p1[g][kb] = mfma(fr[kb], x[g][s].x, p1[g][kb]);
                    p2[g][kb] = mfma(fi[kb], x[g][s].y, p2[g][kb]);
                    p3[g][kb] = mfma(fs[kb], xs, p3[g][kb]);
                }
            }
        }
        const unsigned o = tile / ctiles, c0 = (tile - o * ctiles) * TC;
        const unsigned ohi = o / olo;
        const int64_t col = (int64_t)c0 + l16;
        f32x2* dst = reinterpret_cast<f32x2*>(a.Y) + (int64_t)ohi * a.sYohi + (int64_t)(o - ohi * olo) * a.sYolo + col;
        const int beta = a.Tw ? (int)((uint32_t)c0 / (uint32_t)a.twInner) : 0;     // uniform: twInner is a multiple of TC
#pragma unroll
        for (int kb = 0; kb < NB; ++kb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int k = 16 * kb + 4 * lq + v;
                float2 w = make_float2(1.f, 0.f);
                if (a.Tw) {
                    w = a.Tw[(int64_t)k * a.twB + beta];
                    w.y *= isign;
                }
#pragma unroll
                for (int g = 0; g < CT; ++g) {
                    float yr = p1[g][kb][v] - p2[g][kb][v];
                    float yi = p3[g][kb][v] - p1[g][kb][v] - p2[g][kb][v];
                    if (a.Tw) {
                        const float tr = yr * w.x - yi * w.y;
                        yi = yr * w.y + yi * w.x;
                        yr = tr;
                    }
                    stream_store(&dst[(int64_t)k * a.sYk + 16 * g], f32x2{yr, yi});
                }
            }
    };

    f32x2 xa[CT][NS], xb[CT][NS];
    load_tile(xa, wave);
    const unsigned nt = (unsigned)ntiles;
    for (unsigned tile = wave; tile < nt; tile += 2 * nwaves) {
        // a request past the end re-reads the wave's current tile (in bounds, never used)
        const unsigned t1 = tile + nwaves, t2 = tile + 2 * nwaves;
        load_tile(xb, t1 < nt ? t1 : tile);
        __builtin_amdgcn_sched_barrier(0);
        transform_tile(xa, tile);
        __builtin_amdgcn_sched_barrier(0);
        if (t1 >= nt) break;
        load_tile(xa, t2 < nt ? t2 : tile);
        __builtin_amdgcn_sched_barrier(0);
        transform_tile(xb, t1);
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int NK, int CT, int MINW>
hipError_t launch_csr_inst(const ContractArgs& a, hipStream_t stream)
{
    const int64_t ntiles = a.O * (a.I / (16 * CT));
    const int64_t resident = 256 * MINW;                 // workgroups of 4 waves, MINW waves per SIMD
    const int64_t want = (ntiles + 3) / 4;
    const int64_t blocks = want < resident ? want : resident;
    hipLaunchKernelGGL((k_contract_sr<NK, CT, MINW>), dim3((unsigned)blocks), dim3(256), 0, stream, a, ntiles);
    return hipGetLastError();
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

template <int A, int B, int CV, int CH, int SB>
hipError_t launch_ss_inst(const FftStridedArgs& a, const DeviceMatrix& FA, const DeviceMatrix& FB, const float2* Tw,
                          float scale, int conj, hipStream_t stream)
{
    typedef FftSsLayout<A, B, CV, CH, SB> L;
    const int64_t ntiles = a.O * a.Yn * (a.Zt / (CV * CH));
    const int64_t blocks = ntiles < 256 ? ntiles : 256;          // one persistent workgroup per CU
    hipLaunchKernelGGL((k_fft_ss<A, B, CV, CH, SB>), dim3((unsigned)blocks), dim3(512), L::lds_bytes, stream, a, FA, FB,
                       Tw, scale, conj);
    return hipGetLastError();
}

template <int A, int B, int MINW>
hipError_t launch_s_inst(const FftStridedArgs& a, const DeviceMatrix& FA, const DeviceMatrix& FB, const float2* Tw,
                         float scale, int conj, hipStream_t stream)
{
    const int64_t ntiles = a.O * a.Yn * a.Zt;
    const int64_t resident = 256 * MINW;           // persistent workgroups: MINW per CU
    const int64_t blocks = ntiles < resident ? ntiles : resident;
    hipLaunchKernelGGL((k_fft_sr<A, B, MINW>), dim3((unsigned)blocks), dim3(256), 0, stream, a, FA, FB, Tw, scale,
                       conj);
    return hipGetLastError();
}

}  // namespace

bool contract_sr_supported(const ContractArgs& a)
{
    const int N = a.M.N;
    if (a.M.K != N || (N != 16 && N != 32 && N != 64)) return false;
    if (a.I < 16 || a.I % 16 != 0 || a.three_m || a.bf16x3) return false;
    if (a.Tw && a.twInner % 16 != 0) return false;       // one twiddle column per tile
    // 32-bit tile arithmetic in the kernel, with room for the two-tile look-ahead of 2 * 12288 waves
    if (a.O >= (int64_t(1) << 30) || a.Olo >= (int64_t(1) << 30) || a.O * (a.I / 16) >= (int64_t(1) << 31) - 65536)
        return false;
    return true;
}

hipError_t launch_contract_sr(const ContractArgs& a, hipStream_t stream)
{
    if (!contract_sr_supported(a)) return hipErrorInvalidValue;
    // widest tile (CT groups of 16 columns) that divides the inner extent and, with a twiddle, stays
    // inside one twiddle column
    auto fits = [&](int ct) { return a.I % (16 * ct) == 0 && (!a.Tw || a.twInner % (16 * ct) == 0); };
    if (a.M.N == 16) {
        if (fits(4)) return launch_csr_inst<16, 4, 3>(a, stream);
        if (fits(2)) return launch_csr_inst<16, 2, 4>(a, stream);
        return launch_csr_inst<16, 1, 8>(a, stream);
    }
    if (a.M.N == 32) {
        if (fits(2)) return launch_csr_inst<32, 2, 3>(a, stream);
        return launch_csr_inst<32, 1, 4>(a, stream);
    }
    return launch_csr_inst<64, 1, 2>(a, stream);
}

hipError_t configure_fft_kernels()
{
    hipError_t e = hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_fft_ss<32, 64, 1, 1, 8>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)FftSsLayout<32, 64, 1, 1, 8>::lds_bytes);
    if (e != hipSuccess) return e;
    return configure_fft_nested_kernels();
}

bool fft_sr_supported(int A, int B, int64_t I)
{
    // 32-bit lane offsets inside the kernels: up to 12*A rows (and 3*B rows) of I elements
    if (I % 16 != 0) return false;
    if (fft_sn_supported(A, B, I)) return true;
    if (A == 32 && B == 64) return I <= (int64_t(1) << 23);
    return I <= (int64_t(1) << 21) && A == 16 && B == 16;
}

hipError_t launch_fft_sr_ex(const FftStridedArgs& a, int A, int B, const DeviceMatrix& FA,
                            const DeviceMatrix& FB, const float2* Tw, float scale, int conj, hipStream_t stream)
{
    if (a.O <= 0 || a.Yn <= 0 || a.Zt <= 0) return hipSuccess;
    if (fft_sn_supported(A, B, 16)) return launch_fft_sn(a, A, B, FA, FB, Tw, scale, conj, stream);
    const int64_t lim = int64_t(1) << ((A == 32 && B == 64) ? 23 : 21);
    if (a.inN < 16 || a.outN < 16 || a.inN > lim || a.outN > lim || FA.K != A || FA.N != A || FB.K != B ||
        FB.N != B || !Tw)
        return hipErrorInvalidValue;
    if (A == 32 && B == 64) return launch_ss_inst<32, 64, 1, 1, 8>(a, FA, FB, Tw, scale, conj, stream);
    if (A == 16 && B == 16) return launch_s_inst<16, 16, 4>(a, FA, FB, Tw, scale, conj, stream);
    return hipErrorInvalidValue;
}

hipError_t launch_fft_sr(const float2* in, float2* out, int64_t O, int64_t I, int A, int B,
                         const DeviceMatrix& FA, const DeviceMatrix& FB, const float2* Tw, float scale,
                         int conj, hipStream_t stream)
{
    if (O <= 0 || I <= 0) return hipSuccess;
    if (!fft_sr_supported(A, B, I)) return hipErrorInvalidValue;
    // contiguous [O][A*B][I] on both sides
    FftStridedArgs a{};
    a.X = in;
    a.Y = out;
    a.O = O;
    a.Yn = 1;
    a.Zt = I / 16;
    a.inO = a.outO = (int64_t)A * B * I;
    a.inN = a.outN = I;
    a.inY = a.outY = 0;
    return launch_fft_sr_ex(a, A, B, FA, FB, Tw, scale, conj, stream);
}

bool fft_zr_supported(int A, int B)
{
    return (A == 16 && B == 16) || (A == 32 && B == 32) || (A == 32 && B == 64);
}

hipError_t launch_fft_zr(const float2* in, float2* out, int64_t nrows, int A, int B, const DeviceMatrix& FA,
                         const DeviceMatrix& FB, const float2* Tw, float scale, int conj, hipStream_t stream)
{
    if (nrows <= 0) return hipSuccess;
    // the kernel indexes the stage matrices and the twiddle table without bounds checks
    if (FA.K != A || FA.N != A || FB.K != B || FB.N != B || !Tw) return hipErrorInvalidValue;
    // three-product scheme where its registers allow; 32 x 32 would spill with it and runs the
    // four-product scheme
    if (A == 16 && B == 16) return launch_inst<16, 16, 6, true>(in, out, nrows, FA, FB, Tw, scale, conj, stream);
    if (A == 32 && B == 32) return launch_inst<32, 32, 2, false>(in, out, nrows, FA, FB, Tw, scale, conj, stream);
    if (A == 32 && B == 64) {
        // eight waves per workgroup, one workgroup per CU
        const int64_t want = (nrows + 7) / 8;
        const int64_t blocks = want < 256 ? want : 256;
        hipLaunchKernelGGL((k_fft_zl<32, 64>), dim3((unsigned)blocks), dim3(512), 0, stream, in, out, nrows, FA, FB, Tw,
                           scale, conj);
        return hipGetLastError();
    }
    return hipErrorInvalidValue;
}

}  // namespace dft3d
