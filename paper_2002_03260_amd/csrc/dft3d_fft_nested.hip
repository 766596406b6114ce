// FFT formulation with the second factor split once more: N = A * B with A = 16 and B = C * 16, C = 2, 4
// or 8 (512 = 16 * 32, 1024 = 16 * 64, 2048 = 16 * 128), or A = 32 and B = 4 * 16 (2048 = 32 * 64).
//
// Eq. 13 - 16 for one axis with n = B*l + b, k = k_a + A*k2 read
//     Z[k_a, b]  = T[k_a, b] * sum_l FA[k_a, l] x[B*l + b]
//     X[k_a + A*k2] = sum_b FB[k2, b] Z[k_a, b]
// and cost 6 * (A + B) matrix-core flop per point.  The B-point transform of the second line is a
// DFT like the whole one, so the same split applies to it: b = 16*c + beta, k2 = k_c + C*k_b gives
//     FB[k2, b] = w_C^(c k_c) * w_B^(k_c beta) * F16[k_b, beta]
//     Y[k_a, k_c, beta] = w_B^(k_c beta) * sum_c w_C^(c k_c) Z[k_a, 16*c + beta]      (C-point butterflies)
//     X[k_a + A*(k_c + C*k_b)] = sum_beta F16[k_b, beta] Y[k_a, k_c, beta]
// The last matrix stage is 16-point now (6 * (A + 16) flop per point on the matrix cores: a third of the
// plain 32 x 64 split at N = 2048 with A = 16, less than half with A = 32) and the C-point stage in the
// middle is plain vector arithmetic on values a lane already holds.  Every table the kernels need is part
// of the plan of an A x B split: FA is its first-stage matrix, T its twiddle table,
// w_B^(k_c beta) = FB[k_c, beta] and F16[k_b, beta] = FB[C*k_b, beta].
//
// Longer axes (4096, 8192, 16384 points) put a first factor of 2, 4 or 8 in front: its stage is butterflies
// and a twiddle in one element-wise pass (k_radix_tw, at the end of this file) and its second stage is one
// of the transforms above.
//
// BACKWARD runs the forward transform on data with real and imaginary parts exchanged, and exchanges
// them again in the result: with s(z) = i * conj(z), DFT(s(x)) = s(IDFT(x)).  The exchange is a choice
// of register names, so the inverse costs exactly what the forward transform costs.
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

// In-place C-point forward DFT (w = exp(-2 pi i / C)) of C complex values held as separate real and
// imaginary parts; T is float or a vector of floats (element-wise).  Output k at index k.
template <int C, typename T>
__device__ __forceinline__ void small_dft(T (&r)[C], T (&i)[C])
{
    static_assert(C == 1 || C == 2 || C == 4 || C == 8, "radix");
    if constexpr (C == 2) {
        const T r0 = r[0] + r[1], i0 = i[0] + i[1], r1 = r[0] - r[1], i1 = i[0] - i[1];
        r[0] = r0, i[0] = i0, r[1] = r1, i[1] = i1;
    } else if constexpr (C == 4) {
        const T t0r = r[0] + r[2], t0i = i[0] + i[2], t1r = r[0] - r[2], t1i = i[0] - i[2];
        const T t2r = r[1] + r[3], t2i = i[1] + i[3], t3r = r[1] - r[3], t3i = i[1] - i[3];
        r[0] = t0r + t2r, i[0] = t0i + t2i;
        r[2] = t0r - t2r, i[2] = t0i - t2i;
        r[1] = t1r + t3i, i[1] = t1i - t3r;        // t1 + (-i) t3
        r[3] = t1r - t3i, i[3] = t1i + t3r;
    } else if constexpr (C == 8) {
        T er[4] = {r[0], r[2], r[4], r[6]}, ei[4] = {i[0], i[2], i[4], i[6]};
        T orr[4] = {r[1], r[3], r[5], r[7]}, oi[4] = {i[1], i[3], i[5], i[7]};
        small_dft<4>(er, ei);
        small_dft<4>(orr, oi);
        constexpr float h = 0.70710678118654752440f;
        // w^k o[k]:  w^1 = (1 - i) h,  w^2 = -i,  w^3 = (-1 - i) h
        const T p0r = orr[0], p0i = oi[0];
        const T p1r = (orr[1] + oi[1]) * h, p1i = (oi[1] - orr[1]) * h;
        const T p2r = oi[2], p2i = -orr[2];
        const T p3r = (oi[3] - orr[3]) * h, p3i = -(orr[3] + oi[3]) * h;
        r[0] = er[0] + p0r, i[0] = ei[0] + p0i, r[4] = er[0] - p0r, i[4] = ei[0] - p0i;
        r[1] = er[1] + p1r, i[1] = ei[1] + p1i, r[5] = er[1] - p1r, i[5] = ei[1] - p1i;
        r[2] = er[2] + p2r, i[2] = ei[2] + p2i, r[6] = er[2] - p2r, i[6] = ei[2] - p2i;
        r[3] = er[3] + p3r, i[3] = ei[3] + p3i, r[7] = er[3] - p3r, i[7] = ei[3] - p3i;
    }
}

// ---- contiguous axis -------------------------------------------------------------------------------
// ONE wavefront transforms one row of N points in registers, with no barrier in the row loop; the
// operand layouts of v_mfma_f32_16x16x4_f32 do the transposition between the two matrix stages:
//   stage 1, transposed:  D[beta, k_a] = sum_l x[B*l + 16*c + beta] F16[l, k_a]  for each c,
//     A operand = data straight from global memory (lane: beta = lane % 16, l = 4*s + lane / 16),
//     D register v of a lane = (beta = 4*(lane/16) + v, k_a = lane % 16); twiddle on D;
//   C-point butterflies across the C accumulators of a lane, then w_B^(k_c beta);
//   stage 3:  D[k_b, k_a] = sum_beta F16[k_b, beta] Y[k_a, k_c, beta] for each k_c: register v of the
//     butterfly output is the B operand of k-step v as it stands (lane group g stands for
//     beta = 4*g + v; a sum does not care about the order of its terms), the A operand is F16 loaded
//     once in that order.  D register v = (k_b = 4*(lane/16) + v, k_a = lane % 16): the output index
//     k_a + 16*k_c + 16*C*k_b runs along the lanes, so loads and stores are 128-byte segments.
// Three real products per complex product in both matrix stages: 24 * C matrix instructions per row.
// NAB = A / 16: first stage of 16 or 32 points (32 x (C*16): two blocks of k_a, eight k-steps).
template <int NAB, int C, bool SWAP, int WPC>
__global__ __launch_bounds__(256, WPC) void k_fft_zn(const float2* __restrict__ in, float2* __restrict__ out,
                                                    int64_t nrows, DeviceMatrix FA, DeviceMatrix FB,
                                                    const float2* __restrict__ Tw, float scale)
{
    constexpr int A = 16 * NAB, NS1 = A / 4, B = 16 * C, N = A * B;
    __shared__ float2 tw1s[C * NAB * 4 * 64];    // [c][ab][v][lane]: T[k_a = 16*ab + lane%16][16*c + 4*(lane/16) + v]
    __shared__ __align__(16) float2 tw2s[C * 16];         // [k_c][beta]: w_B^(k_c beta)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int l16 = lane & 15, lq = lane >> 4;

    for (int e = tid; e < C * NAB * 4 * 64; e += 256) {
        const int ln = e & 63, v = (e >> 6) & 3, ab = (e >> 8) % NAB, c = (e >> 8) / NAB;
        tw1s[e] = Tw[(16 * ab + (ln & 15)) * B + 16 * c + 4 * (ln >> 4) + v];
    }
    for (int e = tid; e < C * 16; e += 256) {
        const int beta = e & 15, kc = e >> 4;
        tw2s[e] = make_float2(FB.re[beta * FB.ld + kc], FB.im[beta * FB.ld + kc]);    // FB[k][n] at plane[n * ld + k]
    }
    __syncthreads();

    // (wave-uniform, and told so: row addresses are then a scalar base plus a 32-bit lane offset)
    const int64_t wave = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    if (wave >= nrows) return;                    // after the only barrier

    // stage-1 B operand FA[k_a = 16*ab + l16][l = 4*s + lq]; stage-3 A operand scale * F16[k_b = l16][beta = 4*lq + v]
    // with F16[k_b, beta] = w_16^(k_b beta) = FB[C*k_b, beta]
    float fa_r[NAB][NS1], fa_i[NAB][NS1], fa_s[NAB][NS1], fb_r[4], fb_i[4], fb_s[4];
#pragma unroll
    for (int ab = 0; ab < NAB; ++ab)
#pragma unroll
        for (int s = 0; s < NS1; ++s) {
            const int ia = (4 * s + lq) * FA.ld + 16 * ab + l16;
            fa_r[ab][s] = FA.re[ia];
            fa_i[ab][s] = FA.im[ia];
            fa_s[ab][s] = fa_r[ab][s] + fa_i[ab][s];
        }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int ib = (4 * lq + v) * FB.ld + C * l16;
        fb_r[v] = FB.re[ib] * scale;
        fb_i[v] = FB.im[ib] * scale;
        fb_s[v] = fb_r[v] + fb_i[v];
    }

    const unsigned ld_off = B * lq + l16;         // + 4*B*s + 16*c
    const unsigned st_off = l16 + A * C * 4 * lq;      // + 16*ab + A*k_c + A*C*v
    f32x2 x[C][NS1];
    auto load_block = [&](int64_t row, int c) {
        const f32x2* src = reinterpret_cast<const f32x2*>(in) + row * N + 16 * c;
#pragma unroll
        for (int s = 0; s < NS1; ++s) x[c][s] = __builtin_nontemporal_load(&(src + 4 * B * s)[ld_off]);
    };
#pragma unroll
    for (int c = 0; c < C; ++c) load_block(wave, c);

    // Order of the memory instructions of a row: the requests for the wave's NEXT row (each block as soon
    // as the first stage has consumed it), then the stores of this row.  The counter a wave waits on
    // retires loads and stores in issue order, so data that was requested before the stores can be waited
    // for without waiting for a single store; requested after them (where more registers would be free)
    // every row would begin with the wave idle until all its stores had been acknowledged by memory.
    auto transform_row = [&](int64_t row) {
        const int64_t next = row + nwaves < nrows ? row + nwaves : row;    // past the end: a harmless re-read
        // the tables are loop invariant, but keeping them in registers across rows is exactly what does
        // not fit: make the compiler read them again in every row
        asm volatile("" ::: "memory");
        f32x4 zr[NAB][C], zi[NAB][C];
#pragma unroll
        for (int c = 0; c < C; ++c) {
            f32x4 p1[NAB], p2[NAB], p3[NAB];
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab) {
                p1[ab] = f32x4{0.f, 0.f, 0.f, 0.f};
                p2[ab] = p1[ab];
                p3[ab] = p1[ab];
            }
#pragma unroll
            for (int s = 0; s < NS1; ++s) {
                const float xr = SWAP ? x[c][s].y : x[c][s].x, xi = SWAP ? x[c][s].x : x[c][s].y;
#pragma unroll
                for (int ab = 0; ab < NAB; ++ab) {
                    p1[ab] = mfma(xr, fa_r[ab][s], p1[ab]);
                    p2[ab] = mfma(xi, fa_i[ab][s], p2[ab]);
                    p3[ab] = mfma(xr + xi, fa_s[ab][s], p3[ab]);
                }
            }
            load_block(next, c);
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float2 t = tw1s[((c * NAB + ab) * 4 + v) * 64 + lane];
                    const float a = p1[ab][v] - p2[ab][v], b = p3[ab][v] - p1[ab][v] - p2[ab][v];
                    zr[ab][c][v] = a * t.x - b * t.y;
                    zi[ab][c][v] = a * t.y + b * t.x;
                }
            __builtin_amdgcn_sched_barrier(0);     // keeps the requests where they are
        }
#pragma unroll
        for (int ab = 0; ab < NAB; ++ab) small_dft<C>(zr[ab], zi[ab]);
#pragma unroll
        for (int kc = 1; kc < C; ++kc) {
            const f32x4* t4 = reinterpret_cast<const f32x4*>(&tw2s[kc * 16 + 4 * lq]);   // four twiddles: beta = 4*lq + v
            const f32x4 t01 = t4[0], t23 = t4[1];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float tx = (v < 2 ? t01 : t23)[2 * (v & 1)], ty = (v < 2 ? t01 : t23)[2 * (v & 1) + 1];
#pragma unroll
                for (int ab = 0; ab < NAB; ++ab) {
                    const float a = zr[ab][kc][v], b = zi[ab][kc][v];
                    zr[ab][kc][v] = a * tx - b * ty;
                    zi[ab][kc][v] = a * ty + b * tx;
                }
            }
        }
        f32x2* dst = reinterpret_cast<f32x2*>(out) + row * N;
#pragma unroll
        for (int kc = 0; kc < C; ++kc)
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab) {
                f32x4 q1 = {0.f, 0.f, 0.f, 0.f}, q2 = q1, q3 = q1;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    q1 = mfma(fb_r[v], zr[ab][kc][v], q1);
                    q2 = mfma(fb_i[v], zi[ab][kc][v], q2);
                    q3 = mfma(fb_s[v], zr[ab][kc][v] + zi[ab][kc][v], q3);
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float re = q1[v] - q2[v], im = q3[v] - q1[v] - q2[v];
                    __builtin_nontemporal_store(SWAP ? f32x2{im, re} : f32x2{re, im},
                                                &(dst + 16 * ab + A * kc + A * C * v)[st_off]);
                }
            }
    };
    // The first row runs outside the loop so that the loop is entered in the state every iteration leaves
    // behind (requests, then stores): with the prologue's requests as a second way in, the waits at the
    // top of the loop would have to cover that case too and would wait for stores.
    transform_row(wave);
    // (the requests of that first row must stay where they are, in front of its stores: an empty
    // statement that names their registers keeps the compiler from moving them behind the stores into
    // the path that enters the loop)
#pragma unroll
    for (int c = 0; c < C; ++c)
#pragma unroll
        for (int s = 0; s < NS1; ++s) asm volatile("" : "+v"(x[c][s]));
    for (int64_t row = wave + nwaves; row < nrows; row += nwaves) transform_row(row);
}

template <int NAB, int C, int WPC>
hipError_t launch_zn_inst(const float2* in, float2* out, int64_t nrows, const DeviceMatrix& FA, const DeviceMatrix& FB,
                          const float2* Tw, float scale, int conj, hipStream_t stream)
{
    // persistent waves: WPC workgroups of four per CU, fewer when there are fewer rows
    const int64_t want = (nrows + 3) / 4;
    const int64_t blocks = want < 256 * WPC ? want : 256 * WPC;
    if (conj)
        hipLaunchKernelGGL((k_fft_zn<NAB, C, true, WPC>), dim3((unsigned)blocks), dim3(256), 0, stream, in, out, nrows, FA, FB, Tw,
                           scale);
    else
        hipLaunchKernelGGL((k_fft_zn<NAB, C, false, WPC>), dim3((unsigned)blocks), dim3(256), 0, stream, in, out, nrows, FA, FB, Tw,
                           scale);
    return hipGetLastError();
}

// ---- strided axes ------------------------------------------------------------------------------------
// Tensor viewed as [O][N][I]; a tile is all N positions x 16 contiguous columns, the columns being the
// MFMA column index of both matrix stages (data = B operand, 16 lanes = one 128-byte segment).  Between
// two matrix stages with the data as B operand the row index of the first result has to become the
// contraction index of the second, which takes a trip through LDS; and a whole tile of intermediates
// (N * 16 complex numbers, 256 KiB at N = 2048) does not fit there.  So, as in the streaming kernel of
// the plain split, what stays resident is the RESULT: each of the eight waves keeps the accumulators of
// two k_a (all k_c, k_b and columns: 16*C registers of four) and the other stages feed them one slot of
// four beta at a time through a double-buffered LDS ring:
//   producer, wave w = (beta = 4*slot + w / 2, half h = w % 2), for c = h, h + 2, ..:
//       D[k_a, col] = T[k_a, 16*c + beta] * sum_l F16[k_a, l] x[B*l + 16*c + beta, col]
//       (data straight from global memory, requested one slot ahead into the registers the matrix
//       instructions have just read), then the (C/2)-point butterflies over its own c:
//       E_h[m] = sum_c' w_(C/2)^(c' m) D[c = h + 2*c']   ->  ring[h][m][k_a][beta][col]
//   one barrier
//   consumer, wave w, k_a = 2*w, 2*w + 1:  reads E_0[m], E_1[m] at (beta = lane / 16, col = lane % 16),
//       U[m] = E_0[m] + w_C^m E_1[m],  U[m + C/2] = E_0[m] - w_C^m E_1[m]      (the last butterfly level)
//       Y[k_c] = w_B^(k_c beta) U[k_c]
//       W[k_a, k_c][k_b, col] += sum_(beta in slot) F16[k_b, beta] Y[k_c][beta, col]   (one k-step, four
//       real products: two accumulators per output, which is what fits)
//   after the fourth slot the accumulators are stored to rows k_a + 16*k_c + 16*C*k_b and cleared.
// Matrix-core work per point: 6*16 (first stage) + 8*16 (last stage) flop, against 6*32 + 8*64 of the
// streaming kernel for 32 x 64.  One workgroup of eight waves per CU at C = 8.
// NAB = A / 16: first stage of 16 or 32 points (32 x (C*16): two blocks of k_a, eight k-steps; a wave then
// keeps the accumulators of four k_a).
template <int NAB, int C, int CH>
struct FftSnLayout {
    static constexpr int A = 16 * NAB, NS1 = A / 4, B = 16 * C, N = A * B, CP = C / 2;
    static constexpr int KP = 64 * CH;                                         // elements per (h, m, k_a): [column group][beta 4][col 16]
    static constexpr size_t ring_elems = (size_t)2 * CP * A * KP;             // one buffer: [h][m][k_a][column group][beta][col]
    static constexpr size_t ring_bytes = 2 * ring_elems * 8;
    static constexpr size_t fa_bytes = (size_t)NAB * (NS1 / 4) * 3 * 64 * 16;  // [ab][4 k-steps][re, im, re+im][lane] x (4 k-steps)
    static constexpr size_t tw1_bytes = (size_t)B * A * 8;                     // T[b][k_a]
    static constexpr size_t tw2_bytes = (size_t)16 * C * 8;                    // w_B^(k_c beta) as [beta][k_c]
    static constexpr size_t fb_bytes = 4 * 64 * 8;                             // [slot][lane] x (re, im)
    static constexpr size_t lds_bytes = ring_bytes + fa_bytes + tw1_bytes + tw2_bytes + fb_bytes;
    static_assert(lds_bytes <= 160 * 1024, "LDS of one CU");
};

template <int NAB, int C, int CH, bool SWAP, int WPC>
__global__ __launch_bounds__(512, 2 * WPC) void k_fft_sn(FftStridedArgs a, DeviceMatrix FA, DeviceMatrix FB,
                                                      const float2* __restrict__ Tw, float scale)
{
    typedef FftSnLayout<NAB, C, CH> L;
    constexpr int A = L::A, NS1 = L::NS1, B = L::B, CP = L::CP, KP = L::KP;
    constexpr int KW = A / 8;                          // k_a per wave
    static_assert(C == 2 || C == 4 || C == 8, "second factor 32, 64 or 128");

    extern __shared__ __align__(16) unsigned char smem_sn[];
    f32x2* ring = reinterpret_cast<f32x2*>(smem_sn);
    f32x4* faT = reinterpret_cast<f32x4*>(smem_sn + L::ring_bytes);
    float2* tw1 = reinterpret_cast<float2*>(smem_sn + L::ring_bytes + L::fa_bytes);
    float2* tw2 = reinterpret_cast<float2*>(smem_sn + L::ring_bytes + L::fa_bytes + L::tw1_bytes);
    f32x2* fbT = reinterpret_cast<f32x2*>(smem_sn + L::ring_bytes + L::fa_bytes + L::tw1_bytes + L::tw2_bytes);

    const float2* __restrict__ X = a.X;
    float2* __restrict__ Y = a.Y;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lq = lane >> 4;

    // ---- tables, once per workgroup ------------------------------------------------------------------
    {
        float* faF = reinterpret_cast<float*>(faT);
        for (int e = tid; e < NAB * NS1 * 64; e += 512) {
            const int ln = e & 63, s = (e >> 6) % NS1, ab = (e >> 6) / NS1;
            const int idx = (4 * s + (ln >> 4)) * FA.ld + 16 * ab + (ln & 15);   // FA[k_a = 16*ab + ln%16][l = 4*s + ln/16]
            const float r = FA.re[idx], i = FA.im[idx];
            float* t = faF + ((((ab * (NS1 / 4) + s / 4) * 3) * 64 + ln) * 4 + (s & 3));
            t[0] = r;
            t[64 * 4] = i;
            t[128 * 4] = r + i;
        }
        for (int e = tid; e < B * A; e += 512) tw1[(e % B) * A + e / B] = Tw[e];        // Tw is T[k_a][b]: transposed here
        for (int e = tid; e < 16 * C; e += 512) {
            const int kc = e % C, beta = e / C;
            tw2[e] = make_float2(FB.re[beta * FB.ld + kc], FB.im[beta * FB.ld + kc]);   // FB[k][n] at plane[n * ld + k]
        }
        for (int e = tid; e < 4 * 64; e += 512) {
            const int ln = e & 63, t = e >> 6;
            // F16[k_b = ln%16][beta = 4*t + ln/16] = w_16^(k_b beta) = FB[C*k_b, beta]
            const int idx = (4 * t + (ln >> 4)) * FB.ld + C * (ln & 15);
            fbT[e] = f32x2{FB.re[idx] * scale, FB.im[idx] * scale};
        }
    }

    // ---- geometry --------------------------------------------------------------------------------------
    // tile -> (o, y, column block): tiles are visited first, first + nwg, ..; the position is advanced with
    // carries instead of being divided out of the tile index every time
    const int64_t ztt = a.Zt / CH;                     // tiles along the columns (the host checks that CH divides Zt)
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
    const int64_t mine = first < ntiles ? (ntiles - first + nwg - 1) / nwg : 0;          // tiles of this workgroup
    const int64_t G = mine * 4;                                                           // slots of this workgroup
    if (G == 0) return;                                // (whole workgroup, before any barrier)

    // producer unit of this wave
    const int pb = wave >> 1, ph = wave & 1;
    const unsigned ld_lane = (unsigned)(B * lq) * (unsigned)inN + (unsigned)l16;
    f32x2 xs[CP][NS1][CH];
    const float2* rsrc = X;                             // base of the slot being requested
    auto request_base = [&](int slot) {                // of the tile at rq
        rsrc = X + ((int64_t)rq.o * a.inO + (int64_t)rq.y * a.inY + (int64_t)rq.zt * (16 * CH)) +
               (int64_t)(4 * slot + pb + 16 * ph) * inN;
    };
    auto request_step = [&](int s) {                   // the registers of k-step s
#pragma unroll
        for (int cp = 0; cp < CP; ++cp)
#pragma unroll
            for (int cg = 0; cg < CH; ++cg)              // neighbouring 128-byte pieces of the same rows
                xs[cp][s][cg] = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(
                    &(rsrc + (int64_t)(4 * B * s + 32 * cp) * inN + 16 * cg)[ld_lane]));
    };
    auto request = [&](int slot) {
        request_base(slot);
#pragma unroll
        for (int s = 0; s < NS1; ++s) request_step(s);
    };
    // Requests past the last slot are not skipped: they re-read the last tile (every access in bounds) and
    // the producer step that uses them writes a ring buffer nobody reads.  With unconditional loads the
    // compiler can count how many younger requests may be in flight when the registers are used.
    auto request_begin = [&](int64_t g) {              // called with g = 0, 1, 2, .. in this order
        const int slot = (int)(g & 3);
        if (slot == 0 && g != 0 && g < G) advance(rq);
        request_base(slot);
    };
    auto request_slot = [&](int64_t g) {
        request_begin(g);
#pragma unroll
        for (int s = 0; s < NS1; ++s) request_step(s);
    };

    // accumulators: [k_a = KW*wave + j % KW, column group j / KW][k_c], register v = k_b = 4*lq + v
    f32x4 wr[KW * CH][C], wi[KW * CH][C];
    constexpr int KH = KW / 2;                         // k_a of this wave per half of a tile (all column groups)
    auto clear_half = [&](int h) {
#pragma unroll
        for (int cg = 0; cg < CH; ++cg)
#pragma unroll
            for (int ja = h * KH; ja < (h + 1) * KH; ++ja)
#pragma unroll
                for (int kc = 0; kc < C; ++kc) {
                    wr[KW * cg + ja][kc] = f32x4{0.f, 0.f, 0.f, 0.f};
                    wi[KW * cg + ja][kc] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
    };

    // ---- producer: slot `slot` (0..3) of the tile whose data sits in xs -> ring buffer `buf`; then the
    // request for global slot g_next into the same registers
    auto produce = [&](int slot, int buf, int64_t g_next) {
        f32x4 p1[CH][CP][NAB], p2[CH][CP][NAB], p3[CH][CP][NAB];
#pragma unroll
        for (int cg = 0; cg < CH; ++cg)
#pragma unroll
            for (int cp = 0; cp < CP; ++cp)
#pragma unroll
                for (int ab = 0; ab < NAB; ++ab) {
                    p1[cg][cp][ab] = f32x4{0.f, 0.f, 0.f, 0.f};
                    p2[cg][cp][ab] = p1[cg][cp][ab];
                    p3[cg][cp][ab] = p1[cg][cp][ab];
                }
        // The registers of a k-step are free as soon as its matrix instructions have been issued, and the
        // request for the next slot goes out step by step between them.
        request_begin(g_next);
#pragma unroll
        for (int sq = 0; sq < NS1 / 4; ++sq) {
            f32x4 fr[NAB], fi[NAB], fs[NAB];
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab) {
                const f32x4* t = faT + ((ab * (NS1 / 4) + sq) * 3) * 64 + lane;
                fr[ab] = t[0], fi[ab] = t[64], fs[ab] = t[128];
            }
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
#pragma unroll
                for (int cg = 0; cg < CH; ++cg)
#pragma unroll
                    for (int cp = 0; cp < CP; ++cp) {
                        const f32x2 x = xs[cp][4 * sq + s4][cg];
                        const float xr = SWAP ? x.y : x.x, xi = SWAP ? x.x : x.y;
#pragma unroll
                        for (int ab = 0; ab < NAB; ++ab) {
                            p1[cg][cp][ab] = mfma(fr[ab][s4], xr, p1[cg][cp][ab]);
                            p2[cg][cp][ab] = mfma(fi[ab][s4], xi, p2[cg][cp][ab]);
                            p3[cg][cp][ab] = mfma(fs[ab][s4], xr + xi, p3[cg][cp][ab]);
                        }
                    }
                __builtin_amdgcn_sched_barrier(0);
                request_step(4 * sq + s4);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        const int beta = 4 * slot + pb;
#pragma unroll
        for (int cg = 0; cg < CH; ++cg)
#pragma unroll
            for (int ab = 0; ab < NAB; ++ab) {
                f32x4 zr[CP], zi[CP];
#pragma unroll
                for (int cp = 0; cp < CP; ++cp) {
                    // twiddles of this lane's four k_a = 16*ab + 4*lq + v: 32 contiguous bytes of T[b = 16*c + beta][k_a]
                    const f32x4* t = reinterpret_cast<const f32x4*>(tw1 + (16 * (ph + 2 * cp) + beta) * A + 16 * ab + 4 * lq);
                    const f32x4 t01 = t[0], t23 = t[1];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float tx = (v < 2 ? t01 : t23)[2 * (v & 1)], ty = (v < 2 ? t01 : t23)[2 * (v & 1) + 1];
                        const float re = p1[cg][cp][ab][v] - p2[cg][cp][ab][v];
                        const float im = p3[cg][cp][ab][v] - p1[cg][cp][ab][v] - p2[cg][cp][ab][v];
                        zr[cp][v] = re * tx - im * ty;
                        zi[cp][v] = re * ty + im * tx;
                    }
                }
                if constexpr (CP > 1) small_dft<CP>(zr, zi);
                f32x2* zw = ring + (size_t)buf * L::ring_elems + (size_t)(ph * CP) * (A * KP) + (16 * ab) * KP + cg * 64 +
                            pb * 16 + l16;
#pragma unroll
                for (int m = 0; m < CP; ++m)
#pragma unroll
                    for (int v = 0; v < 4; ++v) zw[m * (A * KP) + (4 * lq + v) * KP] = f32x2{zr[m][v], zi[m][v]};
            }
    };

    // ---- consumer: slot `slot` of the tile at st from ring buffer `buf`
    auto consume = [&](int slot, int buf) {
        __builtin_amdgcn_sched_barrier(0);             // the two steps one after the other: their temporaries share registers
        const f32x2 f2 = fbT[slot * 64 + lane];         // F16[k_b = l16][beta = 4*slot + lq]
        const float f[3] = {f2.x, f2.y, -f2.y};
        // w_B^(k_c beta) for this lane's beta: C contiguous complex numbers
        f32x4 tq[CP];
        {
            const f32x4* t = reinterpret_cast<const f32x4*>(tw2 + (4 * slot + lq) * C);
#pragma unroll
            for (int q = 0; q < CP; ++q) tq[q] = t[q];
        }
        const f32x2* zr0 = ring + (size_t)buf * L::ring_elems + lq * 16 + l16;
#pragma unroll
        for (int j = 0; j < KW * CH; ++j) {            // j = KW * column group + (k_a % KW)
            const f32x2* zp = zr0 + (KW * wave + j % KW) * KP + (j / KW) * 64;
            float ur[C], ui[C];
#pragma unroll
            for (int m = 0; m < CP; ++m) {
                const f32x2 e0 = zp[m * (A * KP)], e1 = zp[(CP + m) * (A * KP)];
                // w_C^m e1 (forward): C = 2: 1;  C = 4: 1, -i;  C = 8: 1, (1 - i) h, -i, (-1 - i) h
                float qr, qi;
                constexpr float h = 0.70710678118654752440f;
                const int k8 = m * (8 / C);
                if (k8 == 0) qr = e1.x, qi = e1.y;
                else if (k8 == 1) qr = (e1.x + e1.y) * h, qi = (e1.y - e1.x) * h;
                else if (k8 == 2) qr = e1.y, qi = -e1.x;
                else qr = (e1.y - e1.x) * h, qi = -(e1.x + e1.y) * h;
                ur[m] = e0.x + qr, ui[m] = e0.y + qi;
                ur[m + CP] = e0.x - qr, ui[m + CP] = e0.y - qi;
            }
#pragma unroll
            for (int kc = 1; kc < C; ++kc) {
                const float tx = tq[kc / 2][2 * (kc & 1)], ty = tq[kc / 2][2 * (kc & 1) + 1];
                const float re = ur[kc], im = ui[kc];
                ur[kc] = re * tx - im * ty;
                ui[kc] = re * ty + im * tx;
            }
#pragma unroll
            for (int kc = 0; kc < C; ++kc) wr[j][kc] = mfma(f[0], ur[kc], wr[j][kc]);
#pragma unroll
            for (int kc = 0; kc < C; ++kc) wi[j][kc] = mfma(f[0], ui[kc], wi[j][kc]);
#pragma unroll
            for (int kc = 0; kc < C; ++kc) wr[j][kc] = mfma(f[2], ui[kc], wr[j][kc]);
#pragma unroll
            for (int kc = 0; kc < C; ++kc) wi[j][kc] = mfma(f[1], ur[kc], wi[j][kc]);
        }
    };

    // Half h of this wave's k_a (accumulator sets j = KW * column group + k_a % KW) of the tile at position p.
    auto store_half = [&](int h, const Pos& p) {
        // rows k_a + A*k_c + A*C*k_b with k_b = 4*lq + v; the lane part needs 64 bits at N = 2048
        float2* dst = Y + ((int64_t)p.o * a.outO + (int64_t)p.y * a.outY + (int64_t)p.zt * (16 * CH)) +
                      ((int64_t)(A * C * 4 * lq) * outN + l16);
#pragma unroll
        for (int ja = h * KH; ja < (h + 1) * KH; ++ja)
#pragma unroll
            for (int kc = 0; kc < C; ++kc)
#pragma unroll
                for (int v = 0; v < 4; ++v)
#pragma unroll
                    for (int cg = 0; cg < CH; ++cg) {     // neighbouring 128-byte pieces of one row
                        const float re = wr[KW * cg + ja][kc][v], im = wi[KW * cg + ja][kc][v];
                        __builtin_nontemporal_store(
                            SWAP ? f32x2{im, re} : f32x2{re, im},
                            reinterpret_cast<f32x2*>(dst + (int64_t)(KW * wave + ja + A * kc + A * C * v) * outN + 16 * cg));
                    }
    };

    // Slots are numbered g = 0, 1, .. across the tiles of this workgroup.  One barrier per slot: before it
    // every wave has written slot g into ring buffer g % 2 and finished reading that buffer for slot g - 2;
    // after it the producer step of slot g + 1 and the consumer step of slot g run.
    // A finished tile is stored in two halves a slot apart: the first right after its last consumer step,
    // the second after the next producer step, whose requests then queue behind half as many stores (the
    // counter a wave waits on retires loads and stores in issue order).
    clear_half(0);
    clear_half(1);
    request_slot(0);
    __syncthreads();                                   // tables
    produce(0, 0, 1);
    Pos done = st;                                     // tile whose second half is still in the accumulators
    for (int64_t g = 0; g < G; ++g) {
        __syncthreads();
        const int slot = (int)(g & 3), buf = (int)(g & 1);
        produce((slot + 1) & 3, buf ^ 1, g + 2);
        if (slot == 0 && g != 0) {
            store_half(1, done);
            clear_half(1);
        }
        consume(slot, buf);
        if (slot == 3) {
            store_half(0, st);
            clear_half(0);
            done = st;
            advance(st);
        }
    }
    store_half(1, done);
}

template <int NAB, int C, int CH, int WPC>
hipError_t launch_sn_inst(const FftStridedArgs& a, const DeviceMatrix& FA, const DeviceMatrix& FB, const float2* Tw,
                          float scale, int conj, hipStream_t stream)
{
    const int64_t ntiles = a.O * a.Yn * (a.Zt / CH);
    const int64_t blocks = ntiles < 256 * WPC ? ntiles : 256 * WPC;      // persistent workgroups
    constexpr size_t lds = FftSnLayout<NAB, C, CH>::lds_bytes;
    if (conj)
        hipLaunchKernelGGL((k_fft_sn<NAB, C, CH, true, WPC>), dim3((unsigned)blocks), dim3(512), lds, stream, a, FA, FB, Tw,
                           scale);
    else
        hipLaunchKernelGGL((k_fft_sn<NAB, C, CH, false, WPC>), dim3((unsigned)blocks), dim3(512), lds, stream, a, FA, FB, Tw,
                           scale);
    return hipGetLastError();
}

// ---- first stage of a split with a small first factor ----------------------------------------------
// N = R * M with R = 2, 4 or 8 and the M-point second stage on one of the fused kernels above (8192 =
// 4 * 2048): the first stage of Eq. 13 - 16, Z[k_a, j] = T[k_a, beta] * sum_l w_R^(k_a l) x[l, j] on the view
// [O][R][I] (I = M * inner, beta = j / inner), is R-point butterflies on R values I elements apart plus one
// complex multiplication: a memory-bound, element-wise pass.  A thread takes two neighbouring j (16-byte
// accesses); the host checks that I is even and that the two share beta or are neighbours in it.
// PERM: the input rows (innermost axis, nz = pA * pB points) still hold the result of a split pA x pB of that
// axis as [k_a][k_b]; the pass reads position (z % pA) * pB + z / pA for column z, which is that axis'
// re-ordering to natural order done on the way in (two 8-byte reads pB apart instead of one of 16 bytes).
template <int R, bool SWAP, bool PERM>
__global__ __launch_bounds__(256) void k_radix_tw(const float2* __restrict__ in, float2* __restrict__ out,
                                                  int64_t npairs, uint32_t halfI, uint32_t inner, int B,
                                                  const float2* __restrict__ Tw, uint32_t nz, uint32_t pA, uint32_t pB)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= npairs) return;
    const int64_t o = t / halfI;
    const uint32_t j = 2u * (uint32_t)(t - o * halfI);
    const int64_t I = 2 * (int64_t)halfI;
    const int64_t base = o * R * I + j;
    f32x2 re[R], im[R];
#pragma unroll
    for (int l = 0; l < R; ++l) {
        f32x4 v;
        if constexpr (PERM) {
            // j even and pA even: columns z and z + 1 share z / pA and sit pB apart in the input
            const uint32_t z = j % nz;
            const f32x2* src = reinterpret_cast<const f32x2*>(in + base + l * I) - z + ((z % pA) * pB + z / pA);
            const f32x2 e0 = __builtin_nontemporal_load(src), e1 = __builtin_nontemporal_load(src + pB);
            v = f32x4{e0.x, e0.y, e1.x, e1.y};
        } else {
            v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(in + base + l * I));
        }
        re[l] = SWAP ? f32x2{v.y, v.w} : f32x2{v.x, v.z};
        im[l] = SWAP ? f32x2{v.x, v.z} : f32x2{v.y, v.w};
    }
    small_dft<R>(re, im);
    if (Tw) {
        const uint32_t b0 = j / inner, b1 = (j + 1) / inner;
#pragma unroll
        for (int k = 1; k < R; ++k) {                  // T[0, beta] = 1
            const float2 w0 = Tw[(int64_t)k * B + b0], w1 = Tw[(int64_t)k * B + b1];
            const f32x2 wr = {w0.x, w1.x}, wi = {w0.y, w1.y};
            const f32x2 r = re[k], i = im[k];
            re[k] = r * wr - i * wi;
            im[k] = r * wi + i * wr;
        }
    }
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const f32x4 v = SWAP ? f32x4{im[k].x, re[k].x, im[k].y, re[k].y} : f32x4{re[k].x, im[k].x, re[k].y, im[k].y};
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(out + base + k * I));
    }
}

template <int R, bool PERM>
hipError_t launch_radix_inst(const float2* in, float2* out, int64_t O, int64_t I, int64_t inner, int B, const float2* Tw,
                             int conj, int64_t nz, int pA, int pB, hipStream_t stream)
{
    const int64_t npairs = O * (I / 2);
    const int64_t blocks = (npairs + 255) / 256;
    if (blocks >= (int64_t(1) << 31)) return hipErrorInvalidValue;
    if (conj)
        hipLaunchKernelGGL((k_radix_tw<R, true, PERM>), dim3((unsigned)blocks), dim3(256), 0, stream, in, out, npairs,
                           (uint32_t)(I / 2), (uint32_t)inner, B, Tw, (uint32_t)nz, (uint32_t)pA, (uint32_t)pB);
    else
        hipLaunchKernelGGL((k_radix_tw<R, false, PERM>), dim3((unsigned)blocks), dim3(256), 0, stream, in, out, npairs,
                           (uint32_t)(I / 2), (uint32_t)inner, B, Tw, (uint32_t)nz, (uint32_t)pA, (uint32_t)pB);
    return hipGetLastError();
}

}  // namespace

bool radix_stage_supported(int R, int64_t B, int64_t inner)
{
    // pairs of neighbouring elements of [B][inner]: in the same beta (inner even) or in neighbouring ones (inner 1)
    return (R == 2 || R == 4 || R == 8) && B >= 1 && inner >= 1 && (B * inner) % 2 == 0 && (inner == 1 || inner % 2 == 0) &&
           B * inner < (int64_t(1) << 32);
}

hipError_t launch_radix_twiddle(const float2* in, float2* out, int64_t O, int R, int64_t B, int64_t inner,
                                const float2* Tw, int conj, int64_t nz, int pA, int pB, hipStream_t stream)
{
    if (O <= 0) return hipSuccess;
    if (!radix_stage_supported(R, B, inner) || B >= (int64_t(1) << 31)) return hipErrorInvalidValue;
    const int64_t I = B * inner;
    if (pA > 1) {
        // the permuted read works on whole rows of the innermost axis below the transformed one
        if (nz < 2 || nz >= (int64_t(1) << 31) || inner % nz != 0 || pA % 2 != 0 || (int64_t)pA * pB != nz)
            return hipErrorInvalidValue;
        if (R == 2) return launch_radix_inst<2, true>(in, out, O, I, inner, (int)B, Tw, conj, nz, pA, pB, stream);
        if (R == 4) return launch_radix_inst<4, true>(in, out, O, I, inner, (int)B, Tw, conj, nz, pA, pB, stream);
        return launch_radix_inst<8, true>(in, out, O, I, inner, (int)B, Tw, conj, nz, pA, pB, stream);
    }
    if (R == 2) return launch_radix_inst<2, false>(in, out, O, I, inner, (int)B, Tw, conj, 1, 1, 1, stream);
    if (R == 4) return launch_radix_inst<4, false>(in, out, O, I, inner, (int)B, Tw, conj, 1, 1, 1, stream);
    return launch_radix_inst<8, false>(in, out, O, I, inner, (int)B, Tw, conj, 1, 1, 1, stream);
}

bool fft_zn_supported(int A, int B)
{
    return (A == 16 && (B == 32 || B == 64 || B == 128)) || (A == 32 && (B == 32 || B == 64));
}

hipError_t launch_fft_zn(const float2* in, float2* out, int64_t nrows, int A, int B, const DeviceMatrix& FA,
                         const DeviceMatrix& FB, const float2* Tw, float scale, int conj, hipStream_t stream)
{
    if (nrows <= 0) return hipSuccess;
    // the kernel indexes the stage matrices and the twiddle table without bounds checks
    if (!fft_zn_supported(A, B) || FA.K != A || FA.N != A || FB.K != B || FB.N != B || !Tw) return hipErrorInvalidValue;
    if (A == 32 && B == 64) return launch_zn_inst<2, 4, 2>(in, out, nrows, FA, FB, Tw, scale, conj, stream);
    if (A == 32 && B == 32) return launch_zn_inst<2, 2, 3>(in, out, nrows, FA, FB, Tw, scale, conj, stream);
    // three workgroups per CU where the registers allow (512^3: 0.383 -> 0.375 ms)
    if (B == 32) return launch_zn_inst<1, 2, 3>(in, out, nrows, FA, FB, Tw, scale, conj, stream);
    if (B == 64) return launch_zn_inst<1, 4, 3>(in, out, nrows, FA, FB, Tw, scale, conj, stream);
    if (B == 128) return launch_zn_inst<1, 8, 2>(in, out, nrows, FA, FB, Tw, scale, conj, stream);
    return hipErrorInvalidValue;
}

bool fft_sn_supported(int A, int B, int64_t I)
{
    // 32-bit lane offsets of the loads: up to 3*B rows of I elements
    return ((A == 16 && (B == 32 || B == 64 || B == 128)) || (A == 32 && (B == 32 || B == 64))) && I % 16 == 0 &&
           I <= (int64_t(1) << 23);
}

namespace {
template <int NAB, int C, int CH, int WPC>
hipError_t configure_sn()
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_fft_sn<NAB, C, CH, false, WPC>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)FftSnLayout<NAB, C, CH>::lds_bytes);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_fft_sn<NAB, C, CH, true, WPC>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)FftSnLayout<NAB, C, CH>::lds_bytes);
}
}  // namespace

hipError_t configure_fft_nested_kernels()
{
    hipError_t e = configure_sn<1, 8, 1, 1>();
    if (e == hipSuccess) e = configure_sn<1, 4, 1, 2>();
    if (e == hipSuccess) e = configure_sn<1, 4, 2, 1>();
    if (e == hipSuccess) e = configure_sn<1, 2, 1, 2>();
    if (e == hipSuccess) e = configure_sn<1, 2, 4, 1>();
    if (e == hipSuccess) e = configure_sn<2, 4, 1, 1>();
    if (e == hipSuccess) e = configure_sn<2, 2, 2, 1>();
    if (e == hipSuccess) e = configure_sn<2, 2, 1, 1>();
    return e;
}

hipError_t launch_fft_sn(const FftStridedArgs& a, int A, int B, const DeviceMatrix& FA, const DeviceMatrix& FB,
                         const float2* Tw, float scale, int conj, hipStream_t stream)
{
    if (a.O <= 0 || a.Yn <= 0 || a.Zt <= 0) return hipSuccess;
    const int64_t lim = int64_t(1) << 23;
    if (!fft_sn_supported(A, B, 16) || a.inN < 16 || a.outN < 16 || a.inN > lim || a.outN > lim || FA.K != A ||
        FA.N != A || FB.K != B || FB.N != B || !Tw)
        return hipErrorInvalidValue;
    if (A == 32 && B == 64) return launch_sn_inst<2, 4, 1, 1>(a, FA, FB, Tw, scale, conj, stream);
    if (A == 32 && B == 32) {
        if (a.Zt % 2 == 0) return launch_sn_inst<2, 2, 2, 1>(a, FA, FB, Tw, scale, conj, stream);
        return launch_sn_inst<2, 2, 1, 1>(a, FA, FB, Tw, scale, conj, stream);
    }
    // Wider tiles mean longer contiguous pieces per row (128 bytes per 16 columns) but one workgroup per CU
    // instead of two once the accumulators of N * columns outputs fill its registers.  Measured: 1024 points,
    // 32 columns: 3.74 -> 3.48 ms (y) and 4.55 -> 3.91 ms (x) at 1024^3; 512 points, 64 columns: 0.474 ->
    // 0.448 ms for the x pass of 512^3 (rows 2 MiB apart) but 0.426 -> 0.442 ms for its y pass (rows 4 KiB
    // apart), so the wide tile is taken for rows at least 32 KiB apart.
    if (B == 128) return launch_sn_inst<1, 8, 1, 1>(a, FA, FB, Tw, scale, conj, stream);
    if (B == 64) {
        if (a.Zt % 2 == 0) return launch_sn_inst<1, 4, 2, 1>(a, FA, FB, Tw, scale, conj, stream);
        return launch_sn_inst<1, 4, 1, 2>(a, FA, FB, Tw, scale, conj, stream);
    }
    if (B == 32) {
        if (a.Zt % 4 == 0 && a.inN >= 4096) return launch_sn_inst<1, 2, 4, 1>(a, FA, FB, Tw, scale, conj, stream);
        return launch_sn_inst<1, 2, 1, 2>(a, FA, FB, Tw, scale, conj, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace dft3d
