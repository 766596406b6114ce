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
// Every row costs three quarters of (A + B) * (A*B / 256) MFMAs (three real products per complex
// product) and nothing else but a few VALU operations per point for the twiddle and the sums.  With
// no LDS and no barriers, six waves per SIMD overlap each other's loads, stores and MFMAs.  In the
// library this kernel serves 16 x 16; the larger splits run the kernels of dft3d_fft_nested.hip.
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

template <int A, int B, int MINW>
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
    f32x2 xa[NBB][NS1], xb[NBB][NS1];
    load_row(xa, wave);
    for (int64_t row = wave; row < nrows; row += 2 * nwaves) {
        // a request past the end re-reads the wave's current row (in bounds, never used)
        const int64_t row1 = row + nwaves, row2 = row + 2 * nwaves;
        load_row(xb, row1 < nrows ? row1 : row);
        __builtin_amdgcn_sched_barrier(0);
        transform_row_3m(xa, row);
        __builtin_amdgcn_sched_barrier(0);
        if (row1 >= nrows) break;
        load_row(xa, row2 < nrows ? row2 : row);
        __builtin_amdgcn_sched_barrier(0);
        transform_row_3m(xb, row1);
        __builtin_amdgcn_sched_barrier(0);
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

template <int A, int B, int MINW>
hipError_t launch_inst(const float2* in, float2* out, int64_t nrows, const DeviceMatrix& FA,
                       const DeviceMatrix& FB, const float2* Tw, float scale, int conj, hipStream_t stream)
{
    // persistent waves: MINW per SIMD on every CU, fewer when there are fewer rows
    const int64_t resident = 256 * MINW;                 // workgroups of 4 waves
    const int64_t want = (nrows + 3) / 4;
    const int64_t blocks = want < resident ? want : resident;
    hipLaunchKernelGGL((k_fft_zr<A, B, MINW>), dim3((unsigned)blocks), dim3(256), 0, stream, in, out, nrows, FA, FB,
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
    return configure_fft_nested_kernels();
}

bool fft_sr_supported(int A, int B, int64_t I)
{
    // 32-bit lane offsets inside the kernels: up to 12*A rows (and 3*B rows) of I elements
    if (I % 16 != 0) return false;
    if (fft_sn_supported(A, B, I)) return true;
    return I <= (int64_t(1) << 21) && A == 16 && B == 16;
}

hipError_t launch_fft_sr_ex(const FftStridedArgs& a, int A, int B, const DeviceMatrix& FA,
                            const DeviceMatrix& FB, const float2* Tw, float scale, int conj, hipStream_t stream)
{
    if (a.O <= 0 || a.Yn <= 0 || a.Zt <= 0) return hipSuccess;
    if (fft_sn_supported(A, B, 16)) return launch_fft_sn(a, A, B, FA, FB, Tw, scale, conj, stream);
    const int64_t lim = int64_t(1) << 21;
    if (a.inN < 16 || a.outN < 16 || a.inN > lim || a.outN > lim || FA.K != A || FA.N != A || FB.K != B ||
        FB.N != B || !Tw)
        return hipErrorInvalidValue;
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
    return A == 16 && B == 16;
}

hipError_t launch_fft_zr(const float2* in, float2* out, int64_t nrows, int A, int B, const DeviceMatrix& FA,
                         const DeviceMatrix& FB, const float2* Tw, float scale, int conj, hipStream_t stream)
{
    if (nrows <= 0) return hipSuccess;
    // the kernel indexes the stage matrices and the twiddle table without bounds checks
    if (FA.K != A || FA.N != A || FB.K != B || FB.N != B || !Tw) return hipErrorInvalidValue;
    if (A == 16 && B == 16) return launch_inst<16, 16, 6>(in, out, nrows, FA, FB, Tw, scale, conj, stream);
    return hipErrorInvalidValue;
}

}  // namespace dft3d
