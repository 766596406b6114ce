// HIP kernels of the dft3d library for gfx950 (CDNA4, 64-wide wavefronts).
//
//  * mode contraction  out[o,k,i] = sum_n M[k,n] in[o,n,i]  on fp32 MFMA (v_mfma_f32_16x16x4_f32),
//    4-real-product complex scheme, matrix tiles and data tiles staged through LDS:
//      - k_contract_s : inner extent I > 1 ("strided" modes): the data tile is the B operand,
//        loaded as rows of the contiguous index i so HBM reads and writes are coalesced;
//      - k_contract_c : I == 1 (the contracted index is the contiguous one): the data tile is
//        the A operand, output rows are written along k.
//    Both take an optional fused twiddle (phase adjustment) and a scale in the epilogue.
//  * k_phase   : standalone twiddle multiply (memory-bound).
//  * k_reorder : sub-index swap that puts the split transform in natural order; the swap of
//    the fastest axis is a transposition through LDS, the other axes only permute row addresses.
//
// MFMA lane layout used throughout (16x16x4, one block): lane l supplies A[l%16][l/16] and
// B[l/16][l%16]; accumulator register v of lane l is D[4*(l/16)+v][l%16].
#include <hip/hip_runtime.h>

#include "dft3d_internal.h"

namespace dft3d {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;  // 4 wavefronts per workgroup

__device__ __forceinline__ f32x4 mfma16(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// Workgroups are handed to the 8 XCDs round-robin by launch index.  Re-map the index so that
// each XCD works on a contiguous range of logical tiles (neighbouring tiles share matrix and
// data tiles, which then hit in that XCD's own L2).
__device__ __forceinline__ int64_t xcd_remap(int64_t wg, int64_t total)
{
    constexpr int64_t kXcds = 8;
    if (total % kXcds != 0) return wg;
    return (wg % kXcds) * (total / kXcds) + wg / kXcds;
}

__device__ __forceinline__ int64_t out_offset(const ContractArgs& a, int64_t o)
{
    return (o / a.Olo) * a.sYohi + (o % a.Olo) * a.sYolo;
}

// ------------------------------------------------------------------------------------------
// Mode contraction on fp32 MFMA.  Two kernels share one software pipeline:
//
//   prologue : chunk 0 global -> registers -> LDS[0]; barrier
//   chunk c  : request chunk c+1 from global memory into registers; MFMAs on LDS[c&1]
//              (operands of k-step s+1 are read from LDS while the MFMAs of k-step s issue);
//              then registers -> LDS[(c+1)&1]; barrier
//
// so a global load always has one full chunk of MFMA work to land, and there is one barrier
// per chunk.  MASKED = false is the fast path for shapes that are whole multiples of the tile:
// no bounds logic at all.  MASKED = true clamps addresses and selects zeros (branch-free).
// EV = complex numbers per global load of the data tile (2 -> 16-byte loads).
// ------------------------------------------------------------------------------------------
template <int EV> struct CVec;
template <> struct CVec<1> { typedef f32x2 type; };   // native vectors: they stay in registers
template <> struct CVec<2> { typedef f32x4 type; };

template <int EV>
__device__ __forceinline__ typename CVec<EV>::type cvec_zero();
template <> __device__ __forceinline__ f32x2 cvec_zero<1>() { return f32x2{0.f, 0.f}; }
template <> __device__ __forceinline__ f32x4 cvec_zero<2>() { return f32x4{0.f, 0.f, 0.f, 0.f}; }

// store one or two complex numbers to an LDS location that is only 8-byte aligned
__device__ __forceinline__ void store_cvec(float2* dst, f32x2 v)
{
    *reinterpret_cast<f32x2*>(dst) = v;
}
__device__ __forceinline__ void store_cvec(float2* dst, f32x4 v)
{
    *reinterpret_cast<f32x2*>(dst) = f32x2{v.x, v.y};
    *reinterpret_cast<f32x2*>(dst + 1) = f32x2{v.z, v.w};
}

// Strided-mode contraction.  Workgroup tile: TM output rows (k) x TN columns (i) of one o.
// Waves tile it as (TM/WM) x (TN/WN); each wave owns WM x WN complex outputs.
template <int TM, int TN, int WM, int WN, int KC, int EV, bool MASKED, int MINW>
__global__ __launch_bounds__(kThreads, MINW) void k_contract_s(ContractArgs a, int tilesK,
                                                               int64_t tilesI, int64_t total)
{
    typedef typename CVec<EV>::type xvec;
    constexpr int NWN = TN / WN;
    static_assert((TM / WM) * NWN == 4, "four waves per workgroup");
    static_assert(!MASKED || EV == 1, "the masked path loads single elements");
    constexpr int BM = WM / 16, BN = WN / 16, KS = KC / 4;
    constexpr int XP = TN + 16;   // float2 pitch: rows n, n+1 land 32 banks apart (b64 reads conflict-free)
    constexpr int VP = TM + 16;   // float pitch: rows n..n+3 land 16 banks apart
    constexpr int TPR = TN / EV;                  // threads per tile row
    static_assert(kThreads % TPR == 0, "row must divide the workgroup");
    constexpr int XRPP = kThreads / TPR;          // rows per pass
    static_assert(KC % XRPP == 0, "KC must be a multiple of the rows per pass");
    constexpr int XL = KC / XRPP;                 // loads per thread per chunk

    __shared__ __align__(16) float2 Xs[2][KC][XP];
    __shared__ __align__(16) float Vr[2][KC][VP];
    __shared__ __align__(16) float Vi[2][KC][VP];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm0 = (wave / NWN) * WM;
    const int wn0 = (wave % NWN) * WN;
    const int l16 = lane & 15;
    const int lq = lane >> 4;

    // logical tile: k-tile fastest, then column tile, then o
    int64_t t = xcd_remap((int64_t)blockIdx.x, total);
    const int kt = (int)(t % tilesK);
    t /= tilesK;
    const int64_t it = t % tilesI;
    const int64_t o = t / tilesI;
    const int k0 = kt * TM;
    const int64_t i0 = it * TN;

    const int N = a.M.N;
    const int64_t I = a.I;
    const float2* __restrict__ Xo = a.X + o * (int64_t)N * I;

    const int xc = (tid % TPR) * EV;
    const int xr = tid / TPR;
    const bool xcol_ok = !MASKED || (i0 + xc) < I;
    const int64_t xcol = MASKED ? ((i0 + xc) < I ? (i0 + xc) : (I - 1)) : (i0 + xc);

    constexpr int VV = KC * TM / 4;               // float4 per matrix plane per chunk
    constexpr int VL = (VV + kThreads - 1) / kThreads;
    xvec xreg[XL];
    f32x4 vrreg[VL], vireg[VL];

    auto gload = [&](int n0) {
#pragma unroll
        for (int j = 0; j < VL; ++j) {
            const int f = tid + j * kThreads;
            if (VV % kThreads == 0 || f < VV) {
                const int r = f / (TM / 4), c4 = f % (TM / 4);
                const int64_t off = (int64_t)(n0 + r) * a.M.ld + k0 + c4 * 4;
                vrreg[j] = *reinterpret_cast<const f32x4*>(a.M.re + off);
                vireg[j] = *reinterpret_cast<const f32x4*>(a.M.im + off);
            }
        }
#pragma unroll
        for (int j = 0; j < XL; ++j) {
            const int n = n0 + xr + j * XRPP;
            if (MASKED) {
                const int nn = n < N ? n : N - 1;
                xvec v = *reinterpret_cast<const xvec*>(Xo + (int64_t)nn * I + xcol);
                xreg[j] = (xcol_ok && n < N) ? v : cvec_zero<EV>();
            } else {
                xreg[j] = *reinterpret_cast<const xvec*>(Xo + (int64_t)n * I + xcol);
            }
        }
    };
    const float vsign = a.conj ? -1.0f : 1.0f;
    auto lstore = [&](int buf) {
#pragma unroll
        for (int j = 0; j < VL; ++j) {
            const int f = tid + j * kThreads;
            if (VV % kThreads == 0 || f < VV) {
                const int r = f / (TM / 4), c4 = f % (TM / 4);
                *reinterpret_cast<f32x4*>(&Vr[buf][r][c4 * 4]) = vrreg[j];
                *reinterpret_cast<f32x4*>(&Vi[buf][r][c4 * 4]) = vireg[j] * vsign;
            }
        }
#pragma unroll
        for (int j = 0; j < XL; ++j)
            *reinterpret_cast<xvec*>(&Xs[buf][xr + j * XRPP][xc]) = xreg[j];
    };

    f32x4 accr[BM][BN], acci[BM][BN];
#pragma unroll
    for (int bm = 0; bm < BM; ++bm)
#pragma unroll
        for (int bn = 0; bn < BN; ++bn) {
            accr[bm][bn] = f32x4{0.f, 0.f, 0.f, 0.f};
            acci[bm][bn] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

    const int nchunks = (N + KC - 1) / KC;
    gload(0);
    lstore(0);
    __syncthreads();

    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        const bool more = (c + 1) < nchunks;
        if (more) gload((c + 1) * KC);      // lands while this chunk's MFMAs run
        float ar[2][BM], ai[2][BM];
        f32x2 bx[2][BN];
        auto read_operands = [&](int slot, int s) {
            const int n = 4 * s + lq;
#pragma unroll
            for (int bm = 0; bm < BM; ++bm) {
                ar[slot][bm] = Vr[buf][n][wm0 + bm * 16 + l16];
                ai[slot][bm] = Vi[buf][n][wm0 + bm * 16 + l16];
            }
#pragma unroll
            for (int bn = 0; bn < BN; ++bn)
                bx[slot][bn] = *reinterpret_cast<const f32x2*>(&Xs[buf][n][wn0 + bn * 16 + l16]);
        };
        read_operands(0, 0);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int cur = s & 1;
            if (s + 1 < KS) read_operands(cur ^ 1, s + 1);
            float an[BM];
#pragma unroll
            for (int bm = 0; bm < BM; ++bm) an[bm] = -ai[cur][bm];
#pragma unroll
            for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                for (int bn = 0; bn < BN; ++bn)
                    accr[bm][bn] = mfma16(ar[cur][bm], bx[cur][bn].x, accr[bm][bn]);
#pragma unroll
            for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                for (int bn = 0; bn < BN; ++bn)
                    acci[bm][bn] = mfma16(ar[cur][bm], bx[cur][bn].y, acci[bm][bn]);
#pragma unroll
            for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                for (int bn = 0; bn < BN; ++bn)
                    accr[bm][bn] = mfma16(an[bm], bx[cur][bn].y, accr[bm][bn]);
#pragma unroll
            for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                for (int bn = 0; bn < BN; ++bn)
                    acci[bm][bn] = mfma16(ai[cur][bm], bx[cur][bn].x, acci[bm][bn]);
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the LDS refill (and its wait) behind the MFMAs
        if (more) lstore(buf ^ 1);
        __syncthreads();
    }

    // epilogue: scale, optional twiddle, store (16 consecutive columns per quarter-wave)
    const int K = a.M.K;
    float2* __restrict__ Yo = a.Y + out_offset(a, o);
#pragma unroll
    for (int bn = 0; bn < BN; ++bn) {
        const int64_t col = i0 + wn0 + bn * 16 + l16;
        if (MASKED && col >= I) continue;
        const int64_t beta = a.Tw ? (col / a.twInner) : 0;
#pragma unroll
        for (int bm = 0; bm < BM; ++bm) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int k = k0 + wm0 + bm * 16 + 4 * lq + v;
                if (MASKED && k >= K) continue;
                float yr = accr[bm][bn][v] * a.scale;
                float yi = acci[bm][bn][v] * a.scale;
                if (a.Tw) {
                    float2 w = a.Tw[(int64_t)k * a.twB + beta];
                    if (a.conj) w.y = -w.y;
                    float tr = yr * w.x - yi * w.y;
                    float ti = yr * w.y + yi * w.x;
                    yr = tr;
                    yi = ti;
                }
                Yo[(int64_t)k * a.sYk + col] = make_float2(yr, yi);
            }
        }
    }
}

// Contiguous-mode contraction (I == 1): out[o, k] = sum_n in[o, n] M[k, n].
// Workgroup tile: TO rows (o) x TK columns (k).  The data tile is the MFMA A operand.
template <int TO, int TK, int WO, int WK, int KC, int EV, bool MASKED, int MINW>
__global__ __launch_bounds__(kThreads, MINW) void k_contract_c(ContractArgs a, int tilesK,
                                                               int64_t tilesO, int64_t total)
{
    typedef typename CVec<EV>::type xvec;
    constexpr int NWK = TK / WK;
    static_assert((TO / WO) * NWK == 4, "four waves per workgroup");
    static_assert(!MASKED || EV == 1, "the masked path loads single elements");
    constexpr int BM = WO / 16, BN = WK / 16, KS = KC / 4;
    constexpr int XP = KC + 1;    // odd pitch (in float2): lanes walking o hit distinct banks
    constexpr int VP = TK + 16;
    constexpr int TPR = KC / EV;                  // threads per data row
    static_assert(kThreads % TPR == 0, "row must divide the workgroup");
    constexpr int XRPP = kThreads / TPR;          // rows per pass
    static_assert(TO % XRPP == 0, "TO must be a multiple of the rows per pass");
    constexpr int XL = TO / XRPP;

    __shared__ __align__(16) float2 Xs[2][TO][XP];
    __shared__ __align__(16) float Vr[2][KC][VP];
    __shared__ __align__(16) float Vi[2][KC][VP];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wo0 = (wave / NWK) * WO;
    const int wk0 = (wave % NWK) * WK;
    const int l16 = lane & 15;
    const int lq = lane >> 4;

    int64_t t = xcd_remap((int64_t)blockIdx.x, total);
    const int kt = (int)(t % tilesK);
    const int64_t ot = t / tilesK;
    const int k0 = kt * TK;
    const int64_t o0 = ot * TO;

    const int N = a.M.N;
    const int64_t O = a.O;

    const int xc = (tid % TPR) * EV;
    const int xr = tid / TPR;

    constexpr int VV = KC * TK / 4;
    constexpr int VL = (VV + kThreads - 1) / kThreads;
    xvec xreg[XL];
    f32x4 vrreg[VL], vireg[VL];

    auto gload = [&](int n0) {
#pragma unroll
        for (int j = 0; j < VL; ++j) {
            const int f = tid + j * kThreads;
            if (VV % kThreads == 0 || f < VV) {
                const int r = f / (TK / 4), c4 = f % (TK / 4);
                const int64_t off = (int64_t)(n0 + r) * a.M.ld + k0 + c4 * 4;
                vrreg[j] = *reinterpret_cast<const f32x4*>(a.M.re + off);
                vireg[j] = *reinterpret_cast<const f32x4*>(a.M.im + off);
            }
        }
#pragma unroll
        for (int j = 0; j < XL; ++j) {
            const int64_t orow = o0 + xr + j * XRPP;
            const int n = n0 + xc;
            if (MASKED) {
                const int64_t oo = orow < O ? orow : O - 1;
                const int nn = n < N ? n : N - 1;
                xvec v = *reinterpret_cast<const xvec*>(a.X + oo * N + nn);
                xreg[j] = (orow < O && n < N) ? v : cvec_zero<EV>();
            } else {
                xreg[j] = *reinterpret_cast<const xvec*>(a.X + orow * N + n);
            }
        }
    };
    const float vsign = a.conj ? -1.0f : 1.0f;
    auto lstore = [&](int buf) {
#pragma unroll
        for (int j = 0; j < VL; ++j) {
            const int f = tid + j * kThreads;
            if (VV % kThreads == 0 || f < VV) {
                const int r = f / (TK / 4), c4 = f % (TK / 4);
                *reinterpret_cast<f32x4*>(&Vr[buf][r][c4 * 4]) = vrreg[j];
                *reinterpret_cast<f32x4*>(&Vi[buf][r][c4 * 4]) = vireg[j] * vsign;
            }
        }
#pragma unroll
        for (int j = 0; j < XL; ++j) {
            float2* dst = &Xs[buf][xr + j * XRPP][xc];     // odd pitch: 8-byte aligned only
            store_cvec(dst, xreg[j]);
        }
    };

    f32x4 accr[BM][BN], acci[BM][BN];
#pragma unroll
    for (int bm = 0; bm < BM; ++bm)
#pragma unroll
        for (int bn = 0; bn < BN; ++bn) {
            accr[bm][bn] = f32x4{0.f, 0.f, 0.f, 0.f};
            acci[bm][bn] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

    const int nchunks = (N + KC - 1) / KC;
    gload(0);
    lstore(0);
    __syncthreads();

    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        const bool more = (c + 1) < nchunks;
        if (more) gload((c + 1) * KC);      // lands while this chunk's MFMAs run
        f32x2 ax[2][BM];
        float br[2][BN], bi[2][BN];
        auto read_operands = [&](int slot, int s) {
            const int n = 4 * s + lq;
#pragma unroll
            for (int bm = 0; bm < BM; ++bm)
                ax[slot][bm] = *reinterpret_cast<const f32x2*>(&Xs[buf][wo0 + bm * 16 + l16][n]);
#pragma unroll
            for (int bn = 0; bn < BN; ++bn) {
                br[slot][bn] = Vr[buf][n][wk0 + bn * 16 + l16];
                bi[slot][bn] = Vi[buf][n][wk0 + bn * 16 + l16];
            }
        };
        read_operands(0, 0);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int cur = s & 1;
            if (s + 1 < KS) read_operands(cur ^ 1, s + 1);
            float bneg[BN];
#pragma unroll
            for (int bn = 0; bn < BN; ++bn) bneg[bn] = -bi[cur][bn];
#pragma unroll
            for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                for (int bn = 0; bn < BN; ++bn)
                    accr[bm][bn] = mfma16(ax[cur][bm].x, br[cur][bn], accr[bm][bn]);
#pragma unroll
            for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                for (int bn = 0; bn < BN; ++bn)
                    acci[bm][bn] = mfma16(ax[cur][bm].x, bi[cur][bn], acci[bm][bn]);
#pragma unroll
            for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                for (int bn = 0; bn < BN; ++bn)
                    accr[bm][bn] = mfma16(ax[cur][bm].y, bneg[bn], accr[bm][bn]);
#pragma unroll
            for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                for (int bn = 0; bn < BN; ++bn)
                    acci[bm][bn] = mfma16(ax[cur][bm].y, br[cur][bn], acci[bm][bn]);
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the LDS refill (and its wait) behind the MFMAs
        if (more) lstore(buf ^ 1);
        __syncthreads();
    }

    const int K = a.M.K;
#pragma unroll
    for (int bn = 0; bn < BN; ++bn) {
        const int k = k0 + wk0 + bn * 16 + l16;
        if (MASKED && k >= K) continue;
#pragma unroll
        for (int bm = 0; bm < BM; ++bm) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int64_t orow = o0 + wo0 + bm * 16 + 4 * lq + v;
                if (MASKED && orow >= O) continue;
                float yr = accr[bm][bn][v] * a.scale;
                float yi = acci[bm][bn][v] * a.scale;
                if (a.Tw) {   // I == 1 means beta == 0
                    float2 w = a.Tw[(int64_t)k * a.twB];
                    if (a.conj) w.y = -w.y;
                    float tr = yr * w.x - yi * w.y;
                    float ti = yr * w.y + yi * w.x;
                    yr = tr;
                    yi = ti;
                }
                a.Y[out_offset(a, orow) + (int64_t)k * a.sYk] = make_float2(yr, yi);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Twiddle multiply: tensor [outer][A][B][inner], out = in * Tw[ka*B + beta].  Each thread moves
// EV consecutive complex numbers (16 bytes when EV == 2).
// ------------------------------------------------------------------------------------------
template <int EV>
__global__ __launch_bounds__(kThreads) void k_phase(const float2* __restrict__ in,
                                                    float2* __restrict__ out, int64_t nvec,
                                                    int AB, int64_t inner,
                                                    const float2* __restrict__ Tw, int conj)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x; v < nvec; v += stride) {
        const int64_t e = v * EV;
        // slot along the split axis = (e / inner) % (A*B); the table is indexed by it directly
        if (EV == 2) {
            float4 x = *reinterpret_cast<const float4*>(in + e);
            float2 w0 = Tw[(e / inner) % AB];
            float2 w1 = Tw[((e + 1) / inner) % AB];
            if (conj) { w0.y = -w0.y; w1.y = -w1.y; }
            float4 y;
            y.x = x.x * w0.x - x.y * w0.y;
            y.y = x.x * w0.y + x.y * w0.x;
            y.z = x.z * w1.x - x.w * w1.y;
            y.w = x.z * w1.y + x.w * w1.x;
            *reinterpret_cast<float4*>(out + e) = y;
        } else {
            float2 x = in[e];
            float2 w = Tw[(e / inner) % AB];
            if (conj) w.y = -w.y;
            out[e] = make_float2(x.x * w.x - x.y * w.y, x.x * w.y + x.y * w.x);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Re-ordering.  One workgroup moves whole rows (the fastest axis) at a time: a row is read
// contiguously, optionally transposed [A][B] -> [B][A] through LDS, and written contiguously
// to the row whose (x, y) indices have their sub-indices swapped.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ int swap_slot(int s, int A, int B)
{
    // slot ka*B + kb  ->  natural index ka + A*kb
    return (s / B) + A * (s % B);
}

constexpr int kReorderMaxRow = 8192;   // complex elements of one row that fit the LDS buffer
constexpr int kReorderPad = 264;       // room for one padding element per [B]-row of the row

__global__ __launch_bounds__(kThreads) void k_reorder_rows(ReorderArgs a, int64_t nrows)
{
    __shared__ float2 row[kReorderMaxRow + kReorderPad];
    const int nz = a.n[2];
    const int A = a.A[2], B = a.B[2];
    for (int64_t r = blockIdx.x; r < nrows; r += gridDim.x) {
        int ix = (int)(r / a.n[1]);
        int iy = (int)(r % a.n[1]);
        int ox = a.swap[0] ? swap_slot(ix, a.A[0], a.B[0]) : ix;
        int oy = a.swap[1] ? swap_slot(iy, a.A[1], a.B[1]) : iy;
        const float2* __restrict__ src = a.in + r * (int64_t)nz;
        float2* __restrict__ dst = a.out + ((int64_t)ox * a.n[1] + oy) * (int64_t)nz;
        if (!a.swap[2]) {
            for (int z = threadIdx.x; z < nz; z += kThreads) dst[z] = src[z];
            continue;
        }
        // stage: element at slot s = ka*B + kb is kept at s + ka (one float2 of padding per
        // row of B) so the transposed read below walks ka with an odd stride in LDS
        for (int s = threadIdx.x; s < nz; s += kThreads) row[s + s / B] = src[s];
        __syncthreads();
        for (int k = threadIdx.x; k < nz; k += kThreads) {
            int kb = k / A, ka = k % A;           // natural index k = ka + A*kb
            dst[k] = row[ka * (B + 1) + kb];
        }
        __syncthreads();
    }
}

// Fallback for rows longer than the LDS buffer: one thread per output element, gather.
__global__ __launch_bounds__(kThreads) void k_reorder_gather(ReorderArgs a, int64_t total)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < total; e += stride) {
        int z = (int)(e % a.n[2]);
        int64_t r = e / a.n[2];
        int y = (int)(r % a.n[1]);
        int x = (int)(r / a.n[1]);
        // invert the swap: natural k = ka + A*kb  <-  slot ka*B + kb
        int sx = a.swap[0] ? (x % a.A[0]) * a.B[0] + x / a.A[0] : x;
        int sy = a.swap[1] ? (y % a.A[1]) * a.B[1] + y / a.A[1] : y;
        int sz = a.swap[2] ? (z % a.A[2]) * a.B[2] + z / a.A[2] : z;
        a.out[e] = a.in[((int64_t)sx * a.n[1] + sy) * a.n[2] + sz];
    }
}

template <typename KernelT>
hipError_t launch_tiles(KernelT kernel, const ContractArgs& a, int tilesK, int64_t tilesOther,
                        int64_t total, hipStream_t stream)
{
    if (total <= 0) return hipSuccess;
    if (total > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kernel, dim3((unsigned)total), dim3(kThreads), 0, stream, a, tilesK,
                       tilesOther, total);
    return hipGetLastError();
}

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Picks a tile configuration for one contraction and launches it.  S<...>/C<...> name the
// template arguments (tile, wave tile, chunk); each is instantiated in a fast (whole tiles,
// 16-byte loads) and a masked (any shape) version.
template <int TM, int TN, int WM, int WN, int KC>
hipError_t launch_s(const ContractArgs& a, hipStream_t stream)
{
    const int K = a.M.K, N = a.M.N;
    const int tk = (int)cdiv(K, TM);
    const int64_t ti = cdiv(a.I, TN);
    const int64_t total = (int64_t)tk * ti * a.O;
    const bool whole = (K % TM == 0) && (N % KC == 0) && (a.I % TN == 0);
    if (whole)
        return launch_tiles(k_contract_s<TM, TN, WM, WN, KC, 2, false, 2>, a, tk, ti, total, stream);
    return launch_tiles(k_contract_s<TM, TN, WM, WN, KC, 1, true, 2>, a, tk, ti, total, stream);
}

template <int TO, int TK, int WO, int WK, int KC>
hipError_t launch_c(const ContractArgs& a, hipStream_t stream)
{
    const int K = a.M.K, N = a.M.N;
    const int tk = (int)cdiv(K, TK);
    const int64_t to = cdiv(a.O, TO);
    const int64_t total = (int64_t)tk * to;
    const bool whole = (K % TK == 0) && (N % KC == 0) && (a.O % TO == 0);
    if (whole)
        return launch_tiles(k_contract_c<TO, TK, WO, WK, KC, 2, false, 2>, a, tk, to, total, stream);
    return launch_tiles(k_contract_c<TO, TK, WO, WK, KC, 1, true, 2>, a, tk, to, total, stream);
}

}  // namespace

hipError_t launch_contract(const ContractArgs& a, hipStream_t stream)
{
    const int K = a.M.K, N = a.M.N;
    if (a.O <= 0 || a.I <= 0 || K <= 0 || N <= 0) return hipSuccess;
    constexpr int64_t kFillTiles = 512;   // two workgroups on each of the 256 CUs
    if (a.I == 1) {
        if (N <= 32 && K <= 32) return launch_c<128, 32, 32, 32, 16>(a, stream);
        if (N <= 64 && K <= 64) return launch_c<128, 64, 32, 64, 16>(a, stream);
        if (cdiv(K, 128) * cdiv(a.O, 128) < kFillTiles) return launch_c<64, 64, 32, 32, 16>(a, stream);
        return launch_c<128, 128, 64, 64, 16>(a, stream);
    }
    if (K <= 16 && N <= 16) return launch_s<16, 256, 16, 64, 16>(a, stream);
    if (K <= 32 && N <= 32) return launch_s<32, 128, 32, 32, 16>(a, stream);
    if (K <= 64 && N <= 64) return launch_s<64, 128, 64, 32, 16>(a, stream);
    if (cdiv(K, 128) * cdiv(a.I, 128) * a.O < kFillTiles) return launch_s<64, 64, 32, 32, 16>(a, stream);
    return launch_s<128, 128, 64, 64, 16>(a, stream);
}

hipError_t launch_phase(const float2* in, float2* out, int64_t outer, int A, int B, int64_t inner,
                        const float2* Tw, int conj, hipStream_t stream)
{
    const int64_t total = outer * A * B * inner;
    if (total <= 0) return hipSuccess;
    const bool vec2 = (total % 2 == 0);
    const int64_t nvec = vec2 ? total / 2 : total;
    int64_t blocks = cdiv(nvec, kThreads);
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (vec2)
        hipLaunchKernelGGL(k_phase<2>, dim3((unsigned)blocks), dim3(kThreads), 0, stream, in, out,
                           nvec, A * B, inner, Tw, conj);
    else
        hipLaunchKernelGGL(k_phase<1>, dim3((unsigned)blocks), dim3(kThreads), 0, stream, in, out,
                           nvec, A * B, inner, Tw, conj);
    return hipGetLastError();
}

hipError_t launch_reorder(const ReorderArgs& a, hipStream_t stream)
{
    const int64_t nrows = (int64_t)a.n[0] * a.n[1];
    const int64_t total = nrows * a.n[2];
    if (total <= 0) return hipSuccess;
    // the staged row takes n[2] + A[2] slots when the fastest axis is transposed
    const bool fits = a.n[2] <= kReorderMaxRow && (!a.swap[2] || a.A[2] <= kReorderPad);
    if (fits) {
        int64_t blocks = nrows < 256 * 16 ? nrows : 256 * 16;
        hipLaunchKernelGGL(k_reorder_rows, dim3((unsigned)blocks), dim3(kThreads), 0, stream, a,
                           nrows);
    } else {
        int64_t blocks = cdiv(total, kThreads);
        if (blocks > 256 * 32) blocks = 256 * 32;
        hipLaunchKernelGGL(k_reorder_gather, dim3((unsigned)blocks), dim3(kThreads), 0, stream, a,
                           total);
    }
    return hipGetLastError();
}

}  // namespace dft3d
