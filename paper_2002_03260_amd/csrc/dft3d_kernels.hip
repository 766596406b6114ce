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

// HIP limits a grid dimension to fewer than 2^32 threads; big launches fold the workgroup index
// into (x, y).
__device__ __forceinline__ int64_t linear_block_id()
{
    return (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
}
inline dim3 grid_for(int64_t blocks)
{
    const int64_t kMaxX = 1 << 22;
    if (blocks <= kMaxX) return dim3((unsigned)blocks);
    return dim3((unsigned)kMaxX, (unsigned)((blocks + kMaxX - 1) / kMaxX));
}

__device__ __forceinline__ int64_t out_offset(const ContractArgs& a, int64_t o)
{
    if (a.Olo == 1) return o * a.sYohi;      // (uniform branch: every KDFT mode; saves two 64-bit divisions)
    return (o / a.Olo) * a.sYohi + (o % a.Olo) * a.sYolo;
}

// ------------------------------------------------------------------------------------------
// Mode contraction on fp32 MFMA.  Two kernels share one software pipeline:
//
//   prologue : chunk 0 global -> registers -> LDS[0]; chunk 1 global -> registers; barrier
//   chunk c  : registers (chunk c+1) -> LDS[(c+1)&1]; request chunk c+2 from global memory into
//              the same registers; MFMAs on LDS[c&1] (operands of k-step s+1 are read from LDS
//              while the MFMAs of k-step s issue); barrier
//
// so a global load always has one full chunk of MFMA work to land, and there is one barrier
// per chunk.  The stores and loads of a chunk are cut into pieces of one vector each that sit
// between the groups of MFMAs (the fast path; the masked path does them up front where it has
// no registers to spare).  MASKED = false is the fast path for shapes that are whole multiples of the tile:
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

// B consecutive floats (B = 1, 2, 4; aligned to their total size) in one LDS read
template <int B>
__device__ __forceinline__ void load_floats(float* dst, const float* src)
{
    static_assert(B == 1 || B == 2 || B == 4, "one, two or four floats");
    if constexpr (B == 1) {
        dst[0] = src[0];
    } else if constexpr (B == 2) {
        const f32x2 v = *reinterpret_cast<const f32x2*>(src);
        dst[0] = v.x;
        dst[1] = v.y;
    } else {
        const f32x4 v = *reinterpret_cast<const f32x4*>(src);
        dst[0] = v.x;
        dst[1] = v.y;
        dst[2] = v.z;
        dst[3] = v.w;
    }
}

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
// In the masked version the columns of ALL o are flattened into one index (col = o*I + i), so a
// narrow inner extent (I < TN) still fills the tile; every thread decodes its own (o, i).
template <int TM, int TN, int WM, int WN, int KC, int NB, int EV, bool MASKED, int MINW, int SCHEME>
__global__ __launch_bounds__(kThreads, MINW) void k_contract_s(ContractArgs a, int tilesK,
                                                               int64_t tilesI, int64_t total)
{
    typedef typename CVec<EV>::type xvec;
    constexpr int NWN = TN / WN;
    static_assert((TM / WM) * NWN == 4, "four waves per workgroup");
    static_assert(!MASKED || EV == 1, "the masked path loads single elements");
    constexpr int BM = WM / 16, BN = WN / 16, KS = KC / 4;
    static_assert(BN % 2 == 0, "column blocks are read and stored in pairs");
    constexpr int XP = TN + 16;   // float2 pitch: rows n, n+1 land 32 banks apart (b64 reads conflict-free)
    constexpr int VP = TM + 16;   // float pitch: rows n..n+3 land 16 banks apart
    constexpr int TPR = TN / EV;                  // threads per tile row
    static_assert(kThreads % TPR == 0, "row must divide the workgroup");
    constexpr int XRPP = kThreads / TPR;          // rows per pass
    static_assert(KC % XRPP == 0, "KC must be a multiple of the rows per pass");
    constexpr int XL = KC / XRPP;                 // loads per thread per chunk

    __shared__ __align__(16) float2 Xs[NB][KC][XP];
    __shared__ __align__(16) float Vr[NB][KC][VP];
    __shared__ __align__(16) float Vi[NB][KC][VP];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm0 = (wave / NWN) * WM;
    const int wn0 = (wave % NWN) * WN;
    const int l16 = lane & 15;
    const int lq = lane >> 4;

    // logical tile: k-tile fastest, then column tile (fast path: of one o; masked: of the
    // flattened (o, i) index)
    int64_t t = linear_block_id();
    if (t >= total) return;
    t = xcd_remap(t, total);
    const int kt = (int)(t % tilesK);
    t /= tilesK;
    const int k0 = kt * TM;

    const int N = a.M.N;
    const int64_t I = a.I;
    const int xc = (tid % TPR) * EV;
    const int xr = tid / TPR;

    int64_t tile_o = 0, c0 = 0;       // fast path: the tile's o and first column; masked: first flat column
    bool xcol_ok = true;
    const float2* __restrict__ Xo;    // this thread's column in row n = 0
    if (MASKED) {
        c0 = t * TN;
        const int64_t cg = c0 + xc;
        xcol_ok = cg < a.O * I;
        const int64_t cc = xcol_ok ? cg : 0;
        const int64_t o = cc / I;
        Xo = a.X + o * (int64_t)N * I + (cc - o * I);
    } else {
        tile_o = t / tilesI;
        c0 = (t % tilesI) * TN;
        Xo = a.X + tile_o * (int64_t)N * I + c0 + xc;
    }

    constexpr int VV = KC * TM / 4;               // float4 per matrix plane per chunk
    constexpr int VL = (VV + kThreads - 1) / kThreads;
    xvec xreg[XL];
    f32x4 vrreg[VL], vireg[VL];

    // Global loads and LDS stores of one chunk come in VL + XL pieces each (piece j < VL: both matrix
    // planes' j-th vector, piece VL + j: the j-th data vector), so the main loop can spread them
    // between its MFMAs.
    // Load addresses are a uniform 64-bit base (tile, chunk, piece: scalar registers and scalar
    // arithmetic) plus a 32-bit lane offset that never changes, so the main loop spends no vector
    // instructions on them.  The launcher keeps the fast path to shapes whose lane offsets fit.
    static_assert(kThreads % (TM / 4) == 0, "a piece covers whole matrix rows");
    constexpr int VRP = kThreads / (TM / 4);      // matrix rows per piece
    // (byte offsets, so that the 32-bit value is added to the base as it stands)
    const unsigned v_lane = ((unsigned)(tid / (TM / 4)) * (unsigned)a.M.ld + (unsigned)(tid % (TM / 4)) * 4u) * 4u;
    const unsigned x_lane = ((unsigned)xr * (unsigned)I + (unsigned)xc) * 8u;     // fast path only
    const float2* __restrict__ Xu = a.X + tile_o * (int64_t)N * I + c0;    // fast path only
    auto gload_piece = [&](int n0, int p) {
        if (p < VL) {
            if (VV % kThreads == 0 || tid + p * kThreads < VV) {
                const int64_t base = (int64_t)(n0 + p * VRP) * a.M.ld + k0;
                vrreg[p] = *reinterpret_cast<const f32x4*>(reinterpret_cast<const char*>(a.M.re + base) + v_lane);
                vireg[p] = *reinterpret_cast<const f32x4*>(reinterpret_cast<const char*>(a.M.im + base) + v_lane);
            }
        } else {
            const int j = p - VL;
            if (MASKED) {
                const int n = n0 + xr + j * XRPP;
                const int nn = n < N ? n : N - 1;
                xvec v = *reinterpret_cast<const xvec*>(Xo + (int64_t)nn * I);
                xreg[j] = (xcol_ok && n < N) ? v : cvec_zero<EV>();
            } else {
                const float2* row = Xu + (int64_t)(n0 + j * XRPP) * I;
                xreg[j] = *reinterpret_cast<const xvec*>(reinterpret_cast<const char*>(row) + x_lane);
            }
        }
    };
    const float vsign = a.conj ? -1.0f : 1.0f;
    auto lstore_piece = [&](int buf, int p) {
        if (p < VL) {
            const int f = tid + p * kThreads;
            if (VV % kThreads == 0 || f < VV) {
                const int r = f / (TM / 4), c4 = f % (TM / 4);
                *reinterpret_cast<f32x4*>(&Vr[buf][r][c4 * 4]) = vrreg[p];
                *reinterpret_cast<f32x4*>(&Vi[buf][r][c4 * 4]) = vireg[p] * vsign;
            }
        } else {
            const int j = p - VL;
            *reinterpret_cast<xvec*>(&Xs[buf][xr + j * XRPP][xc]) = xreg[j];
        }
    };
    auto gload = [&](int n0) {
#pragma unroll
        for (int p = 0; p < VL + XL; ++p) gload_piece(n0, p);
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int p = 0; p < VL + XL; ++p) lstore_piece(buf, p);
    };

    // SCHEME 4: accr / acci hold Re / Im.  SCHEME 3 (three real products per complex one):
    // accr = sum Vr*Xr, acci = sum Vi*Xi, acc3 = sum (Vr+Vi)*(Xr+Xi); Re = accr - acci,
    // Im = acc3 - accr - acci.
    constexpr int B3 = (SCHEME == 3) ? BN : 1, M3 = (SCHEME == 3) ? BM : 1;
    f32x4 accr[BM][BN], acci[BM][BN], acc3[M3][B3];
#pragma unroll
    for (int bm = 0; bm < BM; ++bm)
#pragma unroll
        for (int bn = 0; bn < BN; ++bn) {
            accr[bm][bn] = f32x4{0.f, 0.f, 0.f, 0.f};
            acci[bm][bn] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (SCHEME == 3) acc3[bm % M3][bn % B3] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

    const int nchunks = (N + KC - 1) / KC;
    gload(0);
    lstore(0);
    if (NB == 2 && nchunks > 1) gload(KC);
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        const int buf = (NB == 2) ? (c & 1) : 0;
        const bool more = (c + 1) < nchunks;
        if (NB == 1 && more) gload((c + 1) * KC);
        // NB == 2: chunk c+1 was requested one whole chunk ago: it moves to the other LDS buffer now
        // (nobody reads that buffer any more) and chunk c+2 is requested, piece by piece between the
        // groups of MFMAs below.  The pieces run unconditionally so that they stay in the MFMAs' basic
        // block: past the end they store stale registers into the buffer nobody reads any more and
        // load the last chunk again.
        const int n2 = (c + 2 < nchunks ? c + 2 : nchunks - 1) * KC;
        constexpr int NPH = (SCHEME == 3) ? 3 : 4;          // MFMA groups per k-step
        constexpr int NSLOT = KS * NPH, NPIECE = 2 * (VL + XL);
        auto side = [&](int slot) {
            if (NB != 2) return;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < NPIECE; ++p) {
                if (p * NSLOT / NPIECE != slot) continue;
                // a piece's store is followed by the load that refills its registers, so every
                // load has a whole chunk of MFMAs to arrive
                if (p % 2 == 0) lstore_piece(buf ^ 1, p / 2);
                else gload_piece(n2, p / 2);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        // Which tile row an MFMA row stands for, and which tile column an MFMA column, is free as
        // long as the epilogue stores by the same rule.  Row i of block bm is tile row BM*i + bm and
        // columns j of the blocks 2q, 2q+1 are tile columns 32q + 2j, 32q + 2j + 1 of the wave tile,
        // so a lane's operands for all blocks are contiguous in LDS: one read per plane and column pair.
        float ar[2][BM], ai[2][BM];
        f32x2 bx[2][BN];
        auto read_operands = [&](int slot, int s) {
            const int n = 4 * s + lq;
            load_floats<BM>(ar[slot], &Vr[buf][n][wm0 + BM * l16]);
            load_floats<BM>(ai[slot], &Vi[buf][n][wm0 + BM * l16]);
#pragma unroll
            for (int q = 0; q < BN / 2; ++q) {
                const f32x4 x = *reinterpret_cast<const f32x4*>(&Xs[buf][n][wn0 + 32 * q + 2 * l16]);
                bx[slot][2 * q] = f32x2{x.x, x.y};
                bx[slot][2 * q + 1] = f32x2{x.z, x.w};
            }
        };
        read_operands(0, 0);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int cur = s & 1;
            if (s + 1 < KS) read_operands(cur ^ 1, s + 1);
            if (SCHEME == 3) {
                float as[BM], bs[BN];
#pragma unroll
                for (int bm = 0; bm < BM; ++bm) as[bm] = ar[cur][bm] + ai[cur][bm];
#pragma unroll
                for (int bn = 0; bn < BN; ++bn) bs[bn] = bx[cur][bn].x + bx[cur][bn].y;
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < BN; ++bn)
                        accr[bm][bn] = mfma16(ar[cur][bm], bx[cur][bn].x, accr[bm][bn]);
                side(NPH * s);
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < BN; ++bn)
                        acci[bm][bn] = mfma16(ai[cur][bm], bx[cur][bn].y, acci[bm][bn]);
                side(NPH * s + 1);
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < BN; ++bn)
                        acc3[bm % M3][bn % B3] = mfma16(as[bm], bs[bn], acc3[bm % M3][bn % B3]);
                side(NPH * s + 2);
            } else {
                float an[BM];
#pragma unroll
                for (int bm = 0; bm < BM; ++bm) an[bm] = -ai[cur][bm];
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < BN; ++bn)
                        accr[bm][bn] = mfma16(ar[cur][bm], bx[cur][bn].x, accr[bm][bn]);
                side(NPH * s);
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < BN; ++bn)
                        acci[bm][bn] = mfma16(ar[cur][bm], bx[cur][bn].y, acci[bm][bn]);
                side(NPH * s + 1);
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < BN; ++bn)
                        accr[bm][bn] = mfma16(an[bm], bx[cur][bn].y, accr[bm][bn]);
                side(NPH * s + 2);
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < BN; ++bn)
                        acci[bm][bn] = mfma16(ai[cur][bm], bx[cur][bn].x, acci[bm][bn]);
                side(NPH * s + 3);
            }
        }
        if (NB == 1) {
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();                // single buffer: everyone must be done reading it
            if (more) lstore(0);
        }
        __syncthreads();
    }
    // epilogue: scale, optional twiddle, store.  Accumulator register v of block (bm, bn) is MFMA row
    // 4 * lq + v, column l16: tile row BM * (4 * lq + v) + bm, and the blocks 2q, 2q+1 hold two
    // neighbouring columns, stored together (a quarter-wave writes 256 contiguous bytes per row).
    const int K = a.M.K;
    const bool pair_store = !MASKED && (((a.sYk | a.sYohi | a.sYolo) & 1) == 0) &&
                            ((reinterpret_cast<uintptr_t>(a.Y) & 15) == 0);
#pragma unroll
    for (int q = 0; q < BN / 2; ++q) {
        int64_t col[2];
        bool ok[2];
        float2* __restrict__ Yo[2];
        int beta[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            int64_t o = tile_o;
            col[e] = c0 + wn0 + 32 * q + 2 * l16 + e;
            ok[e] = true;
            if (MASKED) {
                ok[e] = col[e] < a.O * I;
                const int64_t cc = ok[e] ? col[e] : 0;
                o = cc / I;
                col[e] = cc - o * I;
            }
            Yo[e] = a.Y + out_offset(a, o);
            beta[e] = a.Tw ? (int)((uint32_t)col[e] / (uint32_t)a.twInner) : 0;   // col < I < 2^31
        }
#pragma unroll
        for (int bm = 0; bm < BM; ++bm) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int k = k0 + wm0 + BM * (4 * lq + v) + bm;
                if (MASKED && k >= K) continue;
                float2 y[2];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int bn = 2 * q + e;
                    float yr, yi;
                    if (SCHEME == 3) {
                        yr = (accr[bm][bn][v] - acci[bm][bn][v]) * a.scale;
                        yi = (acc3[bm % M3][bn % B3][v] - accr[bm][bn][v] - acci[bm][bn][v]) * a.scale;
                    } else {
                        yr = accr[bm][bn][v] * a.scale;
                        yi = acci[bm][bn][v] * a.scale;
                    }
                    if (a.Tw) {
                        float2 w = a.Tw[(int64_t)k * a.twB + beta[e]];
                        if (a.conj) w.y = -w.y;
                        const float tr = yr * w.x - yi * w.y;
                        const float ti = yr * w.y + yi * w.x;
                        yr = tr;
                        yi = ti;
                    }
                    y[e] = make_float2(yr, yi);
                }
                if (pair_store) {
                    // (streaming store: the output is not read again by this kernel; measured 7 % on
                    // the 128^3 contraction, ~1 % at 256^3)
                    __builtin_nontemporal_store(f32x4{y[0].x, y[0].y, y[1].x, y[1].y},
                                                reinterpret_cast<f32x4*>(Yo[0] + (int64_t)k * a.sYk + col[0]));
                } else {
#pragma unroll
                    for (int e = 0; e < 2; ++e)
                        if (ok[e]) Yo[e][(int64_t)k * a.sYk + col[e]] = y[e];
                }
            }
        }
    }
}

// Contiguous-mode contraction (I == 1): out[o, k] = sum_n in[o, n] M[k, n].
// Workgroup tile: TO rows (o) x TK columns (k).  The data tile is the MFMA A operand.
template <int TO, int TK, int WO, int WK, int KC, int EV, bool MASKED, int MINW, int SCHEME>
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

    int64_t t = linear_block_id();
    if (t >= total) return;
    t = xcd_remap(t, total);
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

    // Loads and LDS stores of one chunk in VL + XL pieces (piece j < VL: both matrix planes' j-th
    // vector, piece VL + j: the j-th data vector), spread between the MFMAs of the main loop.  Load
    // addresses: uniform 64-bit base plus a constant 32-bit lane offset in bytes (the launcher keeps
    // the fast path to shapes whose offsets fit).
    static_assert(kThreads % (TK / 4) == 0, "a piece covers whole matrix rows");
    constexpr int VRP = kThreads / (TK / 4);
    const unsigned v_lane = ((unsigned)(tid / (TK / 4)) * (unsigned)a.M.ld + (unsigned)(tid % (TK / 4)) * 4u) * 4u;
    const unsigned x_lane = ((unsigned)xr * (unsigned)N + (unsigned)xc) * 8u;     // fast path only
    auto gload_piece = [&](int n0, int p) {
        if (p < VL) {
            if (VV % kThreads == 0 || tid + p * kThreads < VV) {
                const int64_t base = (int64_t)(n0 + p * VRP) * a.M.ld + k0;
                vrreg[p] = *reinterpret_cast<const f32x4*>(reinterpret_cast<const char*>(a.M.re + base) + v_lane);
                vireg[p] = *reinterpret_cast<const f32x4*>(reinterpret_cast<const char*>(a.M.im + base) + v_lane);
            }
        } else {
            const int j = p - VL;
            if (MASKED) {
                const int64_t orow = o0 + xr + j * XRPP;
                const int n = n0 + xc;
                const int64_t oo = orow < O ? orow : O - 1;
                const int nn = n < N ? n : N - 1;
                xvec v = *reinterpret_cast<const xvec*>(a.X + oo * N + nn);
                xreg[j] = (orow < O && n < N) ? v : cvec_zero<EV>();
            } else {
                const float2* row = a.X + (o0 + j * XRPP) * (int64_t)N + n0;
                xreg[j] = *reinterpret_cast<const xvec*>(reinterpret_cast<const char*>(row) + x_lane);
            }
        }
    };
    const float vsign = a.conj ? -1.0f : 1.0f;
    auto lstore_piece = [&](int buf, int p) {
        if (p < VL) {
            const int f = tid + p * kThreads;
            if (VV % kThreads == 0 || f < VV) {
                const int r = f / (TK / 4), c4 = f % (TK / 4);
                *reinterpret_cast<f32x4*>(&Vr[buf][r][c4 * 4]) = vrreg[p];
                *reinterpret_cast<f32x4*>(&Vi[buf][r][c4 * 4]) = vireg[p] * vsign;
            }
        } else {
            const int j = p - VL;
            float2* dst = &Xs[buf][xr + j * XRPP][xc];     // odd pitch: 8-byte aligned only
            store_cvec(dst, xreg[j]);
        }
    };
    auto gload = [&](int n0) {
#pragma unroll
        for (int p = 0; p < VL + XL; ++p) gload_piece(n0, p);
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int p = 0; p < VL + XL; ++p) lstore_piece(buf, p);
    };

    // SCHEME 4: accr / acci hold Re / Im.  SCHEME 3 (three real products per complex one):
    // accr = sum Vr*Xr, acci = sum Vi*Xi, acc3 = sum (Vr+Vi)*(Xr+Xi); Re = accr - acci,
    // Im = acc3 - accr - acci.
    constexpr int B3 = (SCHEME == 3) ? BN : 1, M3 = (SCHEME == 3) ? BM : 1;
    f32x4 accr[BM][BN], acci[BM][BN], acc3[M3][B3];
#pragma unroll
    for (int bm = 0; bm < BM; ++bm)
#pragma unroll
        for (int bn = 0; bn < BN; ++bn) {
            accr[bm][bn] = f32x4{0.f, 0.f, 0.f, 0.f};
            acci[bm][bn] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (SCHEME == 3) acc3[bm % M3][bn % B3] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

    const int nchunks = (N + KC - 1) / KC;
    gload(0);
    lstore(0);
    if (nchunks > 1) gload(KC);
    __syncthreads();

    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        // Chunk c+1, requested one whole chunk ago, moves to the other LDS buffer and chunk c+2 is
        // requested, piece by piece between the groups of MFMAs.  The pieces run unconditionally so that
        // they stay in the MFMAs' basic block: past the end they store stale registers into the buffer
        // nobody reads any more and load the last chunk again.
        const int n2 = (c + 2 < nchunks ? c + 2 : nchunks - 1) * KC;
        constexpr int NPH = (SCHEME == 3) ? 3 : 4;
        constexpr int NSLOT = KS * NPH, NPIECE = 2 * (VL + XL);
        if (MASKED) {          // (the masked version has no registers to spare for the spreading)
            lstore(buf ^ 1);
            gload(n2);
        }
        auto side = [&](int slot) {
            if (MASKED) return;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < NPIECE; ++p) {
                if (p * NSLOT / NPIECE != slot) continue;
                if (p % 2 == 0) lstore_piece(buf ^ 1, p / 2);
                else gload_piece(n2, p / 2);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        f32x2 ax[2][BM];
        float br[2][BN], bi[2][BN];
        auto read_operands = [&](int slot, int s) {
            const int n = 4 * s + lq;
#pragma unroll
            for (int bm = 0; bm < BM; ++bm)
                ax[slot][bm] = *reinterpret_cast<const f32x2*>(&Xs[buf][wo0 + bm * 16 + l16][n]);
            // column j of block bn is tile column BN * j + bn of the wave tile: a lane's matrix
            // operands for all blocks are contiguous in LDS (the epilogue stores by the same rule)
            load_floats<BN>(br[slot], &Vr[buf][n][wk0 + BN * l16]);
            load_floats<BN>(bi[slot], &Vi[buf][n][wk0 + BN * l16]);
        };
        read_operands(0, 0);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int cur = s & 1;
            if (s + 1 < KS) read_operands(cur ^ 1, s + 1);
            if (SCHEME == 3) {
                float as[BM], bs[BN];
#pragma unroll
                for (int bm = 0; bm < BM; ++bm) as[bm] = ax[cur][bm].x + ax[cur][bm].y;
#pragma unroll
                for (int bn = 0; bn < BN; ++bn) bs[bn] = br[cur][bn] + bi[cur][bn];
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < BN; ++bn)
                        accr[bm][bn] = mfma16(ax[cur][bm].x, br[cur][bn], accr[bm][bn]);
                side(NPH * s);
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < BN; ++bn)
                        acci[bm][bn] = mfma16(ax[cur][bm].y, bi[cur][bn], acci[bm][bn]);
                side(NPH * s + 1);
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < BN; ++bn)
                        acc3[bm % M3][bn % B3] = mfma16(as[bm], bs[bn], acc3[bm % M3][bn % B3]);
                side(NPH * s + 2);
            } else {
                float bneg[BN];
#pragma unroll
                for (int bn = 0; bn < BN; ++bn) bneg[bn] = -bi[cur][bn];
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < BN; ++bn)
                        accr[bm][bn] = mfma16(ax[cur][bm].x, br[cur][bn], accr[bm][bn]);
                side(NPH * s);
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < BN; ++bn)
                        acci[bm][bn] = mfma16(ax[cur][bm].x, bi[cur][bn], acci[bm][bn]);
                side(NPH * s + 1);
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < BN; ++bn)
                        accr[bm][bn] = mfma16(ax[cur][bm].y, bneg[bn], accr[bm][bn]);
                side(NPH * s + 2);
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                    for (int bn = 0; bn < BN; ++bn)
                        acci[bm][bn] = mfma16(ax[cur][bm].y, br[cur][bn], acci[bm][bn]);
                side(NPH * s + 3);
            }
        }
        __syncthreads();
    }

    // epilogue: block bn holds tile columns BN * l16 + bn, so a lane owns BN consecutive k of each of
    // its rows: stored together where the output keeps k contiguous
    const int K = a.M.K;
    const bool run_store = !MASKED && a.sYk == 1 && (((a.sYohi | a.sYolo) & 1) == 0) &&
                           ((reinterpret_cast<uintptr_t>(a.Y) & 15) == 0);
#pragma unroll
    for (int bm = 0; bm < BM; ++bm) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int64_t orow = o0 + wo0 + bm * 16 + 4 * lq + v;
            if (MASKED && orow >= O) continue;
            float2* __restrict__ Yo = a.Y + out_offset(a, orow);
            float2 y[BN];
#pragma unroll
            for (int bn = 0; bn < BN; ++bn) {
                const int k = k0 + wk0 + BN * l16 + bn;
                float yr, yi;
                if (SCHEME == 3) {
                    yr = (accr[bm][bn][v] - acci[bm][bn][v]) * a.scale;
                    yi = (acc3[bm % M3][bn % B3][v] - accr[bm][bn][v] - acci[bm][bn][v]) * a.scale;
                } else {
                    yr = accr[bm][bn][v] * a.scale;
                    yi = acci[bm][bn][v] * a.scale;
                }
                if (a.Tw && (!MASKED || k < K)) {   // I == 1 means beta == 0
                    float2 w = a.Tw[(int64_t)k * a.twB];
                    if (a.conj) w.y = -w.y;
                    const float tr = yr * w.x - yi * w.y;
                    const float ti = yr * w.y + yi * w.x;
                    yr = tr;
                    yi = ti;
                }
                y[bn] = make_float2(yr, yi);
            }
            const int kb = k0 + wk0 + BN * l16;
            if (run_store && BN % 2 == 0) {
#pragma unroll
                for (int bn = 0; bn + 1 < BN; bn += 2)
                    // (plain store: one instruction writes 16 of a lane's 32 contiguous bytes, so with the
                    // streaming hint the halves of a line reach memory separately: 9 % more bytes written)
                    *reinterpret_cast<f32x4*>(Yo + kb + bn) = f32x4{y[bn].x, y[bn].y, y[bn + 1].x, y[bn + 1].y};
            } else {
#pragma unroll
                for (int bn = 0; bn < BN; ++bn)
                    if (!MASKED || kb + bn < K) Yo[(int64_t)(kb + bn) * a.sYk] = y[bn];
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Fused FFT-formulation pass for the contiguous axis: first stage, twiddle, second stage and the
// in-order placement of one axis in a single read and a single write of the tensor.
//
// A workgroup keeps both stage matrices in LDS and walks over tiles of R complete rows
// (R*A*B contiguous complex numbers).  Per tile:
//   1. registers -> xs[row][l][beta]              (the next tile's global loads are issued here,
//                                                  so they land during the MFMA work below)
//   2. stage 1 (data = MFMA B operand): Z[k_a][(row,beta)] = sum_l FA[k_a][l] xs[row][l][beta],
//      times the twiddle T[k_a][beta], written to zs[(row,k_a)][beta]
//   3. stage 2 (data = MFMA A operand): W[(row,k_a)][k_b] = sum_beta zs[(row,k_a)][beta] FB[k_b][beta],
//      written to os[row][k_b][k_a], i.e. at the natural position k_a + A*k_b of the row
//   4. os -> global, contiguous 16-byte stores.
// LDS pitches: xs rows (l) are B+16 apart so the two l-rows a half-wave reads sit 32 banks apart;
// zs and os have odd pitches (B+1, A+1) so lanes that walk rows hit distinct banks.
// ------------------------------------------------------------------------------------------
// Column swizzle (in floats) of row n of an unpadded [P][P] fp32 plane: rows n, n+1, n+2, n+3
// (n a multiple of 4) land on four distinct 16-bank groups.  Depends on n mod 4 only.
template <int P>
__device__ __forceinline__ constexpr int plane_swz(int n)
{
    return P == 64 ? 16 * (n & 3) : (P == 32 ? 16 * ((n >> 1) & 1) : 0);
}

template <int A, int B, int R, int NW, int MINW>
__global__ __launch_bounds__(NW * 64, MINW) void k_fft_z(const float2* __restrict__ X, float2* __restrict__ Y,
                                                   int64_t nrows, DeviceMatrix FA, DeviceMatrix FB,
                                                   const float2* __restrict__ Tw, float scale, int conj)
{
    constexpr int NT = NW * 64;
    constexpr int N = A * B;
    constexpr int XP = B + 16, ZP = B + 1, OP = A + 1, FAP = A + 16, FBP = B + 16;
    constexpr int XS = R * A * XP, OS = R * B * OP;
    constexpr int XOS = XS > OS ? XS : OS;
    constexpr int TILE = R * N;                    // complex numbers per tile
    static_assert(TILE % (2 * NT) == 0, "tile must split into 16-byte loads evenly");
    constexpr int XL = TILE / (2 * NT);            // 16-byte loads per thread per tile
    static_assert(A % 16 == 0 && B % 16 == 0, "stage lengths must be multiples of the MFMA block");

    __shared__ __align__(16) float2 xos[XOS];      // xs, later reused as os
    __shared__ __align__(16) float2 zs[R * A * ZP];
    __shared__ __align__(16) float far[A * FAP], fai[A * FAP];
    __shared__ __align__(16) float fbr[B * FBP], fbi[B * FBP];
    // twiddles T[k_a][beta] in LDS when there is room: a global load inside the tile loop would
    // queue behind the next tile's prefetch (loads return in order) and stall stage 1 on it
    constexpr bool TWL = (A * B <= 2048);
    __shared__ __align__(16) float2 tws[TWL ? A * B : 1];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l16 = lane & 15;
    const int lq = lane >> 4;
    const float isign = conj ? -1.0f : 1.0f;

    // stage matrices -> LDS (transposed planes [n][k], as stored on the device)
    for (int e = tid; e < A * A; e += NT) {
        const int n = e / A, k = e % A;
        far[n * FAP + k] = FA.re[(int64_t)n * FA.ld + k];
        fai[n * FAP + k] = FA.im[(int64_t)n * FA.ld + k] * isign;
    }
    for (int e = tid; e < B * B; e += NT) {
        const int n = e / B, k = e % B;
        fbr[n * FBP + k] = FB.re[(int64_t)n * FB.ld + k];
        fbi[n * FBP + k] = FB.im[(int64_t)n * FB.ld + k] * isign;
    }

    if (TWL)
        for (int e = tid; e < A * B; e += NT) tws[e] = Tw[e];
    const float2* tw_src = TWL ? tws : Tw;

    const int64_t ntiles = (nrows + R - 1) / R;
    const int64_t nwg = (int64_t)gridDim.x * gridDim.y;
    f32x4 xreg[XL];
    auto gload = [&](int64_t tile) {
        const int64_t base = tile * TILE;
        const int64_t limit = nrows * N;           // first element past the tensor
#pragma unroll
        for (int j = 0; j < XL; ++j) {
            const int64_t e = base + 2 * (tid + j * NT);
            xreg[j] = (e < limit) ? __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(X + e))
                                  : f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };

    int64_t tile = linear_block_id();
    if (tile < ntiles) gload(tile);
    for (; tile < ntiles; tile += nwg) {
        // 1. registers -> xs
#pragma unroll
        for (int j = 0; j < XL; ++j) {
            const int e = 2 * (tid + j * NT);
            const int rl = e / B, beta = e % B;     // rl = row*A + l
            *reinterpret_cast<f32x4*>(&xos[rl * XP + beta]) = xreg[j];
        }
        __syncthreads();
        if (tile + nwg < ntiles) gload(tile + nwg);

        // 2. stage 1: blocks over (row, k_a block, beta block)
        constexpr int S1 = R * (A / 16) * (B / 16);
        constexpr int U1 = (S1 % (2 * NW) == 0) ? 2 : 1;      // blocks in flight per wave
        for (int b0 = wave * U1; b0 < S1; b0 += NW * U1) {
            int bb[U1], bm[U1], row[U1];
            float2 tw[U1][4];
            f32x4 cr[U1], ci[U1];
#pragma unroll
            for (int u = 0; u < U1; ++u) {
                const int b = b0 + u;
                bb[u] = b % (B / 16);
                bm[u] = (b / (B / 16)) % (A / 16);
                row[u] = b / ((B / 16) * (A / 16));
                cr[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                ci[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int v = 0; v < 4; ++v)      // requested now, needed after the MFMAs
                    tw[u][v] = TWL ? tws[(bm[u] * 16 + 4 * lq + v) * B + bb[u] * 16 + l16]
                                   : tw_src[(bm[u] * 16 + 4 * lq + v) * B + bb[u] * 16 + l16];
            }
#pragma unroll
            for (int s = 0; s < A / 4; ++s) {
                const int l = 4 * s + lq;
                float ar[U1], ai[U1];
                f32x2 x[U1];
#pragma unroll
                for (int u = 0; u < U1; ++u) {
                    ar[u] = far[l * FAP + bm[u] * 16 + l16];
                    ai[u] = fai[l * FAP + bm[u] * 16 + l16];
                    x[u] = *reinterpret_cast<const f32x2*>(&xos[(row[u] * A + l) * XP + bb[u] * 16 + l16]);
                }
#pragma unroll
                for (int u = 0; u < U1; ++u) cr[u] = mfma16(ar[u], x[u].x, cr[u]);
#pragma unroll
                for (int u = 0; u < U1; ++u) ci[u] = mfma16(ar[u], x[u].y, ci[u]);
#pragma unroll
                for (int u = 0; u < U1; ++u) cr[u] = mfma16(-ai[u], x[u].y, cr[u]);
#pragma unroll
                for (int u = 0; u < U1; ++u) ci[u] = mfma16(ai[u], x[u].x, ci[u]);
            }
#pragma unroll
            for (int u = 0; u < U1; ++u) {
                const int beta = bb[u] * 16 + l16;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int ka = bm[u] * 16 + 4 * lq + v;
                    const float wx = tw[u][v].x, wy = tw[u][v].y * isign;
                    zs[(row[u] * A + ka) * ZP + beta] =
                        make_float2(cr[u][v] * wx - ci[u][v] * wy, cr[u][v] * wy + ci[u][v] * wx);
                }
            }
        }
        __syncthreads();

        // 3. stage 2: blocks over ((row,k_a) block, k_b block); xs is dead, os takes its place
        constexpr int S2 = (R * A / 16) * (B / 16);
        constexpr int U2 = (S2 % (2 * NW) == 0) ? 2 : 1;
        for (int b0 = wave * U2; b0 < S2; b0 += NW * U2) {
            int bn[U2], bmz[U2];
            f32x4 cr[U2], ci[U2];
#pragma unroll
            for (int u = 0; u < U2; ++u) {
                bn[u] = (b0 + u) % (B / 16);
                bmz[u] = (b0 + u) / (B / 16);
                cr[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                ci[u] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int s = 0; s < B / 4; ++s) {
                const int beta = 4 * s + lq;
                f32x2 z[U2];
                float br[U2], bi[U2];
#pragma unroll
                for (int u = 0; u < U2; ++u) {
                    z[u] = *reinterpret_cast<const f32x2*>(&zs[(bmz[u] * 16 + l16) * ZP + beta]);
                    br[u] = fbr[beta * FBP + bn[u] * 16 + l16];
                    bi[u] = fbi[beta * FBP + bn[u] * 16 + l16];
                }
#pragma unroll
                for (int u = 0; u < U2; ++u) cr[u] = mfma16(z[u].x, br[u], cr[u]);
#pragma unroll
                for (int u = 0; u < U2; ++u) ci[u] = mfma16(z[u].x, bi[u], ci[u]);
#pragma unroll
                for (int u = 0; u < U2; ++u) cr[u] = mfma16(z[u].y, -bi[u], cr[u]);
#pragma unroll
                for (int u = 0; u < U2; ++u) ci[u] = mfma16(z[u].y, br[u], ci[u]);
            }
#pragma unroll
            for (int u = 0; u < U2; ++u) {
                const int kb = bn[u] * 16 + l16;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int m = bmz[u] * 16 + 4 * lq + v;         // (row, k_a)
                    const int row = m / A, ka = m % A;
                    xos[(row * B + kb) * OP + ka] = make_float2(cr[u][v] * scale, ci[u][v] * scale);
                }
            }
        }
        __syncthreads();

        // 4. os -> global in natural order (k = k_a + A*k_b), two complex numbers per store
        {
            const int64_t base = tile * TILE;
            const int64_t limit = nrows * N;
#pragma unroll
            for (int j = 0; j < XL; ++j) {
                const int e = 2 * (tid + j * NT);
                const int row = e / N, k = e % N;
                const int kb = k / A, ka = k % A;          // k even, A even: k+1 is the next k_a
                const float2 p0 = xos[(row * B + kb) * OP + ka];
                const float2 p1 = xos[(row * B + kb) * OP + ka + 1];
                if (base + e < limit)
                    __builtin_nontemporal_store(f32x4{p0.x, p0.y, p1.x, p1.y}, reinterpret_cast<f32x4*>(Y + base + e));
            }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------
// Twiddle multiply (memory-bound).  The tensor [outer][A][B][inner] is walked as a matrix whose
// twiddle depends on the row only (inner > 1: rows = outer*A*B, columns = inner, factor
// Tw[row % (A*B)]) or on the column only (inner == 1: rows = outer, columns = A*B, factor
// Tw[col]); either way the per-element index arithmetic is 32-bit.  Each thread moves EV complex
// numbers (EV = 2 -> 16 bytes) and each workgroup one 4 KiB chunk, launched in memory order --
// the launch shape that gave the best plain-copy bandwidth on this chip.
// ------------------------------------------------------------------------------------------
template <int EV, bool BY_ROW>
__global__ __launch_bounds__(kThreads) void k_phase(const float2* __restrict__ in,
                                                    float2* __restrict__ out, int64_t rows,
                                                    int cols, int chunks_per_row, int AB,
                                                    const float2* __restrict__ Tw, int conj)
{
    typedef typename CVec<EV>::type xvec;
    // one workgroup = one chunk of kThreads*EV columns of one row, launched in memory order
    const int64_t bid = linear_block_id();
    const int64_t r = bid / chunks_per_row;
    const int c = (int)(bid % chunks_per_row) * (kThreads * EV) + threadIdx.x * EV;
    if (r >= rows || c >= cols) return;
    const float s = conj ? -1.0f : 1.0f;
    const xvec x = __builtin_nontemporal_load(reinterpret_cast<const xvec*>(in + r * cols + c));
    float2 wr = make_float2(1.f, 0.f);
    if (BY_ROW) {
        wr = Tw[(int)(r % AB)];
        wr.y *= s;
    }
    xvec y;
#pragma unroll
    for (int e = 0; e < EV; ++e) {
        float2 w = wr;
        if (!BY_ROW) {
            w = Tw[c + e];
            w.y *= s;
        }
        y[2 * e] = x[2 * e] * w.x - x[2 * e + 1] * w.y;
        y[2 * e + 1] = x[2 * e] * w.y + x[2 * e + 1] * w.x;
    }
    __builtin_nontemporal_store(y, reinterpret_cast<xvec*>(out + r * cols + c));
}

// ------------------------------------------------------------------------------------------
// Re-ordering.  The swap of the x and y sub-indices only changes which output row an input row
// goes to; the swap of the z sub-indices is a transposition [A][B] -> [B][A] inside each
// contiguous row, done through LDS.  A workgroup produces a batch of G consecutive output rows
// (G * nz contiguous complex numbers): it reads the input rows that land there with EV-wide
// accesses and writes the batch contiguously.  In LDS the element at slot s = ka*B + kb of batch row g sits at
// g*(nz + A) + s + ka: one padding element per B-row, so the transposed read walks ka with the
// odd stride B + 1 and consecutive lanes hit distinct banks.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ int unswap_slot(int k, int A, int B)
{
    // natural index ka + A*kb  ->  slot ka*B + kb
    return (k % A) * B + k / A;
}

// T = threads per workgroup (long rows take 1024: they are few, large workgroups)
template <int CAP, int EV, int T>
__global__ __launch_bounds__(T) void k_reorder_rows(ReorderArgs a, int64_t nrows, int G)
{
    typedef typename CVec<EV>::type xvec;
    __shared__ __align__(16) float2 buf[CAP];
    const int nz = a.n[2];
    const int A = a.A[2], B = a.B[2];
    const int pitch = nz + A;
    // One batch of G consecutive OUTPUT rows per workgroup, launched in output order: the writes
    // of the whole grid stream through memory contiguously and the reads gather whole input rows
    // (reads tolerate the scatter better than writes do).
    const int64_t b = linear_block_id();
    const int64_t r0 = b * G;
    if (r0 >= nrows) return;
    const int g_here = (int)((nrows - r0) < G ? (nrows - r0) : G);
    const int count = g_here * nz;
    float2* __restrict__ dst = a.out + r0 * (int64_t)nz;
    auto source_row = [&](int64_t r) {   // input row that lands in output row r
        const int ox = (int)(r / a.n[1]), oy = (int)(r % a.n[1]);
        const int ix = a.swap[0] ? unswap_slot(ox, a.A[0], a.B[0]) : ox;
        const int iy = a.swap[1] ? unswap_slot(oy, a.A[1], a.B[1]) : oy;
        return a.in + ((int64_t)ix * a.n[1] + iy) * (int64_t)nz;
    };
    if (!a.swap[2]) {
        // rows keep their content: copy each from its permuted place
        for (int e = threadIdx.x * EV; e < count; e += T * EV) {
            const int g = e / nz, z = e - g * nz;
            __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const xvec*>(source_row(r0 + g) + z)),
                                        reinterpret_cast<xvec*>(dst + e));
        }
        return;
    }
    for (int e = threadIdx.x * EV; e < count; e += T * EV) {
        const int g = e / nz, s = e - g * nz;
        const xvec v = __builtin_nontemporal_load(reinterpret_cast<const xvec*>(source_row(r0 + g) + s));
        store_cvec(&buf[g * pitch + s + s / B], v);   // s and s+1 share a B-row (B even when EV == 2)
    }
    __syncthreads();
    for (int e = threadIdx.x * EV; e < count; e += T * EV) {
        const int g = e / nz, k = e - g * nz;          // natural index k = ka + A*kb
        const int kb = k / A, ka = k - kb * A;
        const float2* p = &buf[g * pitch + ka * (B + 1) + kb];
        xvec v;
#pragma unroll
        for (int q = 0; q < EV; ++q) {                 // k+1 is the next ka (A even when EV == 2)
            const float2 t = p[q * (B + 1)];
            v[2 * q] = t.x;
            v[2 * q + 1] = t.y;
        }
        __builtin_nontemporal_store(v, reinterpret_cast<xvec*>(dst + e));
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
    hipLaunchKernelGGL(kernel, grid_for(total), dim3(kThreads), 0, stream, a, tilesK, tilesOther, total);
    return hipGetLastError();
}

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Picks a tile configuration for one contraction and launches it.  S<...>/C<...> name the
// template arguments (tile, wave tile, chunk); each is instantiated in a fast (whole tiles,
// 16-byte loads) and a masked (any shape) version.
template <int TM, int TN, int WM, int WN, int KC, int NB, int SCHEME = 4, int MINW = 2>
hipError_t launch_s(const ContractArgs& a, hipStream_t stream)
{
    const int K = a.M.K, N = a.M.N;
    const int tk = (int)cdiv(K, TM);
    // (the fast path addresses its loads with 32-bit lane offsets of up to 8 rows of I elements)
    const bool whole = (K % TM == 0) && (N % KC == 0) && (a.I % TN == 0) && a.I < (1 << 25) &&
                       a.M.ld < (1 << 21);
    if (whole) {
        const int64_t ti = a.I / TN;
        const int64_t total = (int64_t)tk * ti * a.O;
        return launch_tiles(k_contract_s<TM, TN, WM, WN, KC, NB, 2, false, MINW, SCHEME>, a, tk, ti, total, stream);
    }
    // masked: column tiles run over the flattened (o, i) index
    const int64_t tc = cdiv(a.O * a.I, TN);
    return launch_tiles(k_contract_s<TM, TN, WM, WN, KC, NB, 1, true, MINW, SCHEME>, a, tk, tc, (int64_t)tk * tc, stream);
}

template <int TO, int TK, int WO, int WK, int KC, int SCHEME = 4>
hipError_t launch_c(const ContractArgs& a, hipStream_t stream)
{
    const int K = a.M.K, N = a.M.N;
    const int tk = (int)cdiv(K, TK);
    const int64_t to = cdiv(a.O, TO);
    const int64_t total = (int64_t)tk * to;
    // (the fast path addresses its loads with 32-bit lane offsets of up to 64 rows of N elements)
    const bool whole = (K % TK == 0) && (N % KC == 0) && (a.O % TO == 0) && N < (1 << 22) && a.M.ld < (1 << 21);
    if (whole)
        return launch_tiles(k_contract_c<TO, TK, WO, WK, KC, 2, false, 2, SCHEME>, a, tk, to, total, stream);
    return launch_tiles(k_contract_c<TO, TK, WO, WK, KC, 1, true, 2, SCHEME>, a, tk, to, total, stream);
}

}  // namespace

// One decision procedure serves the launch and the query of which kernel a contraction takes: with
// `name` set nothing is launched and *name receives the kernel family.
static hipError_t dispatch_contract(const ContractArgs& a, hipStream_t stream, const char** name)
{
#define DFT3D_PICK(family, call)                \
    do {                                        \
        if (name) {                             \
            *name = family;                     \
            return hipSuccess;                  \
        }                                       \
        return call;                            \
    } while (0)
    const int K = a.M.K, N = a.M.N;
    if (a.O <= 0 || a.I <= 0 || K <= 0 || N <= 0) DFT3D_PICK("none", hipSuccess);
    if (a.bf16x3 && contract_bf16x3_supported(a)) DFT3D_PICK("k_contract_bf16x3", launch_contract_bf16x3(a, stream));
    constexpr int64_t kFillTiles = 512;   // two workgroups on each of the 256 CUs
    if (a.I == 1) {
        if (N <= 32 && K <= 32) DFT3D_PICK("k_contract_c", (launch_c<128, 32, 32, 32, 16>(a, stream)));
        if (N <= 64 && K <= 64) DFT3D_PICK("k_contract_c", (launch_c<128, 64, 32, 64, 16>(a, stream)));
        if (cdiv(K, 128) * cdiv(a.O, 128) < kFillTiles) DFT3D_PICK("k_contract_c", (launch_c<64, 64, 32, 32, 16>(a, stream)));
        if (a.three_m) DFT3D_PICK("k_contract_c (3M)", (launch_c<128, 64, 64, 32, 16, 3>(a, stream)));
        DFT3D_PICK("k_contract_c", (launch_c<128, 128, 64, 64, 16>(a, stream)));
    }
    // 64-point first stages of the FFT formulation (24 flop per byte: at the ridge) run faster on the
    // LDS-tiled three-product kernel than on the streaming one (8192 = 64 * 128: 0.39 -> 0.34 ms)
    if (K == 64 && N == 64 && a.Tw && a.Olo == 1 && a.I % 128 == 0)
        DFT3D_PICK("k_contract_s (3M)", (launch_s<64, 128, 32, 64, 16, 2, 3>(a, stream)));
    if (contract_sr_supported(a)) DFT3D_PICK("k_contract_sr", launch_contract_sr(a, stream));
    if (K <= 16 && N <= 16) DFT3D_PICK("k_contract_s", (launch_s<16, 256, 16, 64, 16, 1>(a, stream)));
    if (K <= 32 && N <= 32) DFT3D_PICK("k_contract_s", (launch_s<32, 128, 32, 32, 32, 1>(a, stream)));
    if (K <= 64 && N <= 64) DFT3D_PICK("k_contract_s", (launch_s<64, 128, 64, 32, 16, 2>(a, stream)));
    if (cdiv(K, 128) * cdiv(a.I, 128) * a.O < kFillTiles) DFT3D_PICK("k_contract_s", (launch_s<64, 64, 32, 32, 16, 2>(a, stream)));
    if (a.three_m) DFT3D_PICK("k_contract_s (3M)", (launch_s<64, 128, 32, 64, 16, 2, 3>(a, stream)));
    DFT3D_PICK("k_contract_s", (launch_s<128, 128, 64, 64, 16, 2>(a, stream)));
#undef DFT3D_PICK
}

hipError_t launch_contract(const ContractArgs& a, hipStream_t stream) { return dispatch_contract(a, stream, nullptr); }

const char* contract_kernel_name(const ContractArgs& a)
{
    const char* name = "none";
    (void)dispatch_contract(a, nullptr, &name);
    return name;
}

namespace {
// Plain copy, 16 bytes per lane, UNROLL independent accesses per thread: the achievable-bandwidth
// reference for the memory-bound passes and the calibration kernel for the HBM byte counters.
// STREAM: loads and stores carry the streaming (non-temporal) hint, as in the memory-bound passes.
template <int UNROLL, bool STREAM>
__global__ __launch_bounds__(kThreads) void k_copy(const f32x4* __restrict__ in, f32x4* __restrict__ out,
                                                   int64_t nvec)
{
    const int64_t chunk = (int64_t)kThreads * UNROLL;
    const int64_t nblocks = (int64_t)gridDim.x * gridDim.y;
    for (int64_t base = linear_block_id() * chunk; base < nvec; base += nblocks * chunk) {
        f32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t i = base + threadIdx.x + (int64_t)u * kThreads;
            if (i < nvec) v[u] = STREAM ? __builtin_nontemporal_load(in + i) : in[i];
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t i = base + threadIdx.x + (int64_t)u * kThreads;
            if (i < nvec) {
                if (STREAM) __builtin_nontemporal_store(v[u], out + i);
                else out[i] = v[u];
            }
        }
    }
}
}  // namespace

namespace {
template <int A, int B, int R, int NW, int MINW, int WGS_PER_CU>
hipError_t launch_fft_z_inst(const float2* in, float2* out, int64_t nrows, const DeviceMatrix& FA,
                             const DeviceMatrix& FB, const float2* Tw, float scale, int conj,
                             hipStream_t stream)
{
    const int64_t ntiles = cdiv(nrows, R);
    const int64_t resident = 256 * WGS_PER_CU;             // persistent workgroups
    const int64_t blocks = ntiles < resident ? ntiles : resident;
    hipLaunchKernelGGL((k_fft_z<A, B, R, NW, MINW>), grid_for(blocks), dim3(NW * 64), 0, stream, in, out, nrows,
                       FA, FB, Tw, scale, conj);
    return hipGetLastError();
}
}  // namespace

bool fft_z_supported(int A, int B)
{
    return fft_zr_supported(A, B) || fft_zn_supported(A, B) || (A == 64 && B == 64);
}

hipError_t launch_fft_z(const float2* in, float2* out, int64_t nrows, int A, int B,
                        const DeviceMatrix& FA, const DeviceMatrix& FB, const float2* Tw, float scale,
                        int conj, hipStream_t stream)
{
    if (nrows <= 0) return hipSuccess;
    // the register-resident kernels cover every offered split but 64 x 64
    if (fft_zn_supported(A, B)) return launch_fft_zn(in, out, nrows, A, B, FA, FB, Tw, scale, conj, stream);
    if (fft_zr_supported(A, B)) return launch_fft_zr(in, out, nrows, A, B, FA, FB, Tw, scale, conj, stream);
    if (A == 64 && B == 64) return launch_fft_z_inst<64, 64, 1, 8, 2, 1>(in, out, nrows, FA, FB, Tw, scale, conj, stream);
    return hipErrorInvalidValue;
}

// Strided axes: every fused kernel lives in dft3d_fft_reg.hip / dft3d_fft_nested.hip.
bool fft_s_supported(int A, int B, int64_t I)
{
    return fft_sr_supported(A, B, I);
}

hipError_t launch_fft_s(const float2* in, float2* out, int64_t O, int64_t I, int A, int B,
                        const DeviceMatrix& FA, const DeviceMatrix& FB, const float2* Tw, float scale,
                        int conj, hipStream_t stream)
{
    if (O <= 0 || I <= 0) return hipSuccess;
    return launch_fft_sr(in, out, O, I, A, B, FA, FB, Tw, scale, conj, stream);
}

hipError_t launch_copy(const void* in, void* out, size_t bytes, int variant, hipStream_t stream)
{
    const int64_t nvec = (int64_t)(bytes / 16);
    if (nvec <= 0) return hipSuccess;
    // variant = 100 * streaming + 10 * (workgroups per 256, 0 = one chunk each) + unroll code
    const bool streaming = variant >= 100;
    variant %= 100;
    const int unroll = (variant % 10 == 1) ? 1 : ((variant % 10 == 2) ? 2 : 4);
    const int64_t chunk = (int64_t)kThreads * unroll;
    int64_t blocks = cdiv(nvec, chunk);
    const int cap = variant >= 10 ? 256 * (variant / 10) : 0;     // 0: one chunk per workgroup
    if (cap > 0 && blocks > cap) blocks = cap;
    const dim3 grid = grid_for(blocks), block(kThreads);
    const f32x4* src = (const f32x4*)in;
    f32x4* dst = (f32x4*)out;
    if (streaming) {
        if (unroll == 1) hipLaunchKernelGGL((k_copy<1, true>), grid, block, 0, stream, src, dst, nvec);
        else if (unroll == 2) hipLaunchKernelGGL((k_copy<2, true>), grid, block, 0, stream, src, dst, nvec);
        else hipLaunchKernelGGL((k_copy<4, true>), grid, block, 0, stream, src, dst, nvec);
    } else {
        if (unroll == 1) hipLaunchKernelGGL((k_copy<1, false>), grid, block, 0, stream, src, dst, nvec);
        else if (unroll == 2) hipLaunchKernelGGL((k_copy<2, false>), grid, block, 0, stream, src, dst, nvec);
        else hipLaunchKernelGGL((k_copy<4, false>), grid, block, 0, stream, src, dst, nvec);
    }
    return hipGetLastError();
}

hipError_t launch_phase(const float2* in, float2* out, int64_t outer, int A, int B, int64_t inner,
                        const float2* Tw, int conj, hipStream_t stream)
{
    const int64_t total = outer * A * B * inner;
    if (total <= 0) return hipSuccess;
    const int AB = A * B;
    const bool by_row = inner > 1;
    const int64_t rows = by_row ? outer * AB : outer;
    const int cols = by_row ? (int)inner : AB;
    const bool vec2 = (cols % 2 == 0);
    const int per_wg = kThreads * (vec2 ? 2 : 1);
    const int cpr = (int)cdiv(cols, per_wg);
    const int64_t blocks = rows * cpr;
    const dim3 grid = grid_for(blocks), block(kThreads);
    if (by_row) {
        if (vec2) hipLaunchKernelGGL((k_phase<2, true>), grid, block, 0, stream, in, out, rows, cols, cpr, AB, Tw, conj);
        else hipLaunchKernelGGL((k_phase<1, true>), grid, block, 0, stream, in, out, rows, cols, cpr, AB, Tw, conj);
    } else {
        if (vec2) hipLaunchKernelGGL((k_phase<2, false>), grid, block, 0, stream, in, out, rows, cols, cpr, AB, Tw, conj);
        else hipLaunchKernelGGL((k_phase<1, false>), grid, block, 0, stream, in, out, rows, cols, cpr, AB, Tw, conj);
    }
    return hipGetLastError();
}

namespace {
template <int CAP>
hipError_t launch_reorder_rows(const ReorderArgs& a, int64_t nrows, hipStream_t stream)
{
    const int nz = a.n[2];
    const int pitch = nz + a.A[2];
    // a batch of about 1024 complex numbers (8 KiB, two 16-byte accesses per thread in flight), whole
    // rows: measured on 512^3 0.387 ms with 4 KiB batches, 0.335 ms with 8 KiB, 0.364 ms with 16 KiB
    int G = 1024 / nz;
    if (G > CAP / pitch) G = CAP / pitch;
    if (G < 1) G = 1;
    const int64_t blocks = (nrows + G - 1) / G;
    const bool vec2 = (nz % 2 == 0) && (!a.swap[2] || (a.A[2] % 2 == 0 && a.B[2] % 2 == 0));
    constexpr int T = CAP > 4096 ? 1024 : kThreads;
    if (vec2)
        hipLaunchKernelGGL((k_reorder_rows<CAP, 2, T>), grid_for(blocks), dim3(T), 0, stream, a, nrows, G);
    else
        hipLaunchKernelGGL((k_reorder_rows<CAP, 1, T>), grid_for(blocks), dim3(T), 0, stream, a, nrows, G);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_reorder(const ReorderArgs& a, hipStream_t stream)
{
    const int64_t nrows = (int64_t)a.n[0] * a.n[1];
    const int64_t total = nrows * a.n[2];
    if (total <= 0) return hipSuccess;
    const int need = a.n[2] + a.A[2];      // LDS slots of one staged row
    if (need <= 2304) return launch_reorder_rows<2304>(a, nrows, stream);      // 18 KiB: 8 workgroups per CU
    if (need <= 8448) return launch_reorder_rows<8448>(a, nrows, stream);      // 66 KiB: 2 per CU
    int64_t blocks = cdiv(total, kThreads);
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(k_reorder_gather, dim3((unsigned)blocks), dim3(kThreads), 0, stream, a, total);
    return hipGetLastError();
}

}  // namespace dft3d
