// Mode contraction in double precision (complex128 tensors) on the fp64 matrix cores of gfx950
// (v_mfma_f64_16x16x4_f64): the same mode-wise dense contraction as the single-precision path
// (paper Eq. 6, per-mode products with the transform matrix), for callers that need the
// float64 accuracy the paper names as future work (Section VI).
//
// One kernel serves both contraction types:  out[row, col] = sum_n R[row, n] C[col, n]
//   strided modes   : R = matrix (rows = k), C = data (cols = the contiguous index i)
//   contiguous mode : R = data (rows = o),   C = matrix (cols = k)
// A workgroup is 4 waves on a 64 x 64 tile (each wave 32 x 32 = 2 x 2 MFMA blocks), the contracted
// index advances in chunks of 16 through double-buffered LDS planes [n][row or col] (re and im apart),
// filled from registers that were loaded one chunk earlier.  The complex product takes four real
// MFMAs per block, each into an accumulator of its own; signs and conjugation are applied once, in
// the epilogue.  Two workgroups fit a CU (64 KiB LDS each), so one workgroup's staging and barriers
// hide behind the other's MFMAs.  Shapes that are whole tiles take a path without masks (FAST).
//
// MFMA operand layout (checked on hardware): A[i = lane % 16][k = lane / 16], B[k = lane / 16][j = lane % 16],
// D register v of a lane = row 4 * v + lane / 16, column lane % 16.
#include <hip/hip_runtime.h>

#include "dft3d_internal.h"

namespace dft3d {

namespace {

typedef double f64x2 __attribute__((ext_vector_type(2)));
typedef double f64x4 __attribute__((ext_vector_type(4)));

constexpr int kT = 256;
constexpr int TM = 64, TN = 64, KC = 16;

__device__ __forceinline__ int64_t block_id() { return (int64_t)blockIdx.y * gridDim.x + blockIdx.x; }

__device__ __forceinline__ int64_t remap(int64_t wg, int64_t total)
{
    constexpr int64_t kXcds = 8;
    if (total % kXcds != 0) return wg;
    return (wg % kXcds) * (total / kXcds) + wg / kXcds;
}

__device__ __forceinline__ int64_t y_offset(const ContractArgs64& a, int64_t o)
{
    if (a.Olo == 1) return o * a.sYohi;
    return (o / a.Olo) * a.sYohi + (o % a.Olo) * a.sYolo;
}

__device__ __forceinline__ f64x4 mfma_f64(double a, double b, f64x4 c)
{
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

// FAST: the shape is a whole number of tiles and chunks, so loads need no masks and their addresses
// are a uniform 64-bit base plus a constant 32-bit lane offset in bytes.
template <bool STRIDED, bool FAST>
__global__ __launch_bounds__(kT, 2) void k_contract_f64(ContractArgs64 a, int tilesK, int64_t tilesOther,
                                                        int64_t total)
{
    // [buffer][part: re, im][n][row or col]
    __shared__ double RT[2][2][KC][TM];
    __shared__ double CT[2][2][KC][TN];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wr0 = (wave >> 1) * 32;      // wave tile origin inside the 64 x 64 tile
    const int wc0 = (wave & 1) * 32;
    const int l16 = lane & 15;
    const int lq = lane >> 4;

    int64_t t = block_id();
    if (t >= total) return;
    t = remap(t, total);
    const int kt = (int)(t % tilesK);
    t /= tilesK;
    const int k0 = kt * 64;

    const int N = a.N, K = a.K;
    const int64_t I = a.I;
    const int ld = a.ld;
    const int64_t plane = (int64_t)a.rows * ld;

    // matrix tile: 16 n x 64 k per chunk; this thread: n = tid / 16, four consecutive k (zero padded planes: no masks)
    const int vn = tid >> 4, vk = (tid & 15) * 4;
    const double* vsrc = a.M + (int64_t)vn * ld + k0 + vk;

    // data tile
    int64_t tile_o = 0, c0 = 0, o0 = 0;
    const f64x2* xsrc;
    int xa, xb;          // strided: n = xa, columns xb..xb+3;  contiguous: row = xa, n = xb..xb+3
    bool xok[4];         // strided: column xb+e exists;  contiguous: row exists (all four equal)
    int xcol[4];         // strided: column of element e inside its row of I, 0 where it does not exist
    if (STRIDED) {
        tile_o = t / tilesOther;
        c0 = (t % tilesOther) * TN;
        xa = tid >> 4;
        xb = (tid & 15) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            xok[e] = c0 + xb + e < I;
            xcol[e] = xok[e] ? (int)(c0 + xb + e) : 0;
        }
        xsrc = reinterpret_cast<const f64x2*>(a.X) + tile_o * (int64_t)N * I;
    } else {
        o0 = t * TM;
        xa = tid >> 2;
        xb = (tid & 3) * 4;
        const bool ok = o0 + xa < a.O;
#pragma unroll
        for (int e = 0; e < 4; ++e) xok[e] = ok;
        xsrc = reinterpret_cast<const f64x2*>(a.X) + (ok ? o0 + xa : 0) * (int64_t)N;
    }

    // FAST: lane offsets in bytes (the launcher checks that they fit 32 bits)
    const unsigned v_lane = ((unsigned)vn * (unsigned)ld + (unsigned)vk) * 8u;
    const unsigned x_lane = STRIDED ? ((unsigned)xa * (unsigned)I + (unsigned)xb) * 16u
                                    : ((unsigned)xa * (unsigned)N + (unsigned)xb) * 16u;
    const f64x2* xu = STRIDED ? reinterpret_cast<const f64x2*>(a.X) + tile_o * (int64_t)N * I + c0
                              : reinterpret_cast<const f64x2*>(a.X) + o0 * (int64_t)N;

    f64x4 vr, vi;
    f64x2 xreg[4];
    auto gload = [&](int n0) {
        if (FAST) {
            const char* vb = reinterpret_cast<const char*>(a.M + (int64_t)n0 * ld + k0);
            vr = *reinterpret_cast<const f64x4*>(vb + v_lane);
            vi = *reinterpret_cast<const f64x4*>(vb + plane * 8 + v_lane);
            // strided: row n0 + xa, columns xb..xb+3;  contiguous: row xa, n = n0 + xb..xb+3
            const char* xbse = reinterpret_cast<const char*>(STRIDED ? xu + (int64_t)n0 * I : xu + n0);
#pragma unroll
            for (int e = 0; e < 4; ++e) xreg[e] = *reinterpret_cast<const f64x2*>(xbse + x_lane + 16 * e);
            return;
        }
        vr = *reinterpret_cast<const f64x4*>(vsrc + (int64_t)n0 * ld);
        vi = *reinterpret_cast<const f64x4*>(vsrc + plane + (int64_t)n0 * ld);
        if (STRIDED) {
            const int n = n0 + xa;
            const bool nok = n < N;
            const f64x2* src = xsrc + (int64_t)(nok ? n : 0) * I;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const f64x2 v = src[xcol[e]];
                xreg[e] = (nok && xok[e]) ? v : f64x2{0.0, 0.0};
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int n = n0 + xb + e;
                const bool nok = n < N;
                const f64x2 v = xsrc[nok ? n : 0];
                xreg[e] = (nok && xok[e]) ? v : f64x2{0.0, 0.0};
            }
        }
    };
    auto lstore = [&](int buf) {
        double (*Vt)[KC][TM] = STRIDED ? RT[buf] : CT[buf];
        double (*Xt)[KC][TM] = STRIDED ? CT[buf] : RT[buf];
        *reinterpret_cast<f64x4*>(&Vt[0][vn][vk]) = vr;
        *reinterpret_cast<f64x4*>(&Vt[1][vn][vk]) = vi;
        if (STRIDED) {
            *reinterpret_cast<f64x4*>(&Xt[0][xa][xb]) = f64x4{xreg[0].x, xreg[1].x, xreg[2].x, xreg[3].x};
            *reinterpret_cast<f64x4*>(&Xt[1][xa][xb]) = f64x4{xreg[0].y, xreg[1].y, xreg[2].y, xreg[3].y};
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                Xt[0][xb + e][xa] = xreg[e].x;
                Xt[1][xb + e][xa] = xreg[e].y;
            }
        }
    };

    // The four real products of the complex product are accumulated apart (rr = Re R * Re C, ii, ri, ir)
    // and combined with their signs in the epilogue, so the loop neither negates an operand nor
    // applies the conjugation.
    f64x4 prr[2][2], pii[2][2], pri[2][2], pir[2][2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            prr[rb][cb] = f64x4{0, 0, 0, 0};
            pii[rb][cb] = f64x4{0, 0, 0, 0};
            pri[rb][cb] = f64x4{0, 0, 0, 0};
            pir[rb][cb] = f64x4{0, 0, 0, 0};
        }

    const int nchunks = (N + KC - 1) / KC;
    gload(0);
    lstore(0);
    if (nchunks > 1) gload(KC);
    __syncthreads();

    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        // Chunk c+1, requested one chunk ago, moves to the other LDS buffer after the first k-step's
        // MFMAs and chunk c+2 is requested after the second's.  Both run unconditionally so that they
        // stay in the MFMAs' basic block: past the end they store stale registers into the buffer
        // nobody reads any more and load the last chunk again.
        const int n2 = (c + 2 < nchunks ? c + 2 : nchunks - 1) * KC;
#pragma unroll
        for (int ks = 0; ks < KC / 4; ++ks) {
            const int n = 4 * ks + lq;
            // MFMA row (column) i of block b stands for tile row (column) 2 * i + b of the wave tile,
            // so a lane's operands for both blocks sit side by side in LDS: one 16-byte read per plane
            // (the epilogue stores by the same rule)
            const f64x2 vrr = *reinterpret_cast<const f64x2*>(&RT[buf][0][n][wr0 + 2 * l16]);
            const f64x2 vri = *reinterpret_cast<const f64x2*>(&RT[buf][1][n][wr0 + 2 * l16]);
            const f64x2 vcr = *reinterpret_cast<const f64x2*>(&CT[buf][0][n][wc0 + 2 * l16]);
            const f64x2 vci = *reinterpret_cast<const f64x2*>(&CT[buf][1][n][wc0 + 2 * l16]);
            const double rr[2] = {vrr.x, vrr.y}, ri[2] = {vri.x, vri.y};
            const double cr[2] = {vcr.x, vcr.y}, ci[2] = {vci.x, vci.y};
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) prr[rb][cb] = mfma_f64(rr[rb], cr[cb], prr[rb][cb]);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) pri[rb][cb] = mfma_f64(rr[rb], ci[cb], pri[rb][cb]);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) pii[rb][cb] = mfma_f64(ri[rb], ci[cb], pii[rb][cb]);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) pir[rb][cb] = mfma_f64(ri[rb], cr[cb], pir[rb][cb]);
            if (ks == 0) {
                __builtin_amdgcn_sched_barrier(0);
                lstore(buf ^ 1);
                __builtin_amdgcn_sched_barrier(0);
            } else if (ks == 1) {
                __builtin_amdgcn_sched_barrier(0);
                gload(n2);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
    }

    // (plain stores: a lane's 16 bytes do not fill a memory line on their own, and the streaming hint
    // would send every piece to memory separately -- measured 1.8x the written bytes, no time gained)
    // epilogue: accumulator register v of a lane is MFMA row 4 * v + lane / 16, column lane % 16 of its
    // block, i.e. tile row 2 * (4 * v + lq) + rb and tile columns 2 * l16, 2 * l16 + 1 for cb = 0, 1
    f64x2* Y = reinterpret_cast<f64x2*>(a.Y);
    const double msign = a.conj ? -1.0 : 1.0;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const int row = wr0 + 2 * (4 * v + lq) + rb;
                const int col = wc0 + 2 * l16 + cb;
                // the matrix is the row operand of a strided mode and the column operand of the
                // contiguous one; conjugating it flips the sign of its imaginary part's products
                const double re = prr[rb][cb][v] - msign * pii[rb][cb][v];
                const double im = STRIDED ? pri[rb][cb][v] + msign * pir[rb][cb][v]
                                          : msign * pri[rb][cb][v] + pir[rb][cb][v];
                f64x2 y = f64x2{re * a.scale, im * a.scale};
                if (a.Tw) {      // fused twiddle of the FFT formulation's first stage
                    const int64_t kk = STRIDED ? k0 + row : k0 + col;
                    const int64_t ii = STRIDED ? c0 + col : 0;
                    if (kk < K && (!STRIDED || ii < I)) {
                        const f64x2 w = reinterpret_cast<const f64x2*>(a.Tw)[kk * a.twB + ii / a.twInner];
                        const double wi = a.conj ? -w.y : w.y;
                        y = f64x2{y.x * w.x - y.y * wi, y.x * wi + y.y * w.x};
                    }
                }
                if (STRIDED) {
                    if (k0 + row < K && c0 + col < I)
                        Y[y_offset(a, tile_o) + (int64_t)(k0 + row) * a.sYk + c0 + col] = y;
                } else {
                    if (o0 + row < a.O && k0 + col < K)
                        Y[y_offset(a, o0 + row) + (int64_t)(k0 + col) * a.sYk] = y;
                }
            }
}

// Strided contraction with a small square matrix (16 or 32 points: the stages of the FFT formulation)
// in plain fp64 vector arithmetic.  Such a pass moves 32 bytes per 8 * N flop, below the ridge of the
// fp64 units (whose vector rate equals the matrix-core rate on this chip), and an N-row matrix would
// fill a quarter or half of the matrix-core kernel's 64-row tile.  One thread owns one column (o, i):
// it loads the N points of the column (consecutive threads read consecutive 16-byte elements), forms
// the N outputs with the matrix broadcast from LDS, applies the optional twiddle and stores them.
template <int N>
__global__ __launch_bounds__(kT) void k_stage_f64(ContractArgs64 a, int64_t ncols)
{
    __shared__ f64x2 m[N * N];       // M[k][n] as (re, im), conjugated for BACKWARD
    const int tid = threadIdx.x;
    const int64_t plane = (int64_t)a.rows * a.ld;
    for (int e = tid; e < N * N; e += kT) {
        const int k = e % N, n = e / N;                   // the planes are contiguous along k
        m[k * N + n] = f64x2{a.M[(int64_t)n * a.ld + k], (a.conj ? -1.0 : 1.0) * a.M[plane + (int64_t)n * a.ld + k]};
    }
    __syncthreads();
    const int64_t I = a.I;
    const f64x2* X = reinterpret_cast<const f64x2*>(a.X);
    f64x2* Y = reinterpret_cast<f64x2*>(a.Y);
    const int64_t stride = (int64_t)gridDim.x * gridDim.y * kT;
    for (int64_t c = block_id() * kT + tid; c < ncols; c += stride) {
        const int64_t o = c / I, i = c - o * I;
        const f64x2* src = X + o * N * I + i;
        f64x2 x[N];
#pragma unroll
        for (int n = 0; n < N; ++n) x[n] = src[(int64_t)n * I];
        f64x2* dst = Y + y_offset(a, o) + i;
        const int64_t beta = a.Tw ? i / a.twInner : 0;
#pragma unroll 2
        for (int k = 0; k < N; ++k) {
            double re = 0.0, im = 0.0;
#pragma unroll
            for (int n = 0; n < N; ++n) {
                const f64x2 w = m[k * N + n];
                re = fma(w.x, x[n].x, re);
                re = fma(-w.y, x[n].y, re);
                im = fma(w.x, x[n].y, im);
                im = fma(w.y, x[n].x, im);
            }
            re *= a.scale;
            im *= a.scale;
            if (a.Tw) {
                const f64x2 t = reinterpret_cast<const f64x2*>(a.Tw)[(int64_t)k * a.twB + beta];
                const double ti = a.conj ? -t.y : t.y;
                const double r2 = re * t.x - im * ti;
                im = re * ti + im * t.x;
                re = r2;
            }
            dst[(int64_t)k * a.sYk] = f64x2{re, im};
        }
    }
}

// Sub-index swap of 16-byte elements: output element e gathers its source (natural index
// k_a + A*k_b  <-  slot k_a*B + k_b on every swapped axis).
struct Reorder128 {
    const f64x2* in;
    f64x2* out;
    int n[3], A[3], B[3], swap[3];
};
__global__ __launch_bounds__(kT) void k_reorder_c128(Reorder128 a, int64_t total)
{
    const int64_t stride = (int64_t)gridDim.x * kT;
    for (int64_t e = (int64_t)blockIdx.x * kT + threadIdx.x; e < total; e += stride) {
        const int z = (int)(e % a.n[2]);
        const int64_t r = e / a.n[2];
        const int y = (int)(r % a.n[1]);
        const int x = (int)(r / a.n[1]);
        const int sx = a.swap[0] ? (x % a.A[0]) * a.B[0] + x / a.A[0] : x;
        const int sy = a.swap[1] ? (y % a.A[1]) * a.B[1] + y / a.A[1] : y;
        const int sz = a.swap[2] ? (z % a.A[2]) * a.B[2] + z / a.A[2] : z;
        a.out[e] = a.in[((int64_t)sx * a.n[1] + sy) * a.n[2] + sz];
    }
}

inline dim3 grid_for(int64_t blocks)
{
    const int64_t kMaxX = 1 << 22;
    if (blocks <= kMaxX) return dim3((unsigned)blocks);
    return dim3((unsigned)kMaxX, (unsigned)((blocks + kMaxX - 1) / kMaxX));
}

}  // namespace

hipError_t launch_contract_f64(const ContractArgs64& a, hipStream_t stream)
{
    if (a.O < 1 || a.I < 1 || a.N < 1 || a.K < 1) return hipErrorInvalidValue;
    if (a.I > 1 && a.K == a.N && (a.N == 16 || a.N == 32) && a.ld >= a.K && a.rows >= a.N) {
        // small strided stage: fp64 vector arithmetic, one column per thread
        const int64_t ncols = a.O * a.I;
        int64_t blocks = (ncols + kT - 1) / kT;
        if (blocks > 256 * 64) blocks = 256 * 64;
        if (a.N == 16) hipLaunchKernelGGL(k_stage_f64<16>, grid_for(blocks), dim3(kT), 0, stream, a, ncols);
        else hipLaunchKernelGGL(k_stage_f64<32>, grid_for(blocks), dim3(kT), 0, stream, a, ncols);
        return hipGetLastError();
    }
    // the kernel reads whole 64-wide, 16-deep tiles of the zero-padded planes
    if (a.ld % 64 != 0 || a.ld < a.K || a.rows % KC != 0 || a.rows < a.N) return hipErrorInvalidValue;
    const int tk = (a.K + 63) / 64;
    // (K need not fill the tile: the planes are zero-padded to whole tiles and the stores are masked)
    const bool whole = a.N % KC == 0 && a.ld < (1 << 20);
    if (a.I == 1) {
        // contiguous mode: rows = o, columns = k; the k-tile index runs fastest
        const int64_t to = (a.O + TM - 1) / TM;
        const int64_t total = (int64_t)tk * to;
        if (whole && a.O % TM == 0 && a.N < (1 << 21))
            hipLaunchKernelGGL((k_contract_f64<false, true>), grid_for(total), dim3(kT), 0, stream, a, tk, to, total);
        else
            hipLaunchKernelGGL((k_contract_f64<false, false>), grid_for(total), dim3(kT), 0, stream, a, tk, to, total);
    } else {
        const int64_t ti = (a.I + TN - 1) / TN;
        const int64_t total = (int64_t)tk * ti * a.O;
        if (whole && a.I % TN == 0 && a.I < (1 << 23))
            hipLaunchKernelGGL((k_contract_f64<true, true>), grid_for(total), dim3(kT), 0, stream, a, tk, ti, total);
        else
            hipLaunchKernelGGL((k_contract_f64<true, false>), grid_for(total), dim3(kT), 0, stream, a, tk, ti, total);
    }
    return hipGetLastError();
}

hipError_t launch_reorder_c128(const void* in, void* out, const int n[3], const int A[3], const int B[3],
                               const int swap[3], hipStream_t stream)
{
    Reorder128 a{};
    a.in = reinterpret_cast<const f64x2*>(in);
    a.out = reinterpret_cast<f64x2*>(out);
    for (int j = 0; j < 3; ++j) {
        a.n[j] = n[j];
        a.A[j] = A[j];
        a.B[j] = B[j];
        a.swap[j] = swap[j];
    }
    const int64_t total = (int64_t)n[0] * n[1] * n[2];
    if (total <= 0) return hipSuccess;
    int64_t blocks = (total + kT - 1) / kT;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(k_reorder_c128, dim3((unsigned)blocks), dim3(kT), 0, stream, a, total);
    return hipGetLastError();
}

}  // namespace dft3d
