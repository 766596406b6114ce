// Mode contraction with fp32 accuracy on the bf16 matrix cores (gfx950, v_mfma_f32_32x32x16_bf16).
//
// The paper's MXU multiplies in bfloat16 and reaches float32 precision by decomposing each
// float32 number into several bfloat16 numbers and accumulating the cross products (Section
// II-A).  The same scheme on CDNA4, whose bf16 MFMA rate is 16x its fp32 rate:
//
//     x = x1 + x2 + x3   (each bf16, xj = bf16(x - x1 - .. - x(j-1)), residual ~2^-24 |x|)
//     v*x ~= v1*x1 + v1*x2 + v2*x1 + v1*x3 + v3*x1 + v2*x2          (6 of the 9 cross products)
//
// all accumulated in the fp32 accumulators of the MFMA.  The matrix is split once at plan time
// (from its fp64 entries); the data tile is split while it is staged into LDS.
//
// The complex product takes three real products, each accumulated on its own:
//     P1 = sum Vr*Xr,  P2 = sum Vi*Xi,  P3 = sum (Vr+Vi)*(Xr+Xi);   Re = P1 - P2,  Im = P3 - P1 - P2.
// This is not only 25 % less matrix work than four products.  The 16-term adder inside the bf16 MFMA
// aligns its addends to the largest one and cuts what falls below about 2^-31 of it towards minus
// infinity (measured: 2^24 + 1 + 2^-8 comes back as 2^24, 2^24 + 2 + 1 - 2^-8 as 2^24 + 2), so the many
// small level products of the split give every accumulator a small negative bias that does not
// depend on the data's signs.  A sum accumulated in one register (Re = sum Vr*Xr + (-Vi)*Xi) keeps that
// bias, and the next mode's all-ones matrix row (output index 0) adds it up coherently over the whole
// axis: measured 7e-5 relative at 8192 x 8192, against 2e-6 everywhere else.  In the differences
// P1 - P2 and P3 - (P1 + P2) the biases of the accumulators cancel (P3's operands are twice as large as
// those of P1 and P2, and so is its bias); a four-product kernel was built first and removed for this.
//
// Kernel shape.  One kernel serves both contraction types:  out[row, col] = sum_n R[row,n] C[col,n]
//   strided modes   : R = matrix (rows = k), C = data (cols = the contiguous index i)
//   contiguous mode : R = data (rows = o),   C = matrix (cols = k)
// Both operands of a 32x32x16 bf16 MFMA hold 8 consecutive n per lane, so the LDS tiles are
// [plane][row or col][n] with n contiguous: RT and CT, 9 planes each (re, im, re+im) x (hi, mid, lo),
// 128 rows x 16 n per chunk.  A workgroup is 4 waves (one per SIMD, up to 512 VGPRs each) on a 128x128
// tile, each wave 64x64 = 2x2 MFMA blocks x three accumulators; 72 MFMAs per chunk per wave.
// Double-buffered LDS, register-staged prefetch one chunk ahead, one barrier per chunk.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "dft3d_internal.h"

namespace dft3d {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kT = 256;
constexpr int TM = 128, TN = 128, KC = 16;

__device__ __forceinline__ int64_t block_id() { return (int64_t)blockIdx.y * gridDim.x + blockIdx.x; }

__device__ __forceinline__ int64_t remap(int64_t wg, int64_t total)
{
    constexpr int64_t kXcds = 8;
    if (total % kXcds != 0) return wg;
    return (wg % kXcds) * (total / kXcds) + wg / kXcds;
}

__device__ __forceinline__ int64_t y_offset(const ContractArgs& a, int64_t o)
{
    if (a.Olo == 1) return o * a.sYohi;
    return (o / a.Olo) * a.sYohi + (o % a.Olo) * a.sYolo;
}

// (a, b) -> packed (bf16(a) | bf16(b) << 16), round to nearest even
__device__ __forceinline__ unsigned pack_bf16(float a, float b)
{
    bf16x2 p = __builtin_convertvector(f32x2{a, b}, bf16x2);
    return __builtin_bit_cast(unsigned, p);
}
__device__ __forceinline__ float lo_as_float(unsigned p) { return __builtin_bit_cast(float, p << 16); }
__device__ __forceinline__ float hi_as_float(unsigned p) { return __builtin_bit_cast(float, p & 0xffff0000u); }

// f(integral_constant<int, B>), ..., f(integral_constant<int, E - 1>): unrolling that does not depend
// on the optimizer's size limits
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

__device__ __forceinline__ f32x16 mfma_bf16(u32x4 a, u32x4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                  c, 0, 0, 0);
}

// With P1 = sum Vr*Xr, P2 = sum Vi*Xi and P3 = sum (Vr+Vi)*(Xr+Xi):  Re = P1 - P2,  Im = P3 - P1 - P2,
// each real product as six bf16 level products: 18 MFMAs per complex block and chunk.  The sums
// Vr+Vi (at plan time, from fp64) and Xr+Xi (in fp32 while staging) are split into their own three
// levels, so each operand has nine planes: (re, im, sum) x (hi, mid, lo), plane = 3*part + level.
// LDS rows are 32 bytes (two 16-byte slots) without padding; the slot is XOR-ed with bits 2 and 3 of
// the row, so that any 8 (and any 16) consecutive rows read at the same slot fall on 8 (16) different
// 16-byte bank groups.
// Three accumulator sets (192 AGPRs) and nine operand planes per side (144 VGPRs): one wave per SIMD.
constexpr int kPlanes3 = 9;

// MASKED: any shape.  The matrix planes are zero padded to whole tiles and chunks, so only the data
// loads (clamped to the tensor, and zero beyond the contracted length) and the stores (skipped outside
// the output) know about the edges.
template <bool STRIDED, bool MASKED>
__global__ __launch_bounds__(kT, 1) void k_contract_bf16x3(ContractArgs a, int tilesK, int64_t tilesOther,
                                                            int64_t total)
{
    // [buffer][plane][row][2 x 16 bytes]: slots hold n = 0..7 and 8..15 of the chunk, swizzled by row
    __shared__ u32x4 RT[2][kPlanes3][TM][2];
    __shared__ u32x4 CT[2][kPlanes3][TN][2];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wr0 = (wave >> 1) * 64;      // wave tile origin inside the 128 x 128 tile
    const int wc0 = (wave & 1) * 64;
    const int l32 = lane & 31;
    const int kq = lane >> 5;

    int64_t t = block_id();
    if (t >= total) return;
    t = remap(t, total);
    const int kt = (int)(t % tilesK);
    t /= tilesK;
    const int k0 = kt * 128;

    const int N = a.M.N;
    const int64_t I = a.I;
    // the bf16 planes are stored tile by tile: [k tile of 128][chunk of 16 n][plane][128 k][16 n], so the
    // 128 x 16 piece of every plane that one chunk needs is 4 KiB of contiguous memory
    const unsigned short* __restrict__ Vs = a.M.split;
    const int vchunks = a.M.split_ld / KC;

    // this thread's piece of the matrix tile: row = tid / 2 (k), 8 consecutive n
    const int vrow = tid >> 1, vhalf = tid & 1;
    const unsigned short* vsrc = Vs + (int64_t)kt * vchunks * (kPlanes3 * 2048) + vrow * 16 + 8 * vhalf;

    // this thread's piece of the data tile
    int64_t tile_o = 0, c0 = 0, o0 = 0;
    const float2* xsrc;
    int xrow, xhalf;                       // LDS destination (row or column, which half of the chunk)
    if (STRIDED) {
        tile_o = t / tilesOther;
        c0 = (t % tilesOther) * TN;
        xrow = tid & 127;
        xhalf = tid >> 7;
        xsrc = a.X + tile_o * (int64_t)N * I + (int64_t)(8 * xhalf) * I + c0 + xrow;
    } else {
        o0 = t * TM;
        xrow = tid >> 1;
        xhalf = tid & 1;
        xsrc = a.X + (o0 + xrow) * (int64_t)N + 8 * xhalf;
    }
    const int vslot = vhalf ^ ((vrow >> 2) & 1) ^ ((vrow >> 3) & 1);
    const int xslot = xhalf ^ ((xrow >> 2) & 1) ^ ((xrow >> 3) & 1);

    u32x4 vreg[kPlanes3];
    f32x2 xreg[8];
    constexpr bool kByElement = STRIDED || MASKED;      // one load per complex number (else two per load)
    constexpr int kXLoads = kByElement ? 8 : 4;
    auto load_v = [&](int n0, int p) {
        vreg[p] = *reinterpret_cast<const u32x4*>(vsrc + (int64_t)(n0 / KC) * (kPlanes3 * 2048) + p * 2048);
    };
    auto load_x = [&](int n0, int j) {           // j < kXLoads
        if (MASKED) {
            const int n = n0 + 8 * xhalf + j;
            const int nc = n < N ? n : N - 1;
            const f32x2* src;
            if (STRIDED) {
                const int64_t col = c0 + xrow < I ? c0 + xrow : I - 1;
                src = reinterpret_cast<const f32x2*>(a.X + tile_o * (int64_t)N * I + (int64_t)nc * I + col);
            } else {
                const int64_t row = o0 + xrow < a.O ? o0 + xrow : a.O - 1;
                src = reinterpret_cast<const f32x2*>(a.X + row * (int64_t)N + nc);
            }
            const f32x2 v = *src;
            xreg[j] = n < N ? v : f32x2{0.f, 0.f};
        } else if (STRIDED) {
            xreg[j] = *reinterpret_cast<const f32x2*>(xsrc + (int64_t)(n0 + j) * I);
        } else {
            const f32x4 v = *reinterpret_cast<const f32x4*>(xsrc + n0 + 2 * j);
            xreg[2 * j] = f32x2{v.x, v.y};
            xreg[2 * j + 1] = f32x2{v.z, v.w};
        }
    };
    auto gload = [&](int n0) {           // same order as the main loop requests them
#pragma unroll
        for (int j = 0; j < kXLoads; ++j) load_x(n0, j);
#pragma unroll
        for (int p = 0; p < kPlanes3; ++p) load_v(n0, p);
    };

    // Staging of a chunk into LDS, cut into small steps.  The data values are split into their three
    // bf16 levels two at a time (pair q = values 2q, 2q+1 of the 8 this thread holds; part 0 = real,
    // 1 = imaginary, 2 = their sum); a split takes three steps (one per level).
    // Conjugating the matrix flips the sign of Vi and turns Vr+Vi into Vr-Vi, which is not a stored
    // plane: BACKWARD instead conjugates the data and the result (conj(V) x = conj(V conj(x))).
    const float xsign = a.conj ? -1.0f : 1.0f;
    u32x4 lv[3][3];                 // [part][level], dword q = pair q
    float res0[3], res1[3];
    auto split_step = [&](int part, int q, int step) {
        if (step == 0) {
            float x0, x1;
            if (part == 0) {
                x0 = xreg[2 * q].x;
                x1 = xreg[2 * q + 1].x;
            } else if (part == 1) {
                x0 = xreg[2 * q].y * xsign;
                x1 = xreg[2 * q + 1].y * xsign;
            } else {
                x0 = xreg[2 * q].x + xreg[2 * q].y * xsign;
                x1 = xreg[2 * q + 1].x + xreg[2 * q + 1].y * xsign;
            }
            const unsigned p0 = pack_bf16(x0, x1);
            res0[part] = x0 - lo_as_float(p0);      // exact
            res1[part] = x1 - hi_as_float(p0);
            lv[part][0][q] = p0;
        } else if (step == 1) {
            const unsigned p1 = pack_bf16(res0[part], res1[part]);
            res0[part] -= lo_as_float(p1);          // exact
            res1[part] -= hi_as_float(p1);
            lv[part][1][q] = p1;
        } else {
            lv[part][2][q] = pack_bf16(res0[part], res1[part]);
        }
    };
    auto store_x = [&](int buf, int part, int level) {
        u32x4 (*Xt)[TM][2] = STRIDED ? CT[buf] : RT[buf];
        Xt[3 * part + level][xrow][xslot] = lv[part][level];
    };
    auto store_v = [&](int buf, int p) {
        u32x4 (*Vt)[TM][2] = STRIDED ? RT[buf] : CT[buf];
        Vt[p][vrow][vslot] = vreg[p];
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int part = 0; part < 3; ++part) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int step = 0; step < 3; ++step) split_step(part, q, step);
#pragma unroll
            for (int level = 0; level < 3; ++level) store_x(buf, part, level);
        }
#pragma unroll
        for (int p = 0; p < kPlanes3; ++p) store_v(buf, p);
    };

    f32x16 acc[3][2][2];            // [P1, P2, P3][row block][column block]
#pragma unroll
    for (int part = 0; part < 3; ++part)
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[part][rb][cb][v] = 0.f;

    const int nchunks = vchunks;             // = N / KC for whole chunks; the matrix planes are zero beyond N
    auto chunk_n0 = [&](int j) { return (j < nchunks ? j : nchunks - 1) * KC; };     // clamped: tail re-reads the last chunk
    gload(0);
    lstore(0);
    gload(chunk_n0(1));
    __syncthreads();

    // Level pairs of the six cross products.
    // A wave issues in order and only one MFMA (32 cycles) can be in flight ahead of it, so the
    // wave's other work of the iteration -- converting and storing chunk c+1, requesting chunk
    // c+2 -- is cut into steps of a few instructions and at most one step is placed in front of
    // each of the 72 MFMAs, where it issues in the shadow of the previous one.
    constexpr int PL[6] = {1, 2, 0, 1, 0, 0};
    constexpr int QL[6] = {1, 0, 2, 0, 1, 0};
    // the steps of the side work in order: per pair 9 split steps (3 parts x 3 levels) and the pair's
    // loads; 9 stores of the data planes; 9 x (store a matrix plane, request it again)
    constexpr int kPerPair = 9 + kXLoads / 4;
    constexpr int kXStoreAt = 4 * kPerPair;
    constexpr int kVAt = kXStoreAt + 9;
    constexpr int kSteps = kVAt + 18;
    static_assert(kSteps <= 72, "one step per MFMA at most");
    // read offsets of this lane: rows r0 + l32 (r0 a multiple of 32) share bits 2 and 3 with l32
    const int rslot = kq ^ ((l32 >> 2) & 1) ^ ((l32 >> 3) & 1);
    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        const int n2 = chunk_n0(c + 2);

        u32x4 R[3][2][3], C[3][2][3];        // [part][block][level]
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            const int lr = PL[j], lc = QL[j];        // (1,1), (2,0), (0,2): each level once, in order of first use
#pragma unroll
            for (int part = 0; part < 3; ++part)
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    R[part][b][lr] = RT[buf][3 * part + lr][wr0 + b * 32 + l32][rslot];
                    C[part][b][lc] = CT[buf][3 * part + lc][wc0 + b * 32 + l32][rslot];
                }
        }
        __builtin_amdgcn_sched_barrier(0);

        static_for<0, 72>([&](auto slot) {
            constexpr int s = decltype(slot)::value;
            // ---- at most one step of side work: step i sits in slot i * 72 / kSteps
            constexpr int step = (s * kSteps + 71) / 72;
            if constexpr (step < kSteps && (step * 72) / kSteps == s) {
                if constexpr (step < kXStoreAt) {
                    constexpr int q = step / kPerPair, w = step % kPerPair;
                    if constexpr (w < 9) split_step(w / 3, q, w % 3);
                    else if constexpr (kByElement) load_x(n2, 2 * q + (w - 9));
                    else load_x(n2, q);
                } else if constexpr (step < kVAt) {
                    constexpr int w = step - kXStoreAt;
                    store_x(buf ^ 1, w / 3, w % 3);
                } else {
                    constexpr int w = step - kVAt;
                    if constexpr ((w & 1) == 0) store_v(buf ^ 1, w >> 1);
                    else load_v(n2, w >> 1);
                }
            }
            // ---- one MFMA: product part = s / 24, level pair (s % 24) / 4, block s % 4
            constexpr int part = s / 24, pq = (s % 24) / 4, rb = (s >> 1) & 1, cb = s & 1;
            acc[part][rb][cb] = mfma_bf16(R[part][rb][PL[pq]], C[part][cb][QL[pq]], acc[part][rb][cb]);
            __builtin_amdgcn_sched_barrier(0);
        });
        __syncthreads();
    }

    // epilogue: accumulator register v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int col = wc0 + cb * 32 + l32;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = wr0 + rb * 32 + 8 * (v / 4) + 4 * kq + (v % 4);
                const float p1 = acc[0][rb][cb][v], p2 = acc[1][rb][cb][v], p3 = acc[2][rb][cb][v];
                const f32x2 y = f32x2{(p1 - p2) * a.scale, (p3 - p1 - p2) * (a.scale * xsign)};
                if (MASKED) {
                    if (STRIDED ? (k0 + row >= a.M.K || c0 + col >= I) : (o0 + row >= a.O || k0 + col >= a.M.K)) continue;
                }
                if (STRIDED) {
                    float2* Yo = a.Y + y_offset(a, tile_o);
                    __builtin_nontemporal_store(y, reinterpret_cast<f32x2*>(Yo + (int64_t)(k0 + row) * a.sYk + c0 + col));
                } else {
                    __builtin_nontemporal_store(y, reinterpret_cast<f32x2*>(a.Y + y_offset(a, o0 + row) + (int64_t)(k0 + col) * a.sYk));
                }
            }
        }
    }
}

inline dim3 grid_for(int64_t blocks)
{
    const int64_t kMaxX = 1 << 22;
    if (blocks <= kMaxX) return dim3((unsigned)blocks);
    return dim3((unsigned)kMaxX, (unsigned)((blocks + kMaxX - 1) / kMaxX));
}

}  // namespace

bool contract_bf16x3_supported(const ContractArgs& a)
{
    if (!a.M.split || a.M.split_planes != kPlanes3 || a.Tw) return false;
    // 32-bit tile counts inside the kernel
    const int64_t tk = (a.M.K + 127) / 128;
    const int64_t other = a.I == 1 ? (a.O + TM - 1) / TM : ((a.I + TN - 1) / TN) * a.O;
    return a.M.K >= 1 && a.M.N >= 1 && tk * other < (int64_t(1) << 31);
}

hipError_t launch_contract_bf16x3(const ContractArgs& a, hipStream_t stream)
{
    const int K = a.M.K, N = a.M.N;
    const int tk = (K + 127) / 128;
    const bool whole_kn = K % 128 == 0 && N % KC == 0;
    if (a.I == 1) {
        // contiguous mode: rows = o, columns = k; the k-tile index runs fastest
        const int64_t to = (a.O + TM - 1) / TM;
        const int64_t total = (int64_t)tk * to;
        if (whole_kn && a.O % TM == 0)
            hipLaunchKernelGGL((k_contract_bf16x3<false, false>), grid_for(total), dim3(kT), 0, stream, a, tk, to, total);
        else
            hipLaunchKernelGGL((k_contract_bf16x3<false, true>), grid_for(total), dim3(kT), 0, stream, a, tk, to, total);
    } else {
        const int64_t ti = (a.I + TN - 1) / TN;
        const int64_t total = (int64_t)tk * ti * a.O;
        if (whole_kn && a.I % TN == 0)
            hipLaunchKernelGGL((k_contract_bf16x3<true, false>), grid_for(total), dim3(kT), 0, stream, a, tk, ti, total);
        else
            hipLaunchKernelGGL((k_contract_bf16x3<true, true>), grid_for(total), dim3(kT), 0, stream, a, tk, ti, total);
    }
    return hipGetLastError();
}

}  // namespace dft3d
