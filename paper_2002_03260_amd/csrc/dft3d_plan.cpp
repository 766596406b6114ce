// Host side of the dft3d C ABI: plan creation (split choice, matrix generation and upload),
// argument validation and the sequencing of kernel launches for dft3d_exec and the step calls.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "dft3d_internal.h"

namespace dft3d {

namespace {
thread_local char g_error[512] = "";
}

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}

namespace {

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

void free_matrix(DeviceMatrix& m)
{
    if (m.re) (void)hipFree(m.re);
    if (m.split) (void)hipFree(m.split);
    if (m.f64) (void)hipFree(m.f64);
    m = DeviceMatrix{};
}

// round-to-nearest-even conversion of a double to bfloat16 (returned as its 16 bits)
unsigned short to_bf16(double v)
{
    float f = (float)v;
    unsigned u;
    std::memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return (unsigned short)(u >> 16);   // inf / nan
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}
double from_bf16(unsigned short h)
{
    unsigned u = (unsigned)h << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return (double)f;
}

// Build and upload the three-level bf16 decomposition of a K x N complex matrix given as fp64
// row-major planes: v = v1 + v2 + v3 with vj = bf16(v - v1 - .. - v(j-1)).
// The planes of Re + Im (formed in fp64) follow those of Re and Im: the bf16 kernel uses three real
// products per complex product.
dft3d_status upload_split(const std::vector<double>& re, const std::vector<double>& im, int K, int N,
                          DeviceMatrix* m)
{
    const int ld = round_up(N, 16), rows = round_up(K, 128);
    const size_t plane = (size_t)ld * rows;
    const int parts = 3;
    std::vector<unsigned short> host((size_t)(3 * parts) * plane, 0);
    for (int part = 0; part < parts; ++part) {
        for (int k = 0; k < K; ++k)
            for (int n = 0; n < N; ++n) {
                const size_t e = (size_t)k * N + n;
                double r = part == 0 ? re[e] : (part == 1 ? im[e] : re[e] + im[e]);
                // tiled layout: [k tile of 128][chunk of 16 n][plane][128 k][16 n]
                const size_t tile = ((size_t)(k / 128) * (ld / 16) + n / 16) * (size_t)(3 * parts);
                for (int lvl = 0; lvl < 3; ++lvl) {
                    const unsigned short h = to_bf16(r);
                    host[(tile + 3 * part + lvl) * 2048 + (size_t)(k % 128) * 16 + n % 16] = h;
                    r -= from_bf16(h);
                }
            }
    }
    unsigned short* dev = nullptr;
    hipError_t e = hipMalloc((void**)&dev, host.size() * sizeof(unsigned short));
    if (e != hipSuccess) {
        set_error("hipMalloc of the bf16 decomposition of a %d x %d matrix failed: %s", K, N, hipGetErrorString(e));
        return DFT3D_ERR_ALLOC;
    }
    e = hipMemcpy(dev, host.data(), host.size() * sizeof(unsigned short), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(dev);
        set_error("upload of the bf16 decomposition failed: %s", hipGetErrorString(e));
        return DFT3D_ERR_HIP;
    }
    m->split = dev;
    m->split_ld = ld;
    m->split_rows = rows;
    m->split_planes = 3 * parts;
    return DFT3D_OK;
}

// Upload the fp64 planes of a K x N complex matrix (row-major host planes) in the transposed, zero
// padded layout plane[n * ld + k]: re plane, then im plane.
dft3d_status upload_f64(const std::vector<double>& re, const std::vector<double>& im, int K, int N,
                        DeviceMatrix* m)
{
    const int ld = round_up(K, 64), rows = round_up(N, 16);
    const size_t plane = (size_t)ld * rows;
    std::vector<double> host(2 * plane, 0.0);
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n) {
            host[(size_t)n * ld + k] = re[(size_t)k * N + n];
            host[plane + (size_t)n * ld + k] = im[(size_t)k * N + n];
        }
    double* dev = nullptr;
    hipError_t e = hipMalloc((void**)&dev, 2 * plane * sizeof(double));
    if (e != hipSuccess) {
        set_error("hipMalloc of the fp64 planes of a %d x %d matrix failed: %s", K, N, hipGetErrorString(e));
        return DFT3D_ERR_ALLOC;
    }
    e = hipMemcpy(dev, host.data(), 2 * plane * sizeof(double), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(dev);
        set_error("upload of the fp64 planes failed: %s", hipGetErrorString(e));
        return DFT3D_ERR_HIP;
    }
    m->f64 = dev;
    m->ld64 = ld;
    m->rows64 = rows;
    return DFT3D_OK;
}

// Upload a K x N complex matrix given as row-major host planes into the padded, transposed
// device layout.  re and im share one allocation.
dft3d_status upload_matrix(const std::vector<float>& re, const std::vector<float>& im, int K, int N,
                           DeviceMatrix* out)
{
    DeviceMatrix m;
    m.K = K;
    m.N = N;
    m.ld = round_up(K, kPlaneLdAlign);
    m.rows = round_up(N, kPlaneRowAlign);
    const size_t plane = (size_t)m.ld * m.rows;
    std::vector<float> host(2 * plane, 0.0f);
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n) {
            host[(size_t)n * m.ld + k] = re[(size_t)k * N + n];
            host[plane + (size_t)n * m.ld + k] = im[(size_t)k * N + n];
        }
    float* dev = nullptr;
    hipError_t e = hipMalloc((void**)&dev, 2 * plane * sizeof(float));
    if (e != hipSuccess) {
        set_error("hipMalloc of a %d x %d matrix failed: %s", K, N, hipGetErrorString(e));
        return DFT3D_ERR_ALLOC;
    }
    e = hipMemcpy(dev, host.data(), 2 * plane * sizeof(float), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(dev);
        set_error("upload of a %d x %d matrix failed: %s", K, N, hipGetErrorString(e));
        return DFT3D_ERR_HIP;
    }
    m.re = dev;
    m.im = dev + plane;
    *out = m;
    return DFT3D_OK;
}

// Row-major K x N planes of a matrix -> row-major N x K planes of its conjugate transpose.
template <typename T>
void conjugate_transpose(std::vector<T>& re, std::vector<T>& im, int64_t K, int64_t N)
{
    std::vector<T> tr((size_t)(K * N)), ti((size_t)(K * N));
    for (int64_t k = 0; k < K; ++k)
        for (int64_t n = 0; n < N; ++n) {
            tr[(size_t)(n * K + k)] = re[(size_t)(k * N + n)];
            ti[(size_t)(n * K + k)] = -im[(size_t)(k * N + n)];
        }
    re.swap(tr);
    im.swap(ti);
}

dft3d_status make_axis_matrix(int64_t n, const double* coords, DeviceMatrix* out, bool with_split = false,
                              bool with_f64 = false, bool adjoint = false)
{
    std::vector<float> re((size_t)n * n), im((size_t)n * n);
    dft3d_status s = dft3d_generate_matrix(n, coords, DFT3D_FORWARD, re.data(), im.data());
    if (s != DFT3D_OK) return s;
    if (adjoint) conjugate_transpose(re, im, n, n);
    s = upload_matrix(re, im, (int)n, (int)n, out);
    if (s != DFT3D_OK || (!with_split && !with_f64)) return s;
    // the bf16 levels and the fp64 planes are taken from the fp64 entries, not from their fp32 roundings
    std::vector<double> dre((size_t)n * n), dim((size_t)n * n);
    for (int64_t k = 0; k < n; ++k)
        for (int64_t j = 0; j < n; ++j) {
            if (coords) unit_root_turns((double)k * coords[j], DFT3D_FORWARD, &dre[k * n + j], &dim[k * n + j]);
            else unit_root_ratio(k * j, n, DFT3D_FORWARD, &dre[k * n + j], &dim[k * n + j]);
        }
    if (adjoint) conjugate_transpose(dre, dim, n, n);
    if (with_split) s = upload_split(dre, dim, (int)n, (int)n, out);
    if (s == DFT3D_OK && with_f64) s = upload_f64(dre, dim, (int)n, (int)n, out);
    return s;
}

// The twiddle table T[k_a * B + beta] = exp(-2 pi i k_a beta / (A B)) of an A x B split, on the device.
dft3d_status upload_twiddle(int64_t A, int64_t B, float2** out)
{
    const size_t cnt = (size_t)(A * B);
    std::vector<float> tr(cnt), ti(cnt);
    dft3d_status s = dft3d_generate_twiddle(A, B, DFT3D_FORWARD, tr.data(), ti.data());
    if (s != DFT3D_OK) return s;
    std::vector<float2> tw(cnt);
    for (size_t e = 0; e < cnt; ++e) tw[e] = make_float2(tr[e], ti[e]);
    hipError_t e = hipMalloc((void**)out, cnt * sizeof(float2));
    if (e != hipSuccess) {
        *out = nullptr;
        set_error("plan_create: hipMalloc of a twiddle table failed: %s", hipGetErrorString(e));
        return DFT3D_ERR_ALLOC;
    }
    e = hipMemcpy(*out, tw.data(), cnt * sizeof(float2), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        set_error("plan_create: twiddle upload failed: %s", hipGetErrorString(e));
        return DFT3D_ERR_HIP;
    }
    return DFT3D_OK;
}

int64_t default_split(int64_t n)
{
    // 16 x (C*16), the split whose second factor the fused kernels split once more (2048: a third of the
    // matrix-core work of 32 x 64)
    if (n == 2048 || n == 1024) return 16;
    if ((n & (n - 1)) == 0) {
        int lg = 0;
        while ((int64_t(1) << (lg + 1)) <= n) ++lg;
        return int64_t(1) << (lg / 2);
    }
    int64_t best = 1;
    for (int64_t a = 1; a * a <= n; ++a)
        if (n % a == 0) best = a;
    return best;
}

// Default first factor of `axis` of an n[0] x n[1] x n[2] plan.  4096, 8192 and 16384 points take a first
// stage of 4 or 8 points in vector arithmetic and 1024 or 2048 points on the fused kernels where those can
// run (complex64, not the UNFUSED exhibit, strided axes with an inner extent that is a multiple of 16).
// Measured on 2-D tensors: 4096^2 0.374 ms as 64 x 64 against 0.239 ms as 4 x 1024; 8192^2 1.81 ms as
// 64 x 128 against 0.87 ms; 16384^2 11.6 ms as 128 x 128 against 3.4 ms.  A contiguous axis of 4096 points
// alone is faster on its one-pass 64 x 64 kernel (256 x 256 x 4096: 4.16 against 4.29 ms), unless the
// axis transformed next starts with a butterfly pass too and takes over the re-ordering.
int64_t default_split_for_axis(const int64_t n[3], int axis, uint32_t flags)
{
    const int64_t len = n[axis];
    auto radix_of = [](int64_t m) -> int64_t { return m == 4096 || m == 8192 ? 4 : (m == 16384 ? 8 : 0); };
    auto strided_ok = [&](int ax) {
        const int64_t inner = ax == 1 ? n[2] : n[1] * n[2];
        const int64_t r = radix_of(n[ax]);
        return r > 0 && inner % 16 == 0 && r * inner <= (int64_t(1) << 23);
    };
    const int64_t r = radix_of(len);
    if (r == 0 || (flags & (DFT3D_FLAG_COMPLEX128 | DFT3D_FLAG_UNFUSED))) return default_split(len);
    if (axis != 2) return strided_ok(axis) ? r : default_split(len);
    if (len != 4096) return r;
    const int next = n[1] > 1 ? 1 : (n[0] > 1 ? 0 : -1);
    return (next >= 0 && strided_ok(next)) ? r : default_split(len);
}

}  // namespace
}  // namespace dft3d

using namespace dft3d;

struct dft3d_plan_s {
    int64_t n[3] = {0, 0, 0};      // input lengths
    int64_t k[3] = {0, 0, 0};      // output lengths (== n except for evaluation-point plans)
    bool points = false;           // created by dft3d_plan_create_points
    dft3d_formulation form = DFT3D_KDFT;
    uint32_t flags = 0;
    bool nonuniform[3] = {false, false, false};

    // KDFT: forward matrix per axis; axes with equal length and no coordinates share storage
    DeviceMatrix M[3];
    int M_owner[3] = {0, 1, 2};

    // FFT: per axis first/second-stage matrices and twiddle table (shared between equal axes)
    int64_t A[3] = {1, 1, 1}, B[3] = {1, 1, 1};
    DeviceMatrix FA[3], FB[3];
    float2* Tw[3] = {nullptr, nullptr, nullptr};
    double* Tw64[3] = {nullptr, nullptr, nullptr};   // complex128 plans: the same table in fp64, (re, im) pairs
    int F_owner[3] = {0, 1, 2};
    // FFT, first factor 2, 4 or 8 and a second factor B of 512, 1024 or 2048 points: the B-point second stage
    // is run in the FFT formulation itself (Eq. 13 - 16 applied to it once more, B = A2 x B2) on the fused
    // kernels, with the tables of that split; A2 = 0 where the second stage is the dense B x B contraction
    int64_t A2[3] = {0, 0, 0}, B2[3] = {0, 0, 0};
    DeviceMatrix FA2[3], FB2[3];
    float2* Tw2[3] = {nullptr, nullptr, nullptr};

    void* workspace = nullptr;
    size_t workspace_bytes = 0;
    // FFT, three fused passes: row pitch (elements, > nz) of the intermediate between the y and the
    // x pass, which lives in the workspace; 0 = natural layout.  Rows of the x pass are ny*nz*8
    // bytes apart; when that is a multiple of 8 KiB every row of a tile falls on the same memory
    // channels, and 16 elements of padding per z row spread them (measured: x pass 8 % faster with
    // its reads padded; padding its writes instead, by running it second, gains less).
    int64_t ws_pitch = 0;
    bool x_first = false;          // passes x, y, z with the tensor between x and y stored as [y][z / 16][k_x][16]

    // optional per-pass event timing of exec
    std::vector<hipEvent_t> prof_events;   // [exec][pass][begin,end]
    std::vector<int> prof_npass;           // passes recorded per exec
    int prof_capacity = 0;
    int prof_next = 0;

    bool complex128() const { return (flags & DFT3D_FLAG_COMPLEX128) != 0; }
    size_t elem_bytes() const { return complex128() ? 16 : 8; }
    int64_t elements() const { return n[0] * n[1] * n[2]; }
    int64_t out_elements() const { return k[0] * k[1] * k[2]; }
    // Modes are applied in the order z, y, x, so when `axis` is contracted the axes after it
    // already have their output length and the axes before it still have their input length.
    int64_t inner(int axis) const { return axis == 0 ? k[1] * k[2] : (axis == 1 ? k[2] : 1); }
    int64_t outer(int axis) const { return axis == 0 ? 1 : (axis == 1 ? n[0] : n[0] * n[1]); }
    int64_t stage_in_elements(int axis) const { return outer(axis) * n[axis] * inner(axis); }
    int64_t stage_out_elements(int axis) const { return outer(axis) * k[axis] * inner(axis); }
};

namespace {

bool valid_direction(int d) { return d == DFT3D_FORWARD || d == DFT3D_BACKWARD; }

dft3d_status check_buffers(const dft3d_plan_s* p, const void* in, void* out, const char* who,
                           int64_t in_elems = -1, int64_t out_elems = -1)
{
    if (!p) { set_error("%s: plan is NULL", who); return DFT3D_ERR_INVALID_ARG; }
    if (!in || !out) { set_error("%s: NULL tensor pointer", who); return DFT3D_ERR_INVALID_ARG; }
    if (((uintptr_t)in & 15) || ((uintptr_t)out & 15)) {
        set_error("%s: tensor pointers must be 16-byte aligned", who);
        return DFT3D_ERR_INVALID_ARG;
    }
    const uintptr_t abytes = (uintptr_t)(in_elems >= 0 ? in_elems : p->elements()) * p->elem_bytes();
    const uintptr_t bbytes = (uintptr_t)(out_elems >= 0 ? out_elems : p->out_elements()) * p->elem_bytes();
    const uintptr_t a = (uintptr_t)in, b = (uintptr_t)out;
    if (a < b + bbytes && b < a + abytes) {
        set_error("%s: in and out overlap (the transform is out of place)", who);
        return DFT3D_ERR_INVALID_ARG;
    }
    return DFT3D_OK;
}

dft3d_status hip_status(hipError_t e, const char* who)
{
    if (e == hipSuccess) return DFT3D_OK;
    set_error("%s: kernel launch failed: %s", who, hipGetErrorString(e));
    return DFT3D_ERR_HIP;
}

// Arguments of the complex64 contraction of one KDFT mode.
ContractArgs mode_args(const dft3d_plan_s* p, int axis, const float2* in, float2* out, int conj, float scale)
{
    ContractArgs a{};
    a.X = in;
    a.Y = out;
    a.M = p->M[axis];
    a.O = p->outer(axis);
    a.I = p->inner(axis);
    a.Olo = 1;
    a.sYohi = (int64_t)a.M.K * a.I;
    a.sYolo = 0;
    a.sYk = a.I;
    a.Tw = nullptr;
    a.twB = 1;
    a.twInner = 1;
    a.scale = scale;
    a.conj = conj;
    a.three_m = (p->flags & DFT3D_FLAG_3M) ? 1 : 0;
    a.bf16x3 = (p->flags & DFT3D_FLAG_BF16X3) ? 1 : 0;
    return a;
}

// out[.., k, ..] = sum_n M[k,n] in[.., n, ..] along `axis`, natural layout.
hipError_t run_mode(const dft3d_plan_s* p, int axis, const float2* in, float2* out, int conj,
                    float scale, hipStream_t st)
{
    if (p->complex128()) {
        // `in` / `out` are complex128 tensors here; the pointers are only passed through
        const DeviceMatrix& M = p->M[axis];
        ContractArgs64 d{};
        d.X = in;
        d.Y = out;
        d.M = M.f64;
        d.K = M.K;
        d.N = M.N;
        d.ld = M.ld64;
        d.rows = M.rows64;
        d.O = p->outer(axis);
        d.I = p->inner(axis);
        d.Olo = 1;
        d.sYohi = (int64_t)M.K * d.I;
        d.sYolo = 0;
        d.sYk = d.I;
        d.scale = conj ? 1.0 / (double)M.N : 1.0;     // BACKWARD on a uniform axis: exact reciprocal in fp64
        d.conj = conj;
        (void)scale;
        return launch_contract_f64(d, st);
    }
    return launch_contract(mode_args(p, axis, in, out, conj, scale), st);
}

// A stage of 128 points or more is bound by the matrix cores (8 * 128 / 16 = 64 flop per byte): it
// takes the three-product complex scheme, like the fused kernels.  Shorter stages are memory-bound.
int stage_uses_three_products(const DeviceMatrix& M) { return M.N >= 128 ? 1 : 0; }

// The complex128 form of a stage contraction: same views and strides, fp64 planes and twiddles.
hipError_t run_stage_c128(const DeviceMatrix& M, const void* in, void* out, int64_t O, int64_t I, int64_t Olo,
                          int64_t sYohi, int64_t sYolo, int64_t sYk, const double* Tw, int twB, int64_t twInner,
                          double scale, int conj, hipStream_t st)
{
    ContractArgs64 d{};
    d.X = in;
    d.Y = out;
    d.M = M.f64;
    d.K = M.K;
    d.N = M.N;
    d.ld = M.ld64;
    d.rows = M.rows64;
    d.O = O;
    d.I = I;
    d.Olo = Olo;
    d.sYohi = sYohi;
    d.sYolo = sYolo;
    d.sYk = sYk;
    d.scale = scale;
    d.conj = conj;
    d.Tw = Tw;
    d.twB = twB;
    d.twInner = twInner;
    return launch_contract_f64(d, st);
}

// FFT first stage on `axis`: view [outer][A][B*inner], contract the A index.
// Whether the first stage of `axis` is the element-wise butterfly pass (2, 4 or 8 points).
bool first_stage_is_radix(const dft3d_plan_s* p, int axis)
{
    return p->form == DFT3D_FFT && !p->complex128() && !(p->flags & DFT3D_FLAG_UNFUSED) &&
           radix_stage_supported((int)p->A[axis], p->B[axis], p->inner(axis));
}

// unpermute_z: the input still has the z axis as [k_a][k_b] (its second stage ran without the re-ordering
// pass); a first stage in butterflies reads through that permutation.
hipError_t run_first_stage(const dft3d_plan_s* p, int axis, const float2* in, float2* out, int conj,
                           int fuse_twiddle, hipStream_t st, bool unpermute_z = false)
{
    if (p->complex128()) {
        const int64_t I = p->B[axis] * p->inner(axis);
        return run_stage_c128(p->FA[axis], in, out, p->outer(axis), I, 1, (int64_t)p->FA[axis].K * I, 0, I,
                              fuse_twiddle ? p->Tw64[axis] : nullptr, (int)p->B[axis], p->inner(axis), 1.0, conj, st);
    }
    // 2, 4 or 8 points: butterflies in a memory-bound element-wise pass (the UNFUSED exhibit keeps the contraction)
    if (first_stage_is_radix(p, axis))
        return launch_radix_twiddle(in, out, p->outer(axis), (int)p->A[axis], p->B[axis], p->inner(axis),
                                    fuse_twiddle ? p->Tw[axis] : nullptr, conj, p->n[2], unpermute_z ? (int)p->A[2] : 1,
                                    unpermute_z ? (int)p->B[2] : 1, st);
    if (unpermute_z) return hipErrorInvalidValue;
    ContractArgs a{};
    a.X = in;
    a.Y = out;
    a.M = p->FA[axis];
    a.O = p->outer(axis);
    a.I = p->B[axis] * p->inner(axis);
    a.Olo = 1;
    a.sYohi = (int64_t)a.M.K * a.I;
    a.sYolo = 0;
    a.sYk = a.I;
    a.Tw = fuse_twiddle ? p->Tw[axis] : nullptr;
    a.twB = (int)p->B[axis];
    a.twInner = p->inner(axis);
    a.scale = 1.0f;
    a.conj = conj;
    a.three_m = stage_uses_three_products(a.M);
    return launch_contract(a, st);
}

// Whether the second stage of `axis` runs on a fused kernel with the split B = A2 x B2 (the UNFUSED exhibit
// keeps the dense contraction).
bool second_stage_nested(const dft3d_plan_s* p, int axis, int reorder)
{
    if (!p->A2[axis] || (p->flags & DFT3D_FLAG_UNFUSED)) return false;
    const int A2 = (int)p->A2[axis], B2 = (int)p->B2[axis];
    if (axis == 2) return !reorder && fft_zn_supported(A2, B2);
    const int64_t inner = p->inner(axis);
    return fft_sn_supported(A2, B2, inner) && p->A[axis] * inner <= (int64_t(1) << 23);
}

// FFT second stage on `axis`: view [outer*A][B][inner], contract the B index; with reorder the
// result (k_a, k_b) lands at natural position k_a + A*k_b of the axis.
hipError_t run_second_stage(const dft3d_plan_s* p, int axis, const float2* in, float2* out, int conj,
                            float scale, int reorder, hipStream_t st)
{
    const int64_t A = p->A[axis], B = p->B[axis], inner = p->inner(axis);
    if (p->complex128()) {
        // BACKWARD: the exact fp64 reciprocal of the axis length (the float `scale` is not used)
        const double sc = conj ? 1.0 / (double)p->n[axis] : 1.0;
        return run_stage_c128(p->FB[axis], in, out, p->outer(axis) * A, inner, A, A * B * inner,
                              reorder ? inner : B * inner, reorder ? A * inner : inner, nullptr, 1, 1, sc, conj, st);
    }
    if (second_stage_nested(p, axis, reorder)) {
        const int A2 = (int)p->A2[axis], B2 = (int)p->B2[axis];
        if (axis == 2)     // rows of B contiguous points, [outer * A] of them; the result stays [k_a][k2]
            return launch_fft_zn(in, out, p->outer(axis) * A, A2, B2, p->FA2[axis], p->FB2[axis], p->Tw2[axis], scale,
                                 conj, st);
        // view [outer][k_a][beta][inner] -> [outer][k2][k_a][inner] (re-ordered) or [outer][k_a][k2][inner]
        FftStridedArgs f{};
        f.X = in;
        f.Y = out;
        f.O = p->outer(axis);
        f.Yn = A;
        f.Zt = inner / 16;
        f.inO = f.outO = A * B * inner;
        f.inY = B * inner;
        f.inN = inner;
        f.outY = reorder ? inner : B * inner;
        f.outN = reorder ? A * inner : inner;
        return launch_fft_sr_ex(f, A2, B2, p->FA2[axis], p->FB2[axis], p->Tw2[axis], scale, conj, st);
    }
    ContractArgs a{};
    a.X = in;
    a.Y = out;
    a.M = p->FB[axis];
    a.O = p->outer(axis) * A;
    a.I = inner;
    a.Olo = A;
    a.sYohi = A * B * inner;
    if (reorder) {
        a.sYolo = inner;        // k_a is the fast sub-index
        a.sYk = A * inner;      // k_b the slow one
    } else {
        a.sYolo = B * inner;
        a.sYk = inner;
    }
    a.Tw = nullptr;
    a.twB = 1;
    a.twInner = 1;
    a.scale = scale;
    a.conj = conj;
    a.three_m = stage_uses_three_products(a.M);
    return launch_contract(a, st);
}

// FFT, whole z axis in one fused kernel (both stages, twiddle, natural order).
bool z_axis_fusable(const dft3d_plan_s* p)
{
    return p->form == DFT3D_FFT && !p->complex128() && fft_z_supported((int)p->A[2], (int)p->B[2]);
}

hipError_t run_fused_z(const dft3d_plan_s* p, const float2* in, float2* out, int conj, float scale,
                       hipStream_t st)
{
    return launch_fft_z(in, out, p->n[0] * p->n[1], (int)p->A[2], (int)p->B[2], p->FA[2], p->FB[2],
                        p->Tw[2], scale, conj, st);
}

// FFT, whole x or y axis in one fused kernel.
bool strided_axis_fusable(const dft3d_plan_s* p, int axis)
{
    return p->form == DFT3D_FFT && axis != 2 && !p->complex128() &&
           fft_s_supported((int)p->A[axis], (int)p->B[axis], p->inner(axis));
}

hipError_t run_fused_s(const dft3d_plan_s* p, int axis, const float2* in, float2* out, int conj,
                       float scale, hipStream_t st)
{
    return launch_fft_s(in, out, p->outer(axis), p->inner(axis), (int)p->A[axis], (int)p->B[axis],
                        p->FA[axis], p->FB[axis], p->Tw[axis], scale, conj, st);
}

// The y and x passes of a plan whose workspace intermediate has a padded row pitch: y writes it,
// x reads it.  Tensor views: y pass [nx][ny][1][nz], x pass [1][nx][ny][nz].
hipError_t run_fused_s_padded(const dft3d_plan_s* p, int axis, const float2* in, float2* out, int conj,
                              float scale, hipStream_t st)
{
    const int64_t nx = p->n[0], ny = p->n[1], nz = p->n[2], pitch = p->ws_pitch;
    FftStridedArgs a{};
    a.X = in;
    a.Y = out;
    a.Zt = nz / 16;
    if (axis == 1) {
        a.O = nx;
        a.Yn = 1;
        a.inO = ny * nz;
        a.inN = nz;
        a.inY = 0;
        a.outO = ny * pitch;
        a.outN = pitch;
        a.outY = 0;
    } else {
        a.O = 1;
        a.Yn = ny;
        a.inO = 0;
        a.inN = ny * pitch;
        a.inY = pitch;
        a.outO = 0;
        a.outN = ny * nz;
        a.outY = nz;
    }
    return launch_fft_sr_ex(a, (int)p->A[axis], (int)p->B[axis], p->FA[axis], p->FB[axis], p->Tw[axis], scale,
                            conj, st);
}

// The x and y passes of a plan that transforms x first.  The tensor between them is stored tile by tile,
// [y][z / 16][k_x][16]: the x pass (a tile = all x of one (y, 16 z)) writes every tile's result as one
// contiguous block, the y pass (a tile = all y of one (k_x, 16 z)) reads rows nx*nz apart and writes the
// natural layout [k_x][k_y][z], rows nz apart.  Both passes then read with the long stride and write with
// a short one.  (Measured at 2048^3: a pass that writes rows ny*nz = 32 MiB apart takes 45 ms, one that
// writes rows 16 KiB apart 32 - 35 ms, whatever it reads; contiguous tiles instead of rows 16 KiB apart
// in the intermediate: another 2 %.)  The tile index of the kernels' arguments (Yn) runs over (y, z / 16)
// in the x pass and over z / 16 in the y pass, with one 16-column tile (Zt = 1) per index.
hipError_t run_fused_s_xfirst(const dft3d_plan_s* p, int axis, const float2* in, float2* out, int conj,
                              float scale, hipStream_t st)
{
    const int64_t nx = p->n[0], ny = p->n[1], nz = p->n[2], ztt = nz / 16;
    FftStridedArgs a{};
    a.X = in;
    a.Y = out;
    a.Zt = 1;
    if (axis == 0) {
        a.O = 1;
        a.Yn = ny * ztt;
        a.inO = 0;
        a.inN = ny * nz;
        a.inY = 16;
        a.outO = 0;
        a.outN = 16;
        a.outY = nx * 16;
    } else {
        a.O = nx;
        a.Yn = ztt;
        a.inO = 16;
        a.inN = nx * nz;
        a.inY = nx * 16;
        a.outO = ny * nz;
        a.outN = nz;
        a.outY = 16;
    }
    return launch_fft_sr_ex(a, (int)p->A[axis], (int)p->B[axis], p->FA[axis], p->FB[axis], p->Tw[axis], scale,
                            conj, st);
}

hipError_t run_reorder(const dft3d_plan_s* p, int mask, const float2* in, float2* out, hipStream_t st)
{
    if (p->complex128()) {
        int n[3], A[3], B[3], swap[3];
        for (int j = 0; j < 3; ++j) {
            n[j] = (int)p->n[j];
            A[j] = (int)p->A[j];
            B[j] = (int)p->B[j];
            swap[j] = (mask >> j) & 1;
        }
        return launch_reorder_c128(in, out, n, A, B, swap, st);
    }
    ReorderArgs r{};
    r.in = in;
    r.out = out;
    for (int j = 0; j < 3; ++j) {
        r.n[j] = (int)p->n[j];
        r.A[j] = (int)p->A[j];
        r.B[j] = (int)p->B[j];
        r.swap[j] = (mask >> j) & 1;
    }
    return launch_reorder(r, st);
}

float axis_scale(const dft3d_plan_s* p, int axis, int direction)
{
    return direction == DFT3D_BACKWARD ? (float)(1.0 / (double)p->n[axis]) : 1.0f;
}

// KDFT plans on complex64 tensors whose axes are all at most 32 long run the whole transform in one
// launch and need no workspace.
bool single_launch(const dft3d_plan_s* p)
{
    return p->form == DFT3D_KDFT && !p->complex128() && kdft_small_supported(p->M[0], p->M[1], p->M[2]);
}

dft3d_status require_uniform_for_backward(const dft3d_plan_s* p, int direction, const char* who)
{
    if (direction == DFT3D_BACKWARD && (p->points || p->nonuniform[0] || p->nonuniform[1] || p->nonuniform[2])) {
        set_error("%s: BACKWARD is not defined for a plan with nonuniform axes", who);
        return DFT3D_ERR_UNSUPPORTED;
    }
    return DFT3D_OK;
}

}  // namespace

extern "C" {

const char* dft3d_status_string(dft3d_status s)
{
    switch (s) {
        case DFT3D_OK: return "DFT3D_OK";
        case DFT3D_ERR_INVALID_ARG: return "DFT3D_ERR_INVALID_ARG";
        case DFT3D_ERR_UNSUPPORTED: return "DFT3D_ERR_UNSUPPORTED";
        case DFT3D_ERR_ALLOC: return "DFT3D_ERR_ALLOC";
        case DFT3D_ERR_HIP: return "DFT3D_ERR_HIP";
    }
    return "DFT3D_ERR_UNKNOWN";
}

const char* dft3d_last_error(void) { return g_error; }

dft3d_status dft3d_plan_create(dft3d_plan* plan, int64_t nx, int64_t ny, int64_t nz,
                               dft3d_formulation f, const double* cx, const double* cy,
                               const double* cz)
{
    return dft3d_plan_create_ex(plan, nx, ny, nz, f, cx, cy, cz, nullptr, 0);
}

// Destroys a half-built plan on every exit but the successful one (early returns and exceptions).
struct PlanGuard {
    dft3d_plan_s* p;
    ~PlanGuard() { if (p) dft3d_plan_destroy(p); }
};

static dft3d_status plan_create_impl(dft3d_plan* plan, int64_t nx, int64_t ny, int64_t nz,
                                     dft3d_formulation f, const double* cx, const double* cy,
                                     const double* cz, const int64_t* split, uint32_t flags);

// No exception may cross the C boundary: host allocations that fail (a matrix of 2^24 x 2^24 entries,
// say) become DFT3D_ERR_ALLOC.
dft3d_status dft3d_plan_create_ex(dft3d_plan* plan, int64_t nx, int64_t ny, int64_t nz,
                                  dft3d_formulation f, const double* cx, const double* cy,
                                  const double* cz, const int64_t* split, uint32_t flags)
{
    try {
        return plan_create_impl(plan, nx, ny, nz, f, cx, cy, cz, split, flags);
    } catch (...) {
        if (plan) *plan = nullptr;
        set_error("plan_create: out of host memory while building the matrices");
        return DFT3D_ERR_ALLOC;
    }
}

static dft3d_status plan_create_impl(dft3d_plan* plan, int64_t nx, int64_t ny, int64_t nz,
                                     dft3d_formulation f, const double* cx, const double* cy,
                                     const double* cz, const int64_t* split, uint32_t flags)
{
    if (!plan) { set_error("plan_create: plan pointer is NULL"); return DFT3D_ERR_INVALID_ARG; }
    *plan = nullptr;
    const int64_t n[3] = {nx, ny, nz};
    const double* c[3] = {cx, cy, cz};
    for (int j = 0; j < 3; ++j)
        if (n[j] < 1 || n[j] > (int64_t(1) << 24)) {
            set_error("plan_create: axis %d has length %lld (must be 1..2^24)", j, (long long)n[j]);
            return DFT3D_ERR_INVALID_ARG;
        }
    if (f != DFT3D_KDFT && f != DFT3D_FFT) {
        set_error("plan_create: unknown formulation %d", (int)f);
        return DFT3D_ERR_INVALID_ARG;
    }
    for (int j = 0; j < 3; ++j)
        for (int64_t i = 0; c[j] && i < n[j]; ++i)
            if (!std::isfinite(c[j][i])) {
                set_error("plan_create: coordinate %lld of axis %d is not finite", (long long)i, j);
                return DFT3D_ERR_INVALID_ARG;
            }
    if (flags & ~(DFT3D_FLAG_CLOBBER_INPUT | DFT3D_FLAG_UNFUSED | DFT3D_FLAG_3M | DFT3D_FLAG_BF16X3 |
                  DFT3D_FLAG_COMPLEX128 | DFT3D_FLAG_ADJOINT)) {
        set_error("plan_create: unknown flag bits 0x%x", flags);
        return DFT3D_ERR_INVALID_ARG;
    }
    if ((flags & DFT3D_FLAG_ADJOINT) && f != DFT3D_KDFT) {
        set_error("plan_create: ADJOINT is offered for KDFT plans (on uniform axes it equals BACKWARD up to the 1/N factor)");
        return DFT3D_ERR_UNSUPPORTED;
    }
    if ((flags & DFT3D_FLAG_COMPLEX128) && (flags & (DFT3D_FLAG_3M | DFT3D_FLAG_BF16X3 | DFT3D_FLAG_UNFUSED))) {
        set_error("plan_create: COMPLEX128 is not combined with 3M / BF16X3 / UNFUSED");
        return DFT3D_ERR_UNSUPPORTED;
    }
    if (f == DFT3D_FFT && (flags & (DFT3D_FLAG_3M | DFT3D_FLAG_BF16X3))) {
        set_error("plan_create: 3M and BF16X3 select variants of the KDFT mode contraction; an FFT plan has none");
        return DFT3D_ERR_UNSUPPORTED;
    }
    if (f == DFT3D_FFT && (cx || cy || cz)) {
        set_error("plan_create: the FFT formulation requires uniform sampling on every axis");
        return DFT3D_ERR_UNSUPPORTED;
    }
    // inner / outer extents are handled as 32-bit quantities inside the kernels
    if (ny * nz >= (int64_t(1) << 31) || nx * ny >= (int64_t(1) << 31)) {
        set_error("plan_create: ny*nz and nx*ny must be below 2^31");
        return DFT3D_ERR_UNSUPPORTED;
    }

    dft3d_plan_s* p = new (std::nothrow) dft3d_plan_s();
    if (!p) { set_error("plan_create: out of host memory"); return DFT3D_ERR_ALLOC; }
    PlanGuard guard{p};
    p->form = f;
    p->flags = flags;
    for (int j = 0; j < 3; ++j) {
        p->n[j] = n[j];
        p->k[j] = n[j];
        p->nonuniform[j] = c[j] != nullptr;
    }

    dft3d_status s = DFT3D_OK;
    if (f == DFT3D_KDFT) {
        for (int j = 0; j < 3 && s == DFT3D_OK; ++j) {
            p->M_owner[j] = j;
            for (int i = 0; i < j; ++i)
                if (!c[j] && !c[i] && n[i] == n[j]) { p->M_owner[j] = i; break; }
            if (p->M_owner[j] == j)
                s = make_axis_matrix(n[j], c[j], &p->M[j], (flags & DFT3D_FLAG_BF16X3) != 0,
                                     (flags & DFT3D_FLAG_COMPLEX128) != 0, (flags & DFT3D_FLAG_ADJOINT) != 0);
            else p->M[j] = p->M[p->M_owner[j]];
        }
    } else {
        for (int j = 0; j < 3 && s == DFT3D_OK; ++j) {
            int64_t A = (split && split[j] > 0) ? split[j] : default_split_for_axis(n, j, flags);
            if (A < 1 || n[j] % A != 0) {
                set_error("plan_create: split %lld does not divide axis length %lld", (long long)A,
                          (long long)n[j]);
                s = DFT3D_ERR_INVALID_ARG;
                break;
            }
            p->A[j] = A;
            p->B[j] = n[j] / A;
            p->F_owner[j] = j;
            for (int i = 0; i < j; ++i)
                if (n[i] == n[j] && p->A[i] == A) { p->F_owner[j] = i; break; }
            if (p->F_owner[j] != j) {
                const int i = p->F_owner[j];
                p->FA[j] = p->FA[i];
                p->FB[j] = p->FB[i];
                p->Tw[j] = p->Tw[i];
                p->Tw64[j] = p->Tw64[i];
                p->A2[j] = p->A2[i];
                p->B2[j] = p->B2[i];
                p->FA2[j] = p->FA2[i];
                p->FB2[j] = p->FB2[i];
                p->Tw2[j] = p->Tw2[i];
                continue;
            }
            const bool c128 = (flags & DFT3D_FLAG_COMPLEX128) != 0;
            s = make_axis_matrix(p->A[j], nullptr, &p->FA[j], false, c128);
            if (s == DFT3D_OK) s = make_axis_matrix(p->B[j], nullptr, &p->FB[j], false, c128);
            if (s != DFT3D_OK) break;
            if (c128) {
                // the twiddle table T[k_a * B + beta] = exp(-2 pi i k_a beta / N) in fp64
                const int64_t A64 = p->A[j], B64 = p->B[j];
                std::vector<double> tw((size_t)(2 * A64 * B64));
                for (int64_t ka = 0; ka < A64; ++ka)
                    for (int64_t be = 0; be < B64; ++be)
                        unit_root_ratio(ka * be, A64 * B64, DFT3D_FORWARD, &tw[(size_t)(2 * (ka * B64 + be))],
                                        &tw[(size_t)(2 * (ka * B64 + be) + 1)]);
                hipError_t e64 = hipMalloc((void**)&p->Tw64[j], tw.size() * sizeof(double));
                if (e64 != hipSuccess) {
                    set_error("plan_create: hipMalloc of an fp64 twiddle table failed: %s", hipGetErrorString(e64));
                    s = DFT3D_ERR_ALLOC;
                    break;
                }
                e64 = hipMemcpy(p->Tw64[j], tw.data(), tw.size() * sizeof(double), hipMemcpyHostToDevice);
                if (e64 != hipSuccess) {
                    set_error("plan_create: fp64 twiddle upload failed: %s", hipGetErrorString(e64));
                    s = DFT3D_ERR_HIP;
                    break;
                }
            }
            s = upload_twiddle(p->A[j], p->B[j], &p->Tw[j]);
            if (s != DFT3D_OK) break;
            const int64_t Bj = p->B[j];
            if (!c128 && (A == 2 || A == 4 || A == 8) && (Bj == 512 || Bj == 1024 || Bj == 2048)) {
                p->A2[j] = 16;
                p->B2[j] = Bj / 16;
                s = make_axis_matrix(p->A2[j], nullptr, &p->FA2[j]);
                if (s == DFT3D_OK) s = make_axis_matrix(p->B2[j], nullptr, &p->FB2[j]);
                if (s == DFT3D_OK) s = upload_twiddle(p->A2[j], p->B2[j], &p->Tw2[j]);
                if (s != DFT3D_OK) break;
            }
        }
    }
    if (s != DFT3D_OK) return s;      // (the guard frees the plan)
    guard.p = nullptr;
    // Plans whose three axes all fuse.  Where both strided axes run on kernels that take separate input
    // and output strides and the x axis has 2048 points or more, the x pass comes first and writes a transposed
    // intermediate (see run_fused_s_xfirst); otherwise passes z, y, x, with padded rows in the workspace
    // intermediate between y and x where they help.
    const bool all_fused_candidate = f == DFT3D_FFT &&
                                     !(flags & (DFT3D_FLAG_UNFUSED | DFT3D_FLAG_CLOBBER_INPUT | DFT3D_FLAG_COMPLEX128)) &&
                                     n[0] > 1 && n[1] > 1 && n[2] > 1 && n[2] % 16 == 0 &&
                                     fft_z_supported((int)p->A[2], (int)p->B[2]);
    if (all_fused_candidate && n[0] >= 2048 && fft_sr_supported((int)p->A[1], (int)p->B[1], n[0] * n[2]) &&
        fft_sr_supported((int)p->A[0], (int)p->B[0], n[1] * n[2]))
        p->x_first = true;
    else if (all_fused_candidate && (n[1] * n[2] * 8) % 8192 == 0 && n[1] * (n[2] + 16) <= (int64_t(1) << 21) &&
             fft_sr_supported((int)p->A[1], (int)p->B[1], n[2]) && fft_sr_supported((int)p->A[0], (int)p->B[0], n[1] * n[2]))
        p->ws_pitch = n[2] + 16;
    // set-up for dft3d_exec_noalloc: look up this GPU's copy of the static scratch array now, so that
    // the exec call itself never has to (a failure here is reported by that call, not by this one)
    (void)noalloc_scratch_for_current_device();
    // kernels that need more than the default LDS size are told so now, not at their first launch
    // (which could be inside a graph capture)
    (void)configure_fft_kernels();
    *plan = p;
    return DFT3D_OK;
}

dft3d_status dft3d_plan_enable_profiling(dft3d_plan p, int max_execs)
{
    if (!p || max_execs < 0 || max_execs > 4096) {
        set_error("enable_profiling: invalid argument");
        return DFT3D_ERR_INVALID_ARG;
    }
    for (hipEvent_t ev : p->prof_events) (void)hipEventDestroy(ev);
    p->prof_events.clear();
    p->prof_npass.assign((size_t)max_execs, 0);
    p->prof_capacity = 0;
    p->prof_next = 0;
    const size_t count = (size_t)max_execs * DFT3D_MAX_PASSES * 2;
    p->prof_events.reserve(count);
    for (size_t i = 0; i < count; ++i) {
        hipEvent_t ev;
        hipError_t e = hipEventCreate(&ev);
        if (e != hipSuccess) {
            set_error("enable_profiling: hipEventCreate failed: %s", hipGetErrorString(e));
            for (hipEvent_t x : p->prof_events) (void)hipEventDestroy(x);
            p->prof_events.clear();
            return DFT3D_ERR_HIP;
        }
        p->prof_events.push_back(ev);
    }
    p->prof_capacity = max_execs;
    return DFT3D_OK;
}

dft3d_status dft3d_plan_read_profile(dft3d_plan p, int exec_index, float* ms, int* npass)
{
    if (!p || !ms || !npass || exec_index < 0 || exec_index >= p->prof_next) {
        set_error("read_profile: invalid argument or exec not recorded");
        return DFT3D_ERR_INVALID_ARG;
    }
    const int np = p->prof_npass[(size_t)exec_index];
    for (int i = 0; i < np; ++i) {
        const size_t base = ((size_t)exec_index * DFT3D_MAX_PASSES + i) * 2;
        hipError_t e = hipEventElapsedTime(&ms[i], p->prof_events[base], p->prof_events[base + 1]);
        if (e != hipSuccess) {
            set_error("read_profile: hipEventElapsedTime failed: %s (stream not synchronised?)",
                      hipGetErrorString(e));
            return DFT3D_ERR_HIP;
        }
    }
    *npass = np;
    return DFT3D_OK;
}

static dft3d_status plan_create_points_impl(dft3d_plan* plan, int64_t nx, int64_t ny, int64_t nz,
                                            int64_t kx, int64_t ky, int64_t kz, const double* zx,
                                            const double* zy, const double* zz, uint32_t flags);

dft3d_status dft3d_plan_create_points(dft3d_plan* plan, int64_t nx, int64_t ny, int64_t nz,
                                      int64_t kx, int64_t ky, int64_t kz, const double* zx,
                                      const double* zy, const double* zz, uint32_t flags)
{
    try {
        return plan_create_points_impl(plan, nx, ny, nz, kx, ky, kz, zx, zy, zz, flags);
    } catch (...) {
        if (plan) *plan = nullptr;
        set_error("plan_create_points: out of host memory while building the matrices");
        return DFT3D_ERR_ALLOC;
    }
}

static dft3d_status plan_create_points_impl(dft3d_plan* plan, int64_t nx, int64_t ny, int64_t nz,
                                            int64_t kx, int64_t ky, int64_t kz, const double* zx,
                                            const double* zy, const double* zz, uint32_t flags)
{
    if (!plan) { set_error("plan_create_points: plan pointer is NULL"); return DFT3D_ERR_INVALID_ARG; }
    *plan = nullptr;
    const int64_t n[3] = {nx, ny, nz}, k[3] = {kx, ky, kz};
    const double* z[3] = {zx, zy, zz};
    for (int j = 0; j < 3; ++j) {
        if (n[j] < 1 || n[j] > (int64_t(1) << 24) || k[j] < 1 || k[j] > (int64_t(1) << 24)) {
            set_error("plan_create_points: axis %d has lengths %lld -> %lld (must be 1..2^24)", j,
                      (long long)n[j], (long long)k[j]);
            return DFT3D_ERR_INVALID_ARG;
        }
        if (!z[j] && k[j] != n[j]) {
            set_error("plan_create_points: axis %d has no points, so its output length must equal its input length", j);
            return DFT3D_ERR_INVALID_ARG;
        }
    }
    if (flags & ~(DFT3D_FLAG_3M | DFT3D_FLAG_ADJOINT | DFT3D_FLAG_COMPLEX128)) {
        set_error("plan_create_points: only DFT3D_FLAG_3M, DFT3D_FLAG_ADJOINT and DFT3D_FLAG_COMPLEX128 are accepted");
        return DFT3D_ERR_INVALID_ARG;
    }
    if ((flags & DFT3D_FLAG_COMPLEX128) && (flags & DFT3D_FLAG_3M)) {
        set_error("plan_create_points: COMPLEX128 is not combined with 3M");
        return DFT3D_ERR_UNSUPPORTED;
    }
    const bool adjoint = (flags & DFT3D_FLAG_ADJOINT) != 0;
    if (ky * kz >= (int64_t(1) << 31) || nx * ny >= (int64_t(1) << 31) ||
        (adjoint && (ny * nz >= (int64_t(1) << 31) || kx * ky >= (int64_t(1) << 31)))) {
        set_error("plan_create_points: ky*kz and nx*ny (ADJOINT: also ny*nz and kx*ky) must be below 2^31");
        return DFT3D_ERR_UNSUPPORTED;
    }
    dft3d_plan_s* p = new (std::nothrow) dft3d_plan_s();
    if (!p) { set_error("plan_create_points: out of host memory"); return DFT3D_ERR_ALLOC; }
    PlanGuard guard{p};
    p->form = DFT3D_KDFT;
    p->flags = flags;
    p->points = true;
    dft3d_status s = DFT3D_OK;
    for (int j = 0; j < 3 && s == DFT3D_OK; ++j) {
        // the adjoint plan contracts the k index: its tensors go from kx x ky x kz to nx x ny x nz
        p->n[j] = adjoint ? k[j] : n[j];
        p->k[j] = adjoint ? n[j] : k[j];
        p->nonuniform[j] = z[j] != nullptr;
        p->M_owner[j] = j;
        std::vector<float> re((size_t)(k[j] * n[j])), im((size_t)(k[j] * n[j]));
        s = z[j] ? dft3d_generate_points_matrix(k[j], n[j], z[j], re.data(), im.data())
                 : dft3d_generate_matrix(n[j], nullptr, DFT3D_FORWARD, re.data(), im.data());
        if (s == DFT3D_OK && adjoint) conjugate_transpose(re, im, k[j], n[j]);
        if (s == DFT3D_OK) s = upload_matrix(re, im, (int)p->k[j], (int)p->n[j], &p->M[j]);
        if (s == DFT3D_OK && (flags & DFT3D_FLAG_COMPLEX128)) {
            // the fp64 planes come from the fp64 entries, not from their fp32 roundings
            std::vector<double> dre((size_t)(k[j] * n[j])), dim((size_t)(k[j] * n[j]));
            if (z[j]) s = generate_points_matrix_f64(k[j], n[j], z[j], dre.data(), dim.data());
            else
                for (int64_t r = 0; r < n[j]; ++r)
                    for (int64_t c = 0; c < n[j]; ++c)
                        unit_root_ratio(r * c, n[j], DFT3D_FORWARD, &dre[(size_t)(r * n[j] + c)], &dim[(size_t)(r * n[j] + c)]);
            if (s == DFT3D_OK && adjoint) conjugate_transpose(dre, dim, k[j], n[j]);
            if (s == DFT3D_OK) s = upload_f64(dre, dim, (int)p->k[j], (int)p->n[j], &p->M[j]);
        }
    }
    if (s != DFT3D_OK) return s;      // (the guard frees the plan)
    guard.p = nullptr;
    (void)noalloc_scratch_for_current_device();
    *plan = p;
    return DFT3D_OK;
}

dft3d_status dft3d_plan_get_output_shape(dft3d_plan p, int64_t* kx, int64_t* ky, int64_t* kz)
{
    if (!p || !kx || !ky || !kz) { set_error("get_output_shape: invalid argument"); return DFT3D_ERR_INVALID_ARG; }
    *kx = p->k[0];
    *ky = p->k[1];
    *kz = p->k[2];
    return DFT3D_OK;
}

dft3d_status dft3d_plan_destroy(dft3d_plan p)
{
    if (!p) return DFT3D_OK;
    for (hipEvent_t ev : p->prof_events) (void)hipEventDestroy(ev);
    for (int j = 0; j < 3; ++j) {
        if (p->form == DFT3D_KDFT) {
            if (p->M_owner[j] == j) free_matrix(p->M[j]);
        } else if (p->F_owner[j] == j) {
            free_matrix(p->FA[j]);
            free_matrix(p->FB[j]);
            if (p->Tw[j]) (void)hipFree(p->Tw[j]);
            if (p->Tw64[j]) (void)hipFree(p->Tw64[j]);
            free_matrix(p->FA2[j]);
            free_matrix(p->FB2[j]);
            if (p->Tw2[j]) (void)hipFree(p->Tw2[j]);
        }
    }
    delete p;
    return DFT3D_OK;
}

size_t dft3d_plan_workspace_bytes(dft3d_plan p)
{
    if (!p) return 0;
    if (single_launch(p)) return 0;
    if (p->points)   // two intermediates of different shapes: after mode z and after mode y
        return (size_t)(p->stage_out_elements(2) + p->stage_out_elements(1)) * p->elem_bytes();
    if (p->flags & DFT3D_FLAG_CLOBBER_INPUT) return 0;
    if (p->ws_pitch) return (size_t)(p->n[0] * p->n[1] * p->ws_pitch) * p->elem_bytes();
    return (size_t)p->elements() * p->elem_bytes();
}

dft3d_status dft3d_plan_set_workspace(dft3d_plan p, void* dev, size_t bytes)
{
    if (!p) { set_error("set_workspace: plan is NULL"); return DFT3D_ERR_INVALID_ARG; }
    if (dev && ((uintptr_t)dev & 15)) {
        set_error("set_workspace: workspace must be 16-byte aligned");
        return DFT3D_ERR_INVALID_ARG;
    }
    if (dev && bytes < dft3d_plan_workspace_bytes(p)) {
        set_error("set_workspace: %zu bytes given, %zu needed", bytes, dft3d_plan_workspace_bytes(p));
        return DFT3D_ERR_INVALID_ARG;
    }
    p->workspace = dev;
    p->workspace_bytes = dev ? bytes : 0;
    return DFT3D_OK;
}

dft3d_status dft3d_plan_axis_order(dft3d_plan p, int order[3])
{
    if (!p || !order) {
        set_error("axis_order: invalid argument");
        return DFT3D_ERR_INVALID_ARG;
    }
    for (int step = 0; step < 3; ++step) order[step] = p->x_first ? step : 2 - step;
    return DFT3D_OK;
}

dft3d_status dft3d_plan_get_split(dft3d_plan p, int axis, int64_t* A, int64_t* B)
{
    if (!p || axis < 0 || axis > 2 || !A || !B) {
        set_error("get_split: invalid argument");
        return DFT3D_ERR_INVALID_ARG;
    }
    if (p->form != DFT3D_FFT) {
        set_error("get_split: not an FFT plan");
        return DFT3D_ERR_UNSUPPORTED;
    }
    *A = p->A[axis];
    *B = p->B[axis];
    return DFT3D_OK;
}

dft3d_status dft3d_plan_mode_kernel(dft3d_plan p, int axis, char* name, size_t len)
{
    if (!p || axis < 0 || axis > 2 || !name || len == 0) {
        set_error("plan_mode_kernel: invalid argument");
        return DFT3D_ERR_INVALID_ARG;
    }
    if (p->form != DFT3D_KDFT) {
        // FFT plan: how dft3d_exec transforms this axis (before CLOBBER_INPUT's adjustments of the pass count)
        const char* how;
        if (p->flags & DFT3D_FLAG_UNFUSED) how = "first stage, twiddle pass, second stage";
        else if (p->n[axis] == 1) how = "identity";
        else if (axis == 2 ? z_axis_fusable(p) : strided_axis_fusable(p, axis)) how = "fused";
        else if (first_stage_is_radix(p, axis) && second_stage_nested(p, axis, axis != 2))
            how = "butterflies + fused second stage";
        else if (first_stage_is_radix(p, axis)) how = "butterflies + second stage";
        else how = "first stage + second stage";
        snprintf(name, len, "%s", how);
        return DFT3D_OK;
    }
    const char* k = single_launch(p) ? "k_kdft_small"
                    : p->complex128() ? "k_contract_f64"
                                      : contract_kernel_name(mode_args(p, axis, nullptr, nullptr, 0, 1.0f));
    snprintf(name, len, "%s", k);
    return DFT3D_OK;
}

dft3d_status dft3d_mode_contract(dft3d_plan p, int axis, const void* in, void* out, int direction,
                                 void* stream)
{
    if (p && (axis < 0 || axis > 2 || !valid_direction(direction))) {
        set_error("mode_contract: bad axis or direction");
        return DFT3D_ERR_INVALID_ARG;
    }
    dft3d_status s = check_buffers(p, in, out, "mode_contract", p ? p->stage_in_elements(axis) : -1,
                                   p ? p->stage_out_elements(axis) : -1);
    if (s != DFT3D_OK) return s;
    if (p->form != DFT3D_KDFT) { set_error("mode_contract: not a KDFT plan"); return DFT3D_ERR_UNSUPPORTED; }
    if (direction == DFT3D_BACKWARD && (p->nonuniform[axis] || p->points)) {
        set_error("mode_contract: BACKWARD is not defined for a nonuniform axis");
        return DFT3D_ERR_UNSUPPORTED;
    }
    return hip_status(run_mode(p, axis, (const float2*)in, (float2*)out, direction == DFT3D_BACKWARD,
                               axis_scale(p, axis, direction), (hipStream_t)stream),
                      "mode_contract");
}

dft3d_status dft3d_fft_first_stage(dft3d_plan p, int axis, const void* in, void* out, int direction,
                                   int fuse_twiddle, void* stream)
{
    dft3d_status s = check_buffers(p, in, out, "fft_first_stage");
    if (s != DFT3D_OK) return s;
    if (axis < 0 || axis > 2 || !valid_direction(direction)) {
        set_error("fft_first_stage: bad axis or direction");
        return DFT3D_ERR_INVALID_ARG;
    }
    if (p->form != DFT3D_FFT) { set_error("fft_first_stage: not an FFT plan"); return DFT3D_ERR_UNSUPPORTED; }
    return hip_status(run_first_stage(p, axis, (const float2*)in, (float2*)out,
                                      direction == DFT3D_BACKWARD, fuse_twiddle, (hipStream_t)stream),
                      "fft_first_stage");
}

dft3d_status dft3d_fft_phase(dft3d_plan p, int axis, const void* in, void* out, int direction,
                             void* stream)
{
    dft3d_status s = check_buffers(p, in, out, "fft_phase");
    if (s != DFT3D_OK) return s;
    if (axis < 0 || axis > 2 || !valid_direction(direction)) {
        set_error("fft_phase: bad axis or direction");
        return DFT3D_ERR_INVALID_ARG;
    }
    if (p->form != DFT3D_FFT) { set_error("fft_phase: not an FFT plan"); return DFT3D_ERR_UNSUPPORTED; }
    if (p->complex128()) {
        set_error("fft_phase: complex128 plans apply the twiddle in the first stage only");
        return DFT3D_ERR_UNSUPPORTED;
    }
    return hip_status(launch_phase((const float2*)in, (float2*)out, p->outer(axis), (int)p->A[axis],
                                   (int)p->B[axis], p->inner(axis), p->Tw[axis],
                                   direction == DFT3D_BACKWARD, (hipStream_t)stream),
                      "fft_phase");
}

dft3d_status dft3d_fft_second_stage(dft3d_plan p, int axis, const void* in, void* out, int direction,
                                    int reorder, void* stream)
{
    dft3d_status s = check_buffers(p, in, out, "fft_second_stage");
    if (s != DFT3D_OK) return s;
    if (axis < 0 || axis > 2 || !valid_direction(direction)) {
        set_error("fft_second_stage: bad axis or direction");
        return DFT3D_ERR_INVALID_ARG;
    }
    if (p->form != DFT3D_FFT) { set_error("fft_second_stage: not an FFT plan"); return DFT3D_ERR_UNSUPPORTED; }
    return hip_status(run_second_stage(p, axis, (const float2*)in, (float2*)out,
                                       direction == DFT3D_BACKWARD, axis_scale(p, axis, direction),
                                       reorder, (hipStream_t)stream),
                      "fft_second_stage");
}

dft3d_status dft3d_fft_axis(dft3d_plan p, int axis, const void* in, void* out, int direction,
                            void* stream)
{
    dft3d_status s = check_buffers(p, in, out, "fft_axis");
    if (s != DFT3D_OK) return s;
    if (axis < 0 || axis > 2 || !valid_direction(direction)) {
        set_error("fft_axis: bad axis or direction");
        return DFT3D_ERR_INVALID_ARG;
    }
    if (p->form != DFT3D_FFT) { set_error("fft_axis: not an FFT plan"); return DFT3D_ERR_UNSUPPORTED; }
    const bool ok = axis == 2 ? z_axis_fusable(p) : strided_axis_fusable(p, axis);
    if (!ok) {
        set_error("fft_axis: no fused kernel for axis %d with split %lld x %lld", axis,
                  (long long)p->A[axis], (long long)p->B[axis]);
        return DFT3D_ERR_UNSUPPORTED;
    }
    const int conj = direction == DFT3D_BACKWARD;
    const float sc = axis_scale(p, axis, direction);
    hipError_t e = axis == 2 ? run_fused_z(p, (const float2*)in, (float2*)out, conj, sc, (hipStream_t)stream)
                             : run_fused_s(p, axis, (const float2*)in, (float2*)out, conj, sc, (hipStream_t)stream);
    return hip_status(e, "fft_axis");
}

dft3d_status dft3d_fft_reorder(dft3d_plan p, int axes_mask, const void* in, void* out, void* stream)
{
    dft3d_status s = check_buffers(p, in, out, "fft_reorder");
    if (s != DFT3D_OK) return s;
    if (axes_mask < 0 || axes_mask > 7) { set_error("fft_reorder: bad axes mask"); return DFT3D_ERR_INVALID_ARG; }
    if (p->form != DFT3D_FFT) { set_error("fft_reorder: not an FFT plan"); return DFT3D_ERR_UNSUPPORTED; }
    return hip_status(run_reorder(p, axes_mask, (const float2*)in, (float2*)out, (hipStream_t)stream),
                      "fft_reorder");
}

dft3d_status dft3d_device_copy(const void* in, void* out, size_t bytes, int variant, void* stream)
{
    if (!in || !out || (bytes & 15) || ((uintptr_t)in & 15) || ((uintptr_t)out & 15) || variant < 0) {
        set_error("device_copy: pointers and size must be 16-byte multiples, variant >= 0");
        return DFT3D_ERR_INVALID_ARG;
    }
    const uintptr_t a = (uintptr_t)in, b = (uintptr_t)out;
    if (a < b + bytes && b < a + bytes) {
        set_error("device_copy: in and out overlap");
        return DFT3D_ERR_INVALID_ARG;
    }
    return hip_status(launch_copy(in, out, bytes, variant, (hipStream_t)stream), "device_copy");
}

}  // extern "C"

namespace dft3d {

// The whole transform with the workspace given explicitly (dft3d_exec passes the plan's own; the
// entry point for callers that cannot allocate passes the library's static scratch array).
dft3d_status exec_with_workspace(dft3d_plan p, const void* in, void* out, int direction, void* stream,
                                 void* workspace, size_t workspace_bytes, const char* who)
{
    dft3d_status s = check_buffers(p, in, out, who);
    if (s != DFT3D_OK) return s;
    if (!valid_direction(direction)) { set_error("%s: bad direction", who); return DFT3D_ERR_INVALID_ARG; }
    s = require_uniform_for_backward(p, direction, who);
    if (s != DFT3D_OK) return s;

    if (single_launch(p)) {
        hipStream_t sst = (hipStream_t)stream;
        const int bw = direction == DFT3D_BACKWARD;
        const float sc = bw ? axis_scale(p, 0, direction) * axis_scale(p, 1, direction) * axis_scale(p, 2, direction) : 1.0f;
        const int slot = (p->prof_next < p->prof_capacity) ? p->prof_next++ : -1;
        if (slot >= 0) (void)hipEventRecord(p->prof_events[(size_t)slot * DFT3D_MAX_PASSES * 2], sst);
        const hipError_t se = launch_kdft_small((const float2*)in, (float2*)out, p->M[0], p->M[1], p->M[2], sc, bw, sst);
        if (slot >= 0) {
            (void)hipEventRecord(p->prof_events[(size_t)slot * DFT3D_MAX_PASSES * 2 + 1], sst);
            p->prof_npass[(size_t)slot] = 1;
        }
        return hip_status(se, who);
    }

    if (p->points) {
        // in -> W1 (mode z) -> W2 (mode y) -> out (mode x); the two intermediates live in the workspace
        const size_t need = dft3d_plan_workspace_bytes(p);
        if (!workspace || workspace_bytes < need) {
            set_error("%s: a workspace of %zu bytes must be set first", who, need);
            return DFT3D_ERR_INVALID_ARG;
        }
        const uintptr_t w = (uintptr_t)workspace, a = (uintptr_t)in, b = (uintptr_t)out;
        const uintptr_t abytes = (uintptr_t)p->elements() * p->elem_bytes(), bbytes = (uintptr_t)p->out_elements() * p->elem_bytes();
        if ((w < a + abytes && a < w + need) || (w < b + bbytes && b < w + need)) {
            set_error("%s: the workspace overlaps in or out", who);
            return DFT3D_ERR_INVALID_ARG;
        }
        // (complex128 plans: the pointers are only passed through, an element is two float2)
        float2* w1 = (float2*)workspace;
        float2* w2 = w1 + p->stage_out_elements(2) * (int64_t)(p->elem_bytes() / 8);
        hipStream_t pst = (hipStream_t)stream;
        hipError_t pe = run_mode(p, 2, (const float2*)in, w1, 0, 1.0f, pst);
        if (pe == hipSuccess) pe = run_mode(p, 1, w1, w2, 0, 1.0f, pst);
        if (pe == hipSuccess) pe = run_mode(p, 0, w2, (float2*)out, 0, 1.0f, pst);
        return hip_status(pe, who);
    }

    const bool clobber = (p->flags & DFT3D_FLAG_CLOBBER_INPUT) != 0;
    float2* other = nullptr;     // the ping-pong partner of `out`
    if (clobber) {
        other = (float2*)const_cast<void*>(in);
    } else {
        const size_t need = dft3d_plan_workspace_bytes(p);
        if (!workspace || workspace_bytes < need) {
            set_error("%s: a workspace of %zu bytes must be set first", who, need);
            return DFT3D_ERR_INVALID_ARG;
        }
        // (the workspace may be larger than a tensor: padded rows)
        const uintptr_t w = (uintptr_t)workspace, bytes = (uintptr_t)need;
        const uintptr_t a = (uintptr_t)in, b = (uintptr_t)out, tbytes = (uintptr_t)p->elements() * p->elem_bytes();
        if ((w < a + tbytes && a < w + bytes) || (w < b + tbytes && b < w + bytes)) {
            set_error("%s: the workspace overlaps in or out", who);
            return DFT3D_ERR_INVALID_ARG;
        }
        other = (float2*)workspace;
    }

    hipStream_t st = (hipStream_t)stream;
    const int conj = direction == DFT3D_BACKWARD;
    const bool unfused = (p->flags & DFT3D_FLAG_UNFUSED) != 0;

    // The passes ping-pong between `out` and `other`; the pass count is odd so that, starting
    // with in -> out, the last pass also lands in `out`.
    //   KDFT: modes z, y, x (3 passes).
    //   FFT : every axis whose split has a fused kernel takes one pass (both stages, twiddle and
    //         natural order).  Otherwise: z = first stage, second stage and a transposing
    //         re-ordering pass at the end; y / x = first stage (+twiddle) and second stage with
    //         the re-ordering folded into its stores (they only change row addresses).
    //         3 passes when all axes fuse, 7 when none does.
    //   FFT unfused: per axis first stage, twiddle pass, second stage; one re-ordering pass of
    //         all three axes at the end (10 passes -> starts with in -> other).
    //   An axis of length 1 (a 2-D or 1-D transform given as n1 = 1 and/or n2 = 1) is the identity
    //   and takes no pass, unless that would leave no pass at all or, with CLOBBER_INPUT, an even
    //   number of them.
    const bool zfused = !unfused && z_axis_fusable(p);
    bool sfused[2] = {!unfused && strided_axis_fusable(p, 0), !unfused && strided_axis_fusable(p, 1)};
    bool skip[3] = {!unfused && p->n[0] == 1, !unfused && p->n[1] == 1, !unfused && p->n[2] == 1};
    // The re-ordering pass of a z axis without a fused kernel is saved when the pass right after its second
    // stage is a first stage in butterflies (y, or x when y takes no pass): that pass reads through the
    // permutation.  (Not for complex128 plans, whose first stages are contractions.)
    bool allow_zfold = true;
    auto z_folds_into = [&]() {
        if (!allow_zfold || p->form != DFT3D_FFT || unfused || zfused || skip[2] || p->x_first) return -1;
        const int next = !skip[1] ? 1 : (!skip[0] ? 0 : -1);
        if (next < 0 || sfused[next] || !first_stage_is_radix(p, next) || p->A[2] % 2 != 0 || p->A[2] < 2) return -1;
        return next;
    };
    auto count_passes = [&]() {
        if (p->form != DFT3D_FFT) return 3 - (int)skip[0] - (int)skip[1] - (int)skip[2];
        if (unfused) return 10;
        int c = 0;
        if (!skip[2]) c += zfused ? 1 : (z_folds_into() >= 0 ? 2 : 3);
        for (int axis = 0; axis < 2; ++axis)
            if (!skip[axis]) c += sfused[axis] ? 1 : 2;
        return c;
    };
    int npass = count_passes();
    if (npass == 0) {
        skip[2] = false;
        npass = count_passes();
    }
    if (clobber && (npass % 2 == 0)) {
        // ping-ponging between in and out needs an odd pass count: try, one at a time, keeping the
        // re-ordering pass of the z axis, the identity pass(es) of a length-1 axis, or splitting a fused strided
        // axis into its two stages
        bool* knobs[6] = {&allow_zfold, &skip[2], &skip[1], &skip[0], &sfused[1], &sfused[0]};
        for (bool* knob : knobs) {
            if (!*knob) continue;
            *knob = false;
            npass = count_passes();
            if (npass % 2 == 1) break;
            *knob = true;
        }
        npass = count_passes();
        if (npass % 2 == 0) {
            set_error("%s: CLOBBER_INPUT cannot be combined with this pass structure", who);
            return DFT3D_ERR_UNSUPPORTED;
        }
    }
    const float2* src = (const float2*)in;
    float2* dst = (npass % 2 == 1) ? (float2*)out : other;
    const int prof_slot = (p->prof_next < p->prof_capacity) ? p->prof_next++ : -1;
    int pass = 0;
    auto mark = [&](int which) {   // event before (0) / after (1) the current pass
        if (prof_slot < 0 || pass >= DFT3D_MAX_PASSES) return;
        (void)hipEventRecord(p->prof_events[((size_t)prof_slot * DFT3D_MAX_PASSES + pass) * 2 + which], st);
    };
    auto advance = [&]() {
        mark(1);
        ++pass;
        if (prof_slot >= 0) p->prof_npass[(size_t)prof_slot] = pass < DFT3D_MAX_PASSES ? pass : DFT3D_MAX_PASSES;
        src = dst;
        dst = (dst == (float2*)out) ? other : (float2*)out;
    };

    hipError_t e = hipSuccess;
    const int zfold = z_folds_into();      // (after the pass structure is final)
    if (p->form == DFT3D_KDFT) {
        for (int axis = 2; axis >= 0 && e == hipSuccess; --axis) {
            if (skip[axis]) continue;
            mark(0);
            e = run_mode(p, axis, src, dst, conj, axis_scale(p, axis, direction), st);
            advance();
        }
    } else {
        for (int step = 0; step < 3 && e == hipSuccess; ++step) {
            const int axis = p->x_first ? step : 2 - step;
            if (skip[axis]) continue;
            if (axis == 2 && zfused) {
                mark(0);
                e = run_fused_z(p, src, dst, conj, axis_scale(p, axis, direction), st);
                advance();
                continue;
            }
            if (axis != 2 && sfused[axis]) {
                mark(0);
                // ws_pitch is only set for plans whose passes are z: in -> out, y: out -> workspace,
                // x: workspace -> out
                e = p->ws_pitch  ? run_fused_s_padded(p, axis, src, dst, conj, axis_scale(p, axis, direction), st)
                    : p->x_first ? run_fused_s_xfirst(p, axis, src, dst, conj, axis_scale(p, axis, direction), st)
                                 : run_fused_s(p, axis, src, dst, conj, axis_scale(p, axis, direction), st);
                advance();
                continue;
            }
            mark(0);
            e = run_first_stage(p, axis, src, dst, conj, unfused ? 0 : 1, st, axis == zfold);
            advance();
            if (unfused && e == hipSuccess) {
                mark(0);
                e = launch_phase(src, dst, p->outer(axis), (int)p->A[axis], (int)p->B[axis],
                                 p->inner(axis), p->Tw[axis], conj, st);
                advance();
            }
            if (e != hipSuccess) break;
            const int fold = (!unfused && axis != 2) ? 1 : 0;
            mark(0);
            e = run_second_stage(p, axis, src, dst, conj, axis_scale(p, axis, direction), fold, st);
            advance();
        }
        if (e == hipSuccess && !zfused && !skip[2] && zfold < 0) {
            mark(0);
            e = run_reorder(p, unfused ? 7 : 4, src, dst, st);
            advance();
        }
    }
    return hip_status(e, who);
}

}  // namespace dft3d

extern "C" {

dft3d_status dft3d_exec(dft3d_plan p, const void* in, void* out, int direction, void* stream)
{
    return exec_with_workspace(p, in, out, direction, stream, p ? p->workspace : nullptr,
                               p ? p->workspace_bytes : 0, "exec");
}

}  // extern "C"
