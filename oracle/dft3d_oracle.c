/*
 * CPU oracle for the 3D complex DFT on a tensor-product grid.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain, fp64 statement of what the GPU library must compute.  It is
 * used by the tests, by the smoke check and by the benchmark's CPU-baseline leg; the product
 * path never calls it, and it shares no code, header, table or constant with the HIP sources.
 *
 * What it evaluates (paper, Section III-A):
 *   - Eq. 1 / Eq. 3: a 1-D general DFT is the product of a Vandermonde matrix with the data.
 *   - Eq. 5, Eq. 10, Eq. 11: on a rectangular grid the 2-D / 3-D transform is that product
 *     applied to every mode of the tensor (V1 (x) V2 (x) V3 acting on the row-major vector).
 *   - Eq. 12 (Section III-B): on a uniform grid the matrix entries are exp(-2 pi i n k / N).
 *
 * Readings taken where the paper is silent:
 *   - forward transform: negative exponent, no scaling (Eq. 1 and Eq. 12 agree on this);
 *   - backward transform (uniform axes only): positive exponent, scaled by 1/(N1 N2 N3);
 *   - nonuniform axis: M[k, n] = exp(-2 pi i k c[n]) with integer frequency k = 0..N-1 and
 *     c[n] the sample coordinate in cycles (period 1);
 *   - tensors are C-ordered, last index fastest, complex numbers stored as (re, im) pairs.
 *
 * Everything is accumulated in plain fp64 in the order the sums are written.  No FFT, no BLAS,
 * no re-association of any sum.  OpenMP only splits independent output elements across threads.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_TWO_PI 6.283185307179586476925286766559

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Fraction of a turn, in [0,1), of the phase of entry (k, n).
 * Uniform axis (coords == NULL): (k*n mod N)/N, reduced in integers so no precision is lost
 * for large k*n.  Nonuniform axis: frac(k * c[n]) evaluated in fp64. */
static double oracle_phase_turns(int64_t k, int64_t n, int64_t N, const double* coords)
{
    if (coords == NULL) {
        /* k, n < 2^31 in every use here, so the product fits in 63 bits */
        int64_t r = (int64_t)(((unsigned long long)k * (unsigned long long)n) % (unsigned long long)N);
        return (double)r / (double)N;
    }
    double t = (double)k * coords[n];
    t = t - floor(t);
    return t;
}

/*
 * Rows of the per-axis transform matrix (Eq. 3 with the points on the unit circle):
 *   M[r, n] = exp(sign * 2 pi i * turns(ks[r], n)),   r = 0..K-1, n = 0..N-1.
 * ks == NULL means the rows are the frequencies 0..K-1.  sign = -1 forward, +1 backward.
 * M is K x N, row-major, interleaved (re, im) doubles.
 */
void oracle_dft_matrix(int64_t K, int64_t N, const int64_t* ks, const double* coords, int sign,
                       double* M)
{
    for (int64_t r = 0; r < K; ++r) {
        int64_t k = ks ? ks[r] : r;
        for (int64_t n = 0; n < N; ++n) {
            double t = oracle_phase_turns(k, n, N, coords);
            double ang = (double)sign * ORACLE_TWO_PI * t;
            M[2 * (r * N + n) + 0] = cos(ang);
            M[2 * (r * N + n) + 1] = sin(ang);
        }
    }
}

/*
 * Vandermonde matrix of Eq. 3 for K arbitrary non-zero points z_r of the z-plane:
 *   M[r, n] = z_r^{-n},  n = 0..N-1,
 * built literally as the powers 1, w, w^2, ... of w = 1/z_r by repeated complex multiplication
 * (error grows like n * 1e-16, far below fp32 resolution for the lengths used here).
 * z: K (re, im) pairs.  M: K x N, row-major, interleaved doubles.
 */
void oracle_points_matrix(int64_t K, int64_t N, const double* z, double* M)
{
    for (int64_t r = 0; r < K; ++r) {
        double zr = z[2 * r], zi = z[2 * r + 1];
        double d = zr * zr + zi * zi;
        double wr = zr / d, wi = -zi / d;           /* w = 1 / z */
        double pr = 1.0, pi = 0.0;
        for (int64_t n = 0; n < N; ++n) {
            M[2 * (r * N + n)] = pr;
            M[2 * (r * N + n) + 1] = pi;
            double tr = pr * wr - pi * wi;
            pi = pr * wi + pi * wr;
            pr = tr;
        }
    }
}

/*
 * One mode product (Eq. 2 applied along one index of a tensor, the building block of Eq. 5
 * and Eq. 11):   out[o, k, i] = sum_n M[k, n] * in[o, n, i]
 * in  is O x N x I, out is O x K x I, M is K x N; complex, row-major, interleaved; M and out
 * are fp64, in is fp64 (oracle_mode_contract) or fp32 promoted exactly (oracle_mode_contract_f32).
 * Each output is one sum taken in the order n = 0..N-1.  Threads only split independent
 * outputs: (o, k) pairs and, inside one pair, ranges of i.
 */
#define ORACLE_IBLOCK 2048
#define ORACLE_MODE_CONTRACT_BODY(IN_T)                                                      \
    int64_t OK = O * K;                                                                       \
    int64_t nib = (I + ORACLE_IBLOCK - 1) / ORACLE_IBLOCK;                                    \
    _Pragma("omp parallel for collapse(2) schedule(static)")                                  \
    for (int64_t ok = 0; ok < OK; ++ok) {                                                     \
        for (int64_t ib = 0; ib < nib; ++ib) {                                                \
            int64_t o = ok / K, k = ok % K;                                                   \
            int64_t i0 = ib * ORACLE_IBLOCK;                                                  \
            int64_t i1 = i0 + ORACLE_IBLOCK < I ? i0 + ORACLE_IBLOCK : I;                     \
            double* dst = out + 2 * ((o * K + k) * I);                                        \
            for (int64_t i = i0; i < i1; ++i) { dst[2 * i] = 0.0; dst[2 * i + 1] = 0.0; }     \
            for (int64_t n = 0; n < N; ++n) {                                                 \
                double mr = M[2 * (k * N + n)], mi = M[2 * (k * N + n) + 1];                  \
                const IN_T* src = in + 2 * ((o * N + n) * I);                                 \
                for (int64_t i = i0; i < i1; ++i) {                                           \
                    double xr = (double)src[2 * i], xi = (double)src[2 * i + 1];              \
                    dst[2 * i]     += mr * xr - mi * xi;                                      \
                    dst[2 * i + 1] += mr * xi + mi * xr;                                      \
                }                                                                             \
            }                                                                                 \
        }                                                                                     \
    }

void oracle_mode_contract(int64_t O, int64_t N, int64_t I, int64_t K, const double* M,
                          const double* in, double* out)
{
    ORACLE_MODE_CONTRACT_BODY(double)
}

void oracle_mode_contract_f32(int64_t O, int64_t N, int64_t I, int64_t K, const double* M,
                              const float* in, double* out)
{
    ORACLE_MODE_CONTRACT_BODY(float)
}

/*
 * Full 3-D transform, one axis at a time (Eq. 11): out = (M1 (x) M2 (x) M3) in.
 * in: n1 x n2 x n3 complex64 (floats), promoted exactly to fp64.  out: complex128.
 * c1/c2/c3: NULL for a uniform axis, else n? sample coordinates in cycles.
 * sign: -1 forward, +1 backward.  scale_backward != 0 multiplies the result by 1/(n1 n2 n3).
 * Returns 0, or -1 if scratch memory could not be allocated.
 */
int oracle_dft3d(int64_t n1, int64_t n2, int64_t n3, const float* in, double* out,
                 const double* c1, const double* c2, const double* c3, int sign,
                 int scale_backward)
{
    int64_t E = n1 * n2 * n3;
    int64_t nmax = n1 > n2 ? n1 : n2;
    if (n3 > nmax) nmax = n3;
    double* M = (double*)malloc(sizeof(double) * 2 * (size_t)(nmax * nmax));
    double* a = (double*)malloc(sizeof(double) * 2 * (size_t)E);
    if (!M || !a) { free(M); free(a); return -1; }

    for (int64_t e = 0; e < 2 * E; ++e) a[e] = (double)in[e];

    /* mode 1: a (n1 x [n2 n3]) -> out */
    oracle_dft_matrix(n1, n1, NULL, c1, sign, M);
    oracle_mode_contract(1, n1, n2 * n3, n1, M, a, out);
    /* mode 2: out ([n1] x n2 x [n3]) -> a */
    oracle_dft_matrix(n2, n2, NULL, c2, sign, M);
    oracle_mode_contract(n1, n2, n3, n2, M, out, a);
    /* mode 3: a ([n1 n2] x n3) -> out */
    oracle_dft_matrix(n3, n3, NULL, c3, sign, M);
    oracle_mode_contract(n1 * n2, n3, 1, n3, M, a, out);

    if (scale_backward) {
        double s = 1.0 / (double)E;
        for (int64_t e = 0; e < 2 * E; ++e) out[e] *= s;
    }
    free(M);
    free(a);
    return 0;
}

/*
 * The defining triple sum of Eq. 10 written out literally, one output at a time, with the
 * three phases added as fractions of a turn before a single complex exponential is taken.
 * O((n1 n2 n3)^2): for tiny tensors only.  Used to pin oracle_dft3d.
 */
void oracle_dft3d_brute(int64_t n1, int64_t n2, int64_t n3, const float* in, double* out,
                        const double* c1, const double* c2, const double* c3, int sign)
{
    for (int64_t k1 = 0; k1 < n1; ++k1)
    for (int64_t k2 = 0; k2 < n2; ++k2)
    for (int64_t k3 = 0; k3 < n3; ++k3) {
        double sr = 0.0, si = 0.0;
        for (int64_t a = 0; a < n1; ++a)
        for (int64_t b = 0; b < n2; ++b)
        for (int64_t c = 0; c < n3; ++c) {
            double t = oracle_phase_turns(k1, a, n1, c1) + oracle_phase_turns(k2, b, n2, c2) +
                       oracle_phase_turns(k3, c, n3, c3);
            double ang = (double)sign * ORACLE_TWO_PI * t;
            double wr = cos(ang), wi = sin(ang);
            int64_t e = (a * n2 + b) * n3 + c;
            double xr = (double)in[2 * e], xi = (double)in[2 * e + 1];
            sr += xr * wr - xi * wi;
            si += xr * wi + xi * wr;
        }
        int64_t eo = (k1 * n2 + k2) * n3 + k3;
        out[2 * eo] = sr;
        out[2 * eo + 1] = si;
    }
}
