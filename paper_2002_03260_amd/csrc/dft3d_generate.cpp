// Host-side generator of the transform matrices and twiddle tables (plan time, off the hot path).
//
// Every entry is a point on the unit circle, exp(sign * 2 pi i * t).  The argument t (in turns)
// is reduced exactly before any trigonometric call: to the nearest quarter turn q/4 plus a
// remainder |d| <= 1/8, so entries at multiples of a quarter turn come out as exact 0 / +-1 and
// every other entry carries one fp64 rounding of the angle plus libm's error, far below the
// single rounding to fp32 that follows.
//
//   uniform axis     M[k, n] = exp(-2 pi i (k n mod N) / N)          paper Eq. 3 (roots of unity), Eq. 12
//   nonuniform axis  M[k, n] = exp(-2 pi i frac(k c[n]))             Eq. 3 with unit-circle points
//   twiddle          T[k_a, beta] = exp(-2 pi i beta k_a / (A B))    diagonal factor of Eq. 15
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <vector>

#include "dft3d_internal.h"

namespace dft3d {

namespace {

constexpr double kTwoPi = 6.283185307179586476925286766559;

// quarter in {0,1,2,3}; d in [-1/8, 1/8] turns.  Rotating (cos, sin)(2 pi d) by quarter turns.
inline void finish_root(int quarter, double d, int sign, double* re, double* im)
{
    double c = std::cos(kTwoPi * d);
    double s = std::sin(kTwoPi * d);
    double cr, ci;
    switch (quarter & 3) {
        case 0: cr = c;  ci = s;  break;
        case 1: cr = -s; ci = c;  break;
        case 2: cr = -c; ci = -s; break;
        default: cr = s; ci = -c; break;
    }
    *re = cr;
    *im = (sign < 0) ? -ci : ci;
}

}  // namespace

void unit_root_ratio(int64_t p, int64_t q, int sign, double* re, double* im)
{
    // r = p mod q in [0, q); 4r = quarter*q + m with m in [-q/2, q/2]
    int64_t r = p % q;
    if (r < 0) r += q;
    int64_t quarter = (8 * r + q) / (2 * q);
    int64_t m = 4 * r - quarter * q;
    double d = (double)m / (4.0 * (double)q);
    finish_root((int)(quarter & 3), d, sign, re, im);
}

void unit_root_turns(double t, int sign, double* re, double* im)
{
    t -= std::floor(t);                       // [0, 1)
    double qf = std::nearbyint(4.0 * t);      // 0..4
    double d = t - 0.25 * qf;                 // exact: both operands are multiples of ulp(t)
    finish_root((int)qf & 3, d, sign, re, im);
}

}  // namespace dft3d

using namespace dft3d;

static const double kTwoPiGen = 6.283185307179586476925286766559;

extern "C" dft3d_status dft3d_generate_matrix(int64_t n, const double* coords, int direction,
                                              float* re, float* im)
{
    if (n < 1 || !re || !im || (direction != DFT3D_FORWARD && direction != DFT3D_BACKWARD)) {
        set_error("dft3d_generate_matrix: invalid argument");
        return DFT3D_ERR_INVALID_ARG;
    }
    if (coords)
        for (int64_t j = 0; j < n; ++j)
            if (!std::isfinite(coords[j])) {
                set_error("dft3d_generate_matrix: coordinate %lld is not finite", (long long)j);
                return DFT3D_ERR_INVALID_ARG;
            }
    for (int64_t k = 0; k < n; ++k) {
        for (int64_t j = 0; j < n; ++j) {
            double cr, ci;
            if (coords) unit_root_turns((double)k * coords[j], direction, &cr, &ci);
            else unit_root_ratio(k * j, n, direction, &cr, &ci);
            re[k * n + j] = (float)cr;
            im[k * n + j] = (float)ci;
        }
    }
    return DFT3D_OK;
}

extern "C" dft3d_status dft3d_generate_twiddle(int64_t A, int64_t B, int direction, float* re,
                                               float* im)
{
    if (A < 1 || B < 1 || !re || !im ||
        (direction != DFT3D_FORWARD && direction != DFT3D_BACKWARD)) {
        set_error("dft3d_generate_twiddle: invalid argument");
        return DFT3D_ERR_INVALID_ARG;
    }
    for (int64_t ka = 0; ka < A; ++ka) {
        for (int64_t b = 0; b < B; ++b) {
            double cr, ci;
            unit_root_ratio(ka * b, A * B, direction, &cr, &ci);
            re[ka * B + b] = (float)cr;
            im[ka * B + b] = (float)ci;
        }
    }
    return DFT3D_OK;
}

namespace dft3d {
// V[r, j] = z_r^{-j} in fp64 (Eq. 3 as printed): modulus by exp/log, phase through the exactly reduced
// fraction of a turn (so points on the unit circle keep unit modulus).
dft3d_status generate_points_matrix_f64(int64_t k, int64_t n, const double* z, double* re, double* im)
{
    if (k < 1 || n < 1 || !z || !re || !im) {
        set_error("dft3d_generate_points_matrix: invalid argument");
        return DFT3D_ERR_INVALID_ARG;
    }
    for (int64_t r = 0; r < k; ++r) {
        const double zr = z[2 * r], zi = z[2 * r + 1];
        const double mod = std::hypot(zr, zi);
        if (!(mod > 0.0) || !std::isfinite(mod)) {
            set_error("dft3d_generate_points_matrix: point %lld is zero or not finite", (long long)r);
            return DFT3D_ERR_INVALID_ARG;
        }
        const double turns = std::atan2(zi, zr) / kTwoPiGen;
        const double lnmod = (mod == 1.0) ? 0.0 : std::log(mod);
        for (int64_t j = 0; j < n; ++j) {
            double cr, ci;
            unit_root_turns((double)j * turns, DFT3D_FORWARD, &cr, &ci);
            const double m = (lnmod == 0.0) ? 1.0 : std::exp(-(double)j * lnmod);
            re[r * n + j] = m * cr;
            im[r * n + j] = m * ci;
            if (!std::isfinite(re[r * n + j]) || !std::isfinite(im[r * n + j])) {
                set_error("dft3d_generate_points_matrix: entry (%lld, %lld) overflows", (long long)r, (long long)j);
                return DFT3D_ERR_INVALID_ARG;
            }
        }
    }
    return DFT3D_OK;
}
}  // namespace dft3d

extern "C" dft3d_status dft3d_generate_points_matrix(int64_t k, int64_t n, const double* z, float* re,
                                                     float* im)
{
    if (k < 1 || n < 1 || !z || !re || !im) {
        set_error("dft3d_generate_points_matrix: invalid argument");
        return DFT3D_ERR_INVALID_ARG;
    }
    std::vector<double> dre((size_t)(k * n)), dim((size_t)(k * n));
    const dft3d_status s = dft3d::generate_points_matrix_f64(k, n, z, dre.data(), dim.data());
    if (s != DFT3D_OK) return s;
    for (int64_t e = 0; e < k * n; ++e) {
        const float fr = (float)dre[(size_t)e], fi = (float)dim[(size_t)e];
        if (!std::isfinite(fr) || !std::isfinite(fi)) {
            set_error("dft3d_generate_points_matrix: entry (%lld, %lld) overflows fp32", (long long)(e / n), (long long)(e % n));
            return DFT3D_ERR_INVALID_ARG;
        }
        re[e] = fr;
        im[e] = fi;
    }
    return DFT3D_OK;
}
