// Drives the C ABI of libdft3d on the CPU, against the stand-in HIP runtime, under ASan + UBSan:
// plan creation (generator, uploads), argument validation, and for every exec the sequence of kernel
// launches -- which buffer each pass reads and writes, that every launch stays inside its buffers, and
// that plans free what they allocate.  Prints one line per group of scenarios; exit status 0 = all held.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <string>
#include <vector>

#include "dft3d.h"
#include "hostsim.h"

static int g_failed = 0;
static long g_checked = 0;

#define EXPECT(cond, ...)                                   \
    do {                                                    \
        ++g_checked;                                        \
        if (!(cond)) {                                      \
            ++g_failed;                                     \
            printf("FAILED %s:%d: %s -- ", __FILE__, __LINE__, #cond); \
            printf(__VA_ARGS__);                            \
            printf("\n");                                   \
        }                                                   \
    } while (0)

struct Case {
    int64_t n[3];
    dft3d_formulation form;
    uint32_t flags;
    bool nonuniform;
    int64_t split[3];      // 0 = default
    std::string label() const
    {
        char b[160];
        snprintf(b, sizeof(b), "%lldx%lldx%lld %s flags 0x%x%s split %lld,%lld,%lld", (long long)n[0], (long long)n[1],
                 (long long)n[2], form == DFT3D_KDFT ? "KDFT" : "FFT", flags, nonuniform ? " nonuniform" : "",
                 (long long)split[0], (long long)split[1], (long long)split[2]);
        return b;
    }
};

// One plan, forward and (where defined) backward exec, launch log checked.  Returns the number of passes.
static int run_case(const Case& c)
{
    const std::string lab = c.label();
    std::vector<double> cx, cy, cz;
    if (c.nonuniform) {
        std::mt19937_64 rng(c.n[0] * 131 + c.n[1] * 17 + c.n[2]);
        std::uniform_real_distribution<double> u(0.0, 1.0);
        for (auto* v : {&cx, &cy, &cz}) {
            const int64_t n = c.n[v == &cx ? 0 : (v == &cy ? 1 : 2)];
            v->resize(n);
            for (auto& x : *v) x = u(rng);
        }
    }
    dft3d_plan plan = nullptr;
    dft3d_status s = dft3d_plan_create_ex(&plan, c.n[0], c.n[1], c.n[2], c.form, c.nonuniform ? cx.data() : nullptr,
                                          c.nonuniform ? cy.data() : nullptr, c.nonuniform ? cz.data() : nullptr,
                                          (c.split[0] || c.split[1] || c.split[2]) ? c.split : nullptr, c.flags);
    if (s == DFT3D_ERR_UNSUPPORTED) return -1;       // combination not offered
    EXPECT(s == DFT3D_OK && plan, "%s: plan_create -> %s (%s)", lab.c_str(), dft3d_status_string(s), dft3d_last_error());
    if (s != DFT3D_OK) return -1;

    const size_t esz = (c.flags & DFT3D_FLAG_COMPLEX128) ? 16 : 8;
    const size_t bytes = (size_t)(c.n[0] * c.n[1] * c.n[2]) * esz;
    const size_t wsb = dft3d_plan_workspace_bytes(plan);
    const bool clobber = (c.flags & DFT3D_FLAG_CLOBBER_INPUT) != 0;
    // (HOSTSIM_SHORT_OUTPUT registers an output tensor that is one element short: the launch checks of
    // the stand-in runtime must then report the last pass -- the test of the checker itself)
    const size_t short_by = getenv("HOSTSIM_SHORT_OUTPUT") ? esz : 0;
    void* in = hostsim_reserve(bytes);
    void* out = hostsim_reserve(bytes - short_by);
    void* ws = wsb ? hostsim_reserve(wsb) : nullptr;
    EXPECT(in && out && (ws || !wsb), "%s: reserve", lab.c_str());
    if (wsb) {
        s = dft3d_plan_set_workspace(plan, ws, wsb);
        EXPECT(s == DFT3D_OK, "%s: set_workspace -> %s", lab.c_str(), dft3d_last_error());
    }
    int npass_seen = 0;
    for (int dir : {DFT3D_FORWARD, DFT3D_BACKWARD}) {
        if (dir == DFT3D_BACKWARD && (c.nonuniform || (c.flags & DFT3D_FLAG_ADJOINT))) {
            s = dft3d_exec(plan, in, out, dir, nullptr);
            if (c.nonuniform) EXPECT(s == DFT3D_ERR_UNSUPPORTED, "%s: backward on nonuniform axes must be refused", lab.c_str());
            continue;
        }
        hostsim_clear_log();
        EXPECT(dft3d_plan_enable_profiling(plan, 1) == DFT3D_OK, "%s: enable_profiling", lab.c_str());
        s = dft3d_exec(plan, in, out, dir, nullptr);
        if (s == DFT3D_ERR_UNSUPPORTED && clobber) continue;      // pass structure cannot ping-pong in place
        EXPECT(s == DFT3D_OK, "%s: exec -> %s (%s)", lab.c_str(), dft3d_status_string(s), dft3d_last_error());
        if (s != DFT3D_OK) continue;
        float ms[DFT3D_MAX_PASSES];
        int npass = 0;
        EXPECT(dft3d_plan_read_profile(plan, 0, ms, &npass) == DFT3D_OK, "%s: read_profile", lab.c_str());
        const size_t nl = hostsim_launch_count();
        const hostsim_launch* L = hostsim_launches();
        EXPECT((int)nl == npass && nl >= 1 && nl <= DFT3D_MAX_PASSES, "%s: %zu launches, %d passes reported", lab.c_str(), nl, npass);
        npass_seen = (int)nl;
        EXPECT(!hostsim_failure(), "%s: %s", lab.c_str(), hostsim_failure() ? hostsim_failure() : "");
        // the ping-pong chain: in -> .. -> out, every pass out of place, `in` written only with CLOBBER_INPUT
        const void* expect_src = in;
        for (size_t i = 0; i < nl; ++i) {
            if (!L[i].src || !L[i].dst) {       // arguments of this kernel are not decoded: the chain restarts after it
                expect_src = nullptr;
                continue;
            }
            if (expect_src) EXPECT(L[i].src == expect_src, "%s: pass %zu (%s) reads %p, expected %p", lab.c_str(), i, L[i].name, L[i].src, expect_src);
            EXPECT(L[i].src != L[i].dst, "%s: pass %zu (%s) runs in place", lab.c_str(), i, L[i].name);
            EXPECT(L[i].dst == out || L[i].dst == ws || (clobber && L[i].dst == in), "%s: pass %zu (%s) writes %p (in %p out %p ws %p)",
                   lab.c_str(), i, L[i].name, L[i].dst, in, out, ws);
            if (!clobber) EXPECT(L[i].dst != in, "%s: pass %zu (%s) overwrites the input", lab.c_str(), i, L[i].name);
            expect_src = L[i].dst;
        }
        if (L[nl - 1].dst) EXPECT(L[nl - 1].dst == out, "%s: the last pass (%s) does not write `out`", lab.c_str(), L[nl - 1].name);
        // the entry point that allocates nothing launches the same kernels on its own scratch array
        if (wsb && wsb <= DFT3D_NOALLOC_MAX_BYTES && !clobber) {
            std::vector<std::string> names;
            for (size_t i = 0; i < nl; ++i) names.push_back(L[i].name);
            const size_t live = hostsim_live_allocations();
            hostsim_clear_log();
            s = dft3d_exec_noalloc(plan, in, out, dir, nullptr);
            EXPECT(s == DFT3D_OK, "%s: exec_noalloc -> %s", lab.c_str(), dft3d_last_error());
            EXPECT(hostsim_live_allocations() == live, "%s: exec_noalloc changed the set of allocations", lab.c_str());
            const size_t n2 = hostsim_launch_count();
            EXPECT(n2 == names.size(), "%s: exec_noalloc launches %zu kernels, exec %zu", lab.c_str(), n2, names.size());
            const hostsim_launch* L2 = hostsim_launches();
            for (size_t i = 0; i < n2 && i < names.size(); ++i) {
                EXPECT(names[i] == L2[i].name, "%s: exec_noalloc pass %zu is %s", lab.c_str(), i, L2[i].name);
                if (L2[i].dst) EXPECT(L2[i].dst != ws, "%s: exec_noalloc uses the plan's workspace", lab.c_str());
            }
            EXPECT(!hostsim_failure(), "%s: exec_noalloc: %s", lab.c_str(), hostsim_failure() ? hostsim_failure() : "");
        }
    }
    // argument errors never launch
    hostsim_clear_log();
    EXPECT(dft3d_exec(plan, in, in, DFT3D_FORWARD, nullptr) == DFT3D_ERR_INVALID_ARG, "%s: in-place exec", lab.c_str());
    EXPECT(dft3d_exec(plan, (char*)in + 8, out, DFT3D_FORWARD, nullptr) == DFT3D_ERR_INVALID_ARG, "%s: misaligned in", lab.c_str());
    EXPECT(dft3d_exec(plan, in, out, 0, nullptr) == DFT3D_ERR_INVALID_ARG, "%s: bad direction", lab.c_str());
    EXPECT(hostsim_launch_count() == 0, "%s: a refused call launched a kernel", lab.c_str());
    EXPECT(dft3d_plan_destroy(plan) == DFT3D_OK, "%s: destroy", lab.c_str());
    hostsim_release(in, bytes);
    hostsim_release(out, bytes - short_by);
    if (ws) hostsim_release(ws, wsb);
    return npass_seen;
}

static void steps_case(int64_t nx, int64_t ny, int64_t nz, uint32_t flags)
{
    // single-step entry points of an FFT plan and of a KDFT plan, every axis
    const size_t esz = (flags & DFT3D_FLAG_COMPLEX128) ? 16 : 8;
    const size_t bytes = (size_t)(nx * ny * nz) * esz;
    void* in = hostsim_reserve(bytes);
    void* out = hostsim_reserve(bytes);
    dft3d_plan pf = nullptr, pk = nullptr;
    EXPECT(dft3d_plan_create_ex(&pf, nx, ny, nz, DFT3D_FFT, nullptr, nullptr, nullptr, nullptr, flags) == DFT3D_OK, "fft plan");
    EXPECT(dft3d_plan_create_ex(&pk, nx, ny, nz, DFT3D_KDFT, nullptr, nullptr, nullptr, nullptr, flags) == DFT3D_OK, "kdft plan");
    for (int axis = 0; axis < 3 && pf && pk; ++axis)
        for (int dir : {DFT3D_FORWARD, DFT3D_BACKWARD}) {
            hostsim_clear_log();
            EXPECT(dft3d_mode_contract(pk, axis, in, out, dir, nullptr) == DFT3D_OK, "mode_contract axis %d: %s", axis, dft3d_last_error());
            EXPECT(dft3d_fft_first_stage(pf, axis, in, out, dir, 1, nullptr) == DFT3D_OK, "first_stage axis %d: %s", axis, dft3d_last_error());
            EXPECT(dft3d_fft_first_stage(pf, axis, in, out, dir, 0, nullptr) == DFT3D_OK, "first_stage (no twiddle) axis %d", axis);
            EXPECT(dft3d_fft_second_stage(pf, axis, in, out, dir, 0, nullptr) == DFT3D_OK, "second_stage axis %d", axis);
            EXPECT(dft3d_fft_second_stage(pf, axis, in, out, dir, 1, nullptr) == DFT3D_OK, "second_stage+reorder axis %d", axis);
            if (!(flags & DFT3D_FLAG_COMPLEX128)) EXPECT(dft3d_fft_phase(pf, axis, in, out, dir, nullptr) == DFT3D_OK, "phase axis %d", axis);
            const dft3d_status sa = dft3d_fft_axis(pf, axis, in, out, dir, nullptr);
            EXPECT(sa == DFT3D_OK || sa == DFT3D_ERR_UNSUPPORTED, "fft_axis axis %d: %s", axis, dft3d_last_error());
            EXPECT(dft3d_fft_reorder(pf, 1 << axis, in, out, nullptr) == DFT3D_OK, "reorder axis %d", axis);
            const size_t nl = hostsim_launch_count();
            const hostsim_launch* L = hostsim_launches();
            for (size_t i = 0; i < nl; ++i)
                if (L[i].src) EXPECT(L[i].src == in && L[i].dst == out, "step launch %s touches other buffers", L[i].name);
            EXPECT(!hostsim_failure(), "%lldx%lldx%lld steps: %s", (long long)nx, (long long)ny, (long long)nz, hostsim_failure() ? hostsim_failure() : "");
            char name[64];
            EXPECT(dft3d_plan_mode_kernel(pk, axis, name, sizeof(name)) == DFT3D_OK && name[0], "mode_kernel");
        }
    dft3d_plan_destroy(pf);
    dft3d_plan_destroy(pk);
    hostsim_release(in, bytes);
    hostsim_release(out, bytes);
}

static void points_case(bool adjoint)
{
    const int64_t n[3] = {40, 33, 70}, k[3] = {33, 50, 70};
    std::vector<double> z[3];
    std::mt19937_64 rng(5);
    std::uniform_real_distribution<double> u(0.0, 1.0);
    for (int j = 0; j < 3; ++j)
        for (int64_t r = 0; r < k[j]; ++r) {
            const double mod = 1.0 + (u(rng) - 0.5) / n[j], ph = 6.283185307179586 * u(rng);
            z[j].push_back(mod * std::cos(ph));
            z[j].push_back(mod * std::sin(ph));
        }
    dft3d_plan p = nullptr;
    dft3d_status s = dft3d_plan_create_points(&p, n[0], n[1], n[2], k[0], k[1], k[2], z[0].data(), z[1].data(), nullptr,
                                              adjoint ? DFT3D_FLAG_ADJOINT : 0);
    EXPECT(s == DFT3D_OK, "points plan: %s", dft3d_last_error());
    if (s != DFT3D_OK) return;
    const size_t ib = (size_t)(adjoint ? k[0] * k[1] * k[2] : n[0] * n[1] * n[2]) * 8;
    const size_t ob = (size_t)(adjoint ? n[0] * n[1] * n[2] : k[0] * k[1] * k[2]) * 8;
    const size_t wsb = dft3d_plan_workspace_bytes(p);
    void* in = hostsim_reserve(ib);
    void* out = hostsim_reserve(ob);
    void* ws = hostsim_reserve(wsb);
    EXPECT(dft3d_exec(p, in, out, DFT3D_FORWARD, nullptr) == DFT3D_ERR_INVALID_ARG, "points exec without workspace");
    EXPECT(dft3d_plan_set_workspace(p, ws, wsb - 8) == DFT3D_ERR_INVALID_ARG, "short workspace");
    EXPECT(dft3d_plan_set_workspace(p, ws, wsb) == DFT3D_OK, "workspace");
    hostsim_clear_log();
    EXPECT(dft3d_exec(p, in, out, DFT3D_FORWARD, nullptr) == DFT3D_OK, "points exec: %s", dft3d_last_error());
    EXPECT(hostsim_launch_count() == 3, "points exec: three mode products");
    EXPECT(!hostsim_failure(), "points exec: %s", hostsim_failure() ? hostsim_failure() : "");
    EXPECT(dft3d_exec(p, in, out, DFT3D_BACKWARD, nullptr) == DFT3D_ERR_UNSUPPORTED, "points backward");
    dft3d_plan_destroy(p);
    hostsim_release(in, ib);
    hostsim_release(out, ob);
    hostsim_release(ws, wsb);
}

int main()
{
    const size_t baseline_allocs = hostsim_live_allocations();      // device variables of the library
    // ---- the five named configurations (and the 2-D size), both formulations where defined
    const Case named[] = {
        {{32, 32, 32}, DFT3D_KDFT, 0, false, {0, 0, 0}},
        {{256, 256, 256}, DFT3D_KDFT, 0, false, {0, 0, 0}},
        {{256, 256, 256}, DFT3D_KDFT, DFT3D_FLAG_BF16X3, false, {0, 0, 0}},
        {{256, 256, 256}, DFT3D_KDFT, DFT3D_FLAG_COMPLEX128, false, {0, 0, 0}},
        {{512, 512, 512}, DFT3D_FFT, 0, false, {16, 16, 16}},
        {{512, 512, 512}, DFT3D_FFT, DFT3D_FLAG_UNFUSED, false, {16, 16, 16}},
        {{128, 128, 128}, DFT3D_KDFT, 0, true, {0, 0, 0}},
        {{2048, 2048, 2048}, DFT3D_KDFT, 0, false, {0, 0, 0}},
        {{2048, 2048, 2048}, DFT3D_KDFT, DFT3D_FLAG_CLOBBER_INPUT | DFT3D_FLAG_3M, false, {0, 0, 0}},
        {{2048, 2048, 2048}, DFT3D_FFT, 0, false, {32, 32, 32}},
        {{2048, 2048, 2048}, DFT3D_FFT, DFT3D_FLAG_CLOBBER_INPUT, false, {32, 32, 32}},
        // default split of 2048: 16 x 128 with the second factor split again; x pass first, transposed intermediate
        {{2048, 2048, 2048}, DFT3D_FFT, 0, false, {0, 0, 0}},
        {{2048, 2048, 2048}, DFT3D_FFT, DFT3D_FLAG_CLOBBER_INPUT, false, {0, 0, 0}},
        {{2048, 48, 1024}, DFT3D_FFT, 0, false, {0, 0, 0}},
        {{2048, 512, 2048}, DFT3D_FFT, 0, false, {0, 0, 0}},
        {{32, 2048, 16}, DFT3D_FFT, 0, false, {0, 0, 0}},
        {{1, 8192, 8192}, DFT3D_KDFT, 0, false, {0, 0, 0}},
        {{1, 8192, 8192}, DFT3D_FFT, DFT3D_FLAG_CLOBBER_INPUT, false, {0, 0, 0}},
        // first factor 2, 4 or 8 in vector arithmetic, second factor on the fused kernels
        {{1, 8192, 8192}, DFT3D_FFT, 0, false, {0, 0, 0}},
        {{1, 16384, 16384}, DFT3D_FFT, 0, false, {0, 0, 0}},
        {{8, 4096, 1024}, DFT3D_FFT, 0, false, {2, 2, 2}},
        {{4096, 3, 4112}, DFT3D_FFT, 0, false, {8, 1, 2}},
    };
    for (const Case& c : named) {
        const int np = run_case(c);
        printf("  %-60s %d passes\n", c.label().c_str(), np);
    }
    printf("named configurations: %ld checks, %d failed\n", g_checked, g_failed);

    // ---- seeded sweep over shapes next to the tile edges, formulations, flags
    std::mt19937_64 rng(20020326);
    const int64_t pool[] = {1, 2, 3, 5, 8, 15, 16, 17, 24, 31, 32, 33, 48, 63, 64, 65, 96, 127, 128, 129, 130, 160, 192, 256, 512};
    const int npool = (int)(sizeof(pool) / sizeof(pool[0]));
    int ran = 0, refused = 0;
    for (int it = 0; it < 400; ++it) {
        Case c{};
        for (int j = 0; j < 3; ++j) c.n[j] = pool[rng() % npool];
        if (c.n[0] * c.n[1] * c.n[2] > (int64_t)1 << 24) continue;
        c.form = (rng() % 100 < 45) ? DFT3D_FFT : DFT3D_KDFT;
        if (rng() % 100 < 30) c.flags |= DFT3D_FLAG_CLOBBER_INPUT;
        if (c.form == DFT3D_KDFT) {
            if (rng() % 100 < 25) c.flags |= DFT3D_FLAG_3M;
            if (rng() % 100 < 25) c.flags |= DFT3D_FLAG_BF16X3;
            if (rng() % 100 < 15) c.flags = (c.flags & DFT3D_FLAG_CLOBBER_INPUT) | DFT3D_FLAG_COMPLEX128;
            if (rng() % 100 < 15) c.flags |= DFT3D_FLAG_ADJOINT;
            c.nonuniform = rng() % 100 < 25;
        } else {
            if (rng() % 100 < 20 && !(c.flags & DFT3D_FLAG_CLOBBER_INPUT)) c.flags |= DFT3D_FLAG_UNFUSED;
            if (rng() % 100 < 15) c.flags = (c.flags & DFT3D_FLAG_CLOBBER_INPUT) | DFT3D_FLAG_COMPLEX128;
        }
        const int np = run_case(c);
        if (np < 0) ++refused;
        else ++ran;
    }
    printf("sweep: %d plans run, %d combinations refused, %ld checks, %d failed\n", ran, refused, g_checked, g_failed);

    // ---- seeded sweep over FFT plans with long axes: fused kernels, butterfly first stages, the z re-ordering
    // read by the next pass, explicit splits, CLOBBER_INPUT's odd pass count
    {
        const int64_t lpool[] = {1, 2, 16, 48, 256, 512, 1024, 2048, 4096, 8192};
        const int64_t spool[] = {0, 0, 0, 2, 4, 8, 16, 32};
        int lran = 0;
        for (int it = 0; it < 70; ++it) {
            Case c{};
            for (int j = 0; j < 3; ++j) c.n[j] = lpool[rng() % 10];
            if (c.n[0] * c.n[1] * c.n[2] > (int64_t)1 << 33 || c.n[1] * c.n[2] >= (int64_t)1 << 31) continue;
            c.form = DFT3D_FFT;
            if (rng() % 100 < 35) c.flags |= DFT3D_FLAG_CLOBBER_INPUT;
            else if (rng() % 100 < 10) c.flags |= DFT3D_FLAG_UNFUSED;
            for (int j = 0; j < 3; ++j) {
                const int64_t a = spool[rng() % 8];
                c.split[j] = (a && c.n[j] % a == 0) ? a : 0;
            }
            if (run_case(c) >= 0) ++lran;
        }
        printf("long-axis sweep: %d plans run, %ld checks, %d failed\n", lran, g_checked, g_failed);
    }

    steps_case(64, 32, 128, 0);
    steps_case(36, 20, 48, 0);
    steps_case(512, 3, 48, 0);
    steps_case(2, 2048, 32, 0);
    steps_case(4, 8192, 16, 0);
    steps_case(64, 32, 128, DFT3D_FLAG_COMPLEX128);
    points_case(false);
    points_case(true);
    printf("steps and evaluation-point plans: %ld checks, %d failed\n", g_checked, g_failed);

    // ---- generator under the sanitizers: extreme coordinates and sizes
    {
        std::vector<float> re(64 * 64), im(64 * 64);
        std::vector<double> c(64);
        for (int i = 0; i < 64; ++i) c[i] = (i % 2 ? -1.0 : 1.0) * std::ldexp(1.0, i % 60);     // huge, negative, exact
        EXPECT(dft3d_generate_matrix(64, c.data(), DFT3D_FORWARD, re.data(), im.data()) == DFT3D_OK, "generate_matrix");
        for (int i = 0; i < 64 * 64; ++i) EXPECT(std::isfinite(re[i]) && std::isfinite(im[i]), "finite matrix entry");
        c[7] = NAN;
        EXPECT(dft3d_generate_matrix(64, c.data(), DFT3D_FORWARD, re.data(), im.data()) == DFT3D_ERR_INVALID_ARG, "NaN coordinate");
        EXPECT(dft3d_generate_twiddle(64, 64, DFT3D_BACKWARD, re.data(), im.data()) == DFT3D_OK, "twiddle");
    }
    EXPECT(hostsim_live_allocations() == baseline_allocs, "plans leaked %zu device allocations",
           hostsim_live_allocations() - baseline_allocs);
    printf("total: %ld checks, %d failed\n", g_checked, g_failed);
    return g_failed ? 1 : 0;
}
