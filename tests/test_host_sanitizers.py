"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU.

Every source of libdft3d is compiled host-only (no device code, seconds per file) with
-fsanitize=address,undefined and linked with a stand-in for the HIP runtime (tests/hostsim/): device
memory is host memory with a registry, a launch records its kernel and checks that the tensors it
describes lie inside live allocations.  The driver then creates plans for the named configurations and
a seeded sweep of shapes, formulations and flags, and checks for every exec the order of the passes,
the buffers they read and write (ping-pong between out and workspace, or in with CLOBBER_INPUT), the
launch shapes, the LDS sizes, and that destroying a plan frees everything.  The C oracle gets the
same sanitizers on a small transform."""
import os
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOSTSIM = os.path.join(ROOT, "tests", "hostsim")
CSRC = os.path.join(ROOT, "paper_2002_03260_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert res.returncode == 0, f"{' '.join(cmd)}\n{res.stdout[-4000:]}\n{res.stderr[-4000:]}"
    return res


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_host_code_under_asan_and_ubsan(tmp_path):
    from paper_2002_03260_amd import build

    objs = []
    procs = []
    common = [HIPCC, "--offload-arch=gfx950", "--cuda-host-only", "-O1", "-g", "-std=c++17", "-Wno-unused-command-line-argument",
              "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-I" + HOSTSIM] + SAN
    sources = [os.path.join(CSRC, s) for s in build.SOURCES] + [os.path.join(HOSTSIM, "fake_hip_runtime.cpp"),
                                                                 os.path.join(HOSTSIM, "driver.cpp")]
    for src in sources:
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        objs.append(obj)
        procs.append((src, subprocess.Popen(common + ["-x", "hip", "-c", src, "-o", obj], stdout=subprocess.PIPE,
                                            stderr=subprocess.STDOUT, text=True)))
    for src, pr in procs:
        out, _ = pr.communicate()
        assert pr.returncode == 0, f"compiling {src}:\n{out[-4000:]}"
    # the host-only objects refer to the device code they would embed: give those symbols a body
    syms = set()
    for obj in objs:
        for line in _run(["nm", "-u", obj]).stdout.splitlines():
            name = line.split()[-1]
            if name.startswith("__hip_fatbin"):
                syms.add(name)
    fat = tmp_path / "fatbin_stubs.c"
    fat.write_text("".join(f"const char {s}[8] = {{0}};\n" for s in sorted(syms)))
    exe = str(tmp_path / "hostsim_driver")
    _run([HIPCC, "--cuda-host-only", "-x", "c", str(fat), "-x", "none"] + objs + SAN + ["-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    sys.stdout.write(res.stdout[-3000:])
    assert res.returncode == 0, f"driver failed:\n{res.stdout[-6000:]}\n{res.stderr[-6000:]}"
    assert "0 failed" in res.stdout.splitlines()[-1]
    assert "ERROR: AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr, res.stderr[-4000:]
    # the checker must itself be able to fail: with output tensors registered one element short, every
    # last pass writes outside its allocation and the stand-in runtime has to say so
    bad = subprocess.run([exe], capture_output=True, text=True, env=dict(env, HOSTSIM_SHORT_OUTPUT="1"), timeout=600)
    assert bad.returncode == 1
    assert "output region" in bad.stdout and "is not inside a live allocation" in bad.stdout


def test_c_oracle_under_asan_and_ubsan(tmp_path):
    """oracle/dft3d_oracle.c with the same sanitizers: a small transform, the brute-force sum and the
    sampled forms, called from a C driver (values are compared with the regular build elsewhere)."""
    src = os.path.join(ROOT, "oracle", "dft3d_oracle.c")
    drv = tmp_path / "oracle_driver.c"
    drv.write_text(r'''
#include <complex.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
int oracle_dft3d(int64_t, int64_t, int64_t, const void*, void*, const double*, const double*, const double*, int, int);
void oracle_dft3d_brute(int64_t, int64_t, int64_t, const void*, void*, const double*, const double*, const double*, int);
void oracle_mode_contract(int64_t, int64_t, int64_t, int64_t, const void*, const void*, void*);
void oracle_dft_matrix(int64_t, int64_t, const int64_t*, const double*, int, void*);
int main(void) {
    const int64_t n1 = 3, n2 = 5, n3 = 4, E = n1 * n2 * n3;
    float* x = malloc(sizeof(float) * 2 * E);
    double *a = malloc(sizeof(double) * 2 * E), *b = malloc(sizeof(double) * 2 * E);
    double c2[5] = {0.01, 0.2, 0.35, 0.6, 0.93};
    for (int64_t i = 0; i < 2 * E; ++i) x[i] = (float)sin(0.37 * (double)i + 0.1);
    for (int pass = 0; pass < 2; ++pass) {
        const double* cy = pass ? c2 : NULL;
        if (oracle_dft3d(n1, n2, n3, x, a, NULL, cy, NULL, -1, 0)) return 2;
        oracle_dft3d_brute(n1, n2, n3, x, b, NULL, cy, NULL, -1);
        double num = 0, den = 0;
        for (int64_t i = 0; i < 2 * E; ++i) { num += (a[i] - b[i]) * (a[i] - b[i]); den += b[i] * b[i]; }
        printf("pass %d rel %.3e\n", pass, sqrt(num / den));
        if (!(sqrt(num / den) < 1e-13)) return 1;
    }
    /* a rectangular mode product with selected rows */
    int64_t ks[2] = {0, 3};
    double* M = malloc(sizeof(double) * 2 * 2 * n3);
    oracle_dft_matrix(2, n3, ks, NULL, -1, M);
    double* y = malloc(sizeof(double) * 2 * n1 * n2 * 2);
    double* xd = malloc(sizeof(double) * 2 * E);
    for (int64_t i = 0; i < 2 * E; ++i) xd[i] = x[i];
    oracle_mode_contract(n1 * n2, n3, 1, 2, M, xd, y);
    free(x); free(a); free(b); free(M); free(y); free(xd);
    return 0;
}
''')
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
          "-static-libasan", src, str(drv), "-o", exe, "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", OMP_NUM_THREADS="2")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-3000:]
