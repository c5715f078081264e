"""The GPU-free part of the library (layout, trees, schedule, validation) and the C oracle,
built with AddressSanitizer + UBSan on the host and run on small drivers.  GPU code is not
sanitised (not available for device code here)."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1711_00705_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def _run(cmd, **kw):
    return subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"),
                    reason="needs hipcc")
def test_host_side_of_the_library_under_asan_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    exe = str(tmp_path / "host_driver")
    srcs = [os.path.join(ROOT, "tests", "host_driver", "host_driver.cpp")]
    srcs += [os.path.join(CSRC, f) for f in
             ("mc_layout.cpp", "mc_trees.cpp", "mc_pack.hip", "mc_reduce_update.hip", "mc_fused.hip",
              "mc_schedule.hip", "mc_copy.hip")]
    san_host = []
    for flag in SAN[:2]:
        san_host += ["-Xarch_host", flag]
    cmd = [hipcc, "--offload-arch=gfx950", "-std=c++17", "-O1", "-g", "-ffp-contract=off",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           *san_host, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", exe, *srcs]
    res = _run(cmd)
    if res.returncode != 0 and "sanitize" in res.stderr and "unsupported" in res.stderr:
        pytest.skip("host sanitizers not available in this toolchain")
    assert res.returncode == 0, res.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:protect_shadow_gap=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = _run([exe], env=env)
    assert run.returncode == 0, (run.stdout + run.stderr)[-3000:]
    assert "host_driver: ok" in run.stdout
    assert "ERROR: AddressSanitizer" not in run.stderr and "runtime error" not in run.stderr


def test_oracle_under_asan_ubsan(tmp_path):
    """The plain C oracle with sanitizers, driven through a few ragged shapes."""
    drv = tmp_path / "drv.c"
    drv.write_text(r'''
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
int mco_layout(const int64_t*, int32_t, int32_t, int64_t*, int64_t*);
void mco_pack(const int64_t*, int32_t, const uint32_t* const*, uint32_t*);
void mco_unpack(const int64_t*, int32_t, const uint32_t*, uint32_t* const*);
int mco_reduce_update(const int64_t*, int32_t, const float* const*, int32_t, const int32_t*, float*, float*, float*, float, float, float);
int mco_reduce_update_roles(const int64_t*, int32_t, const float* const*, int32_t, const int32_t*, const int32_t*, const uint8_t*, float*, float*, float*, float, float, float);
int main(void) {
    int64_t numel[4] = {257, 0, 3, 1000};
    for (int32_t k = 1; k <= 1300; k += 433) {
        int64_t off[5];
        int64_t* b = malloc(sizeof(int64_t) * (k + 1));
        if (mco_layout(numel, 4, k, off, b) != 0) return 1;
        int64_t N = off[4];
        uint32_t* t[4];
        for (int i = 0; i < 4; ++i) { t[i] = malloc(4 * (numel[i] ? numel[i] : 1)); for (int64_t j = 0; j < numel[i]; ++j) t[i][j] = 0x3f800000u + (uint32_t)j; }
        float* x[3]; for (int p = 0; p < 3; ++p) { x[p] = malloc(4 * N); mco_pack(off, 4, (const uint32_t* const*)t, (uint32_t*)x[p]); }
        float* g = malloc(4 * N); float* w = calloc(N, 4); float* v = calloc(N, 4);
        int32_t* order = malloc(sizeof(int32_t) * 3 * k); int32_t* nt = malloc(sizeof(int32_t) * k); uint8_t* du = malloc(k);
        for (int32_t c = 0; c < k; ++c) { for (int q = 0; q < 3; ++q) order[c * 3 + q] = (c + q) % 3; nt[c] = c % 4 == 3 ? 0 : 1 + c % 3; du[c] = c & 1; }
        if (mco_reduce_update(b, k, (const float* const*)x, 3, order, g, w, v, 0.1f, 0.9f, 1e-4f) != 0) return 2;
        if (mco_reduce_update_roles(b, k, (const float* const*)x, 3, order, nt, du, g, w, v, 0.1f, 0.9f, 1e-4f) != 0) return 3;
        mco_unpack(off, 4, (const uint32_t*)w, (uint32_t* const*)t);
        for (int i = 0; i < 4; ++i) free(t[i]);
        for (int p = 0; p < 3; ++p) free(x[p]);
        free(g); free(w); free(v); free(order); free(nt); free(du); free(b);
    }
    puts("oracle driver: ok");
    return 0;
}
''')
    exe = str(tmp_path / "drv")
    res = _run(["gcc", "-std=c11", *SAN, "-ffp-contract=off", "-o", exe, str(drv),
                os.path.join(ROOT, "oracle", "mc_oracle.c")])
    if res.returncode != 0 and ("asan" in res.stderr.lower() or "ubsan" in res.stderr.lower()):
        pytest.skip("gcc sanitizer runtimes not installed")
    assert res.returncode == 0, res.stderr[-3000:]
    run = _run([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1", UBSAN_OPTIONS="halt_on_error=1"))
    assert run.returncode == 0 and "oracle driver: ok" in run.stdout, (run.stdout + run.stderr)[-3000:]
