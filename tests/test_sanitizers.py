"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, no GPU needed).

Two executables are built here and run:
  * the C oracle, compiled together with a small C driver that runs every oracle routine over a
    sweep of tiny shapes (padding, strides, asymmetric filters, a filter as large as the padded
    input) and checks the routes against each other -- any out-of-bounds index, signed overflow
    or misaligned access in the oracle aborts the run;
  * the host side of the GPU library (argument validation, shape derivation, kernel and grid
    selection), compiled host-only with an empty device-code bundle, driven through the planning
    calls and the argument checks with ordinary and extreme shapes (dimensions, strides and
    paddings up to INT_MAX).  No kernel is launched.
"""
import os
import shutil
import struct
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")

ORACLE_DRIVER = r"""
#include "im2win_oracle.c"
#include <stdio.h>

static unsigned long long rng = 88172645463325252ull;
static float rnd(void)
{
    rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17;
    return (float)((double)(rng >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}

static int check(int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf, int s, int p)
{
    int Ho = oracle_out_dim(Hi, Hf, s, p), Wo = oracle_out_dim(Wi, Wf, s, p);
    if (Ho < 1 || Wo < 1) return 1;
    size_t n_in = (size_t)N * Ci * Hi * Wi, n_f = (size_t)Co * Ci * Hf * Wf, n_o = (size_t)N * Co * Ho * Wo;
    int64_t n_w = oracle_im2win_elems(N, Ci, Hi, Wi, Hf, Wf, s, p);
    if (n_w != (int64_t)N * Ci * Ho * (Wi + 2 * p) * Hf) return 2;
    if (oracle_im2col_elems(N, Ci, Hi, Wi, Hf, Wf, s, p) != (int64_t)N * Ho * Wo * Ci * Hf * Wf) return 3;
    float *I = malloc(n_in * 4), *F = malloc(n_f * 4), *W = malloc((size_t)n_w * 4);
    double *O = malloc(n_o * 8), *B = malloc(n_o * 8), *O2 = malloc(n_o * 8), *O3 = malloc(n_o * 8);
    for (size_t k = 0; k < n_in; ++k) I[k] = rnd();
    for (size_t k = 0; k < n_f; ++k) F[k] = rnd();
    int rc = 0;
    if (oracle_conv2d_direct(I, F, N, Ci, Hi, Wi, Co, Hf, Wf, s, p, O, B)) rc = 4;
    if (!rc && oracle_im2win(I, W, N, Ci, Hi, Wi, Hf, Wf, s, p)) rc = 5;
    if (!rc && oracle_conv2d_im2col_gemm(I, F, N, Ci, Hi, Wi, Co, Hf, Wf, s, p, O2)) rc = 6;
    if (!rc && oracle_conv2d_over_im2win(W, F, N, Ci, Hi, Wi, Co, Hf, Wf, s, p, O3)) rc = 7;
    for (size_t k = 0; !rc && k < n_o; ++k) {
        if (fabs(O[k] - O2[k]) > 1e-12 || fabs(O[k] - O3[k]) > 1e-12 || fabs(O[k]) > B[k] + 1e-12) rc = 8;
    }
    /* the sampled form equals the full pass, at the four corners of the output */
    int32_t idx[16] = {0, 0, 0, 0,  N - 1, Co - 1, Ho - 1, Wo - 1,  0, Co - 1, 0, Wo - 1,  N - 1, 0, Ho - 1, 0};
    double Os[4], Bs[4];
    if (!rc && oracle_conv2d_direct_at(I, F, N, Ci, Hi, Wi, Co, Hf, Wf, s, p, idx, 4, Os, Bs)) rc = 9;
    for (int q = 0; !rc && q < 4; ++q) {
        size_t o = (((size_t)idx[4 * q] * Co + idx[4 * q + 1]) * Ho + idx[4 * q + 2]) * Wo + idx[4 * q + 3];
        if (Os[q] != O[o] || Bs[q] != B[o]) rc = 10;
    }
    int32_t bad[4] = {N, 0, 0, 0};
    if (!rc && oracle_conv2d_direct_at(I, F, N, Ci, Hi, Wi, Co, Hf, Wf, s, p, bad, 1, Os, Bs) != -2) rc = 11;
    free(I); free(F); free(W); free(O); free(B); free(O2); free(O3);
    return rc;
}

int main(void)
{
    static const int shapes[][9] = {
        {1, 3, 3, 3, 2, 2, 2, 1, 0}, {2, 3, 7, 9, 4, 3, 2, 1, 0}, {2, 3, 9, 7, 5, 2, 3, 2, 1},
        {1, 2, 11, 13, 3, 5, 3, 3, 3}, {3, 4, 12, 10, 2, 4, 1, 4, 0}, {1, 5, 6, 8, 3, 6, 2, 1, 0},
        {2, 2, 6, 6, 3, 8, 8, 1, 1}, {1, 3, 10, 10, 6, 1, 1, 2, 0}, {1, 1, 5, 5, 1, 3, 3, 1, 0},
        {1, 2, 5, 4, 2, 3, 3, 1000000, 0}, {1, 1, 9, 9, 2, 7, 7, 2, 3}, {2, 1, 4, 12, 1, 2, 11, 4, 0},
    };
    for (unsigned k = 0; k < sizeof shapes / sizeof shapes[0]; ++k) {
        const int *q = shapes[k];
        int rc = check(q[0], q[1], q[2], q[3], q[4], q[5], q[6], q[7], q[8]);
        if (rc) { fprintf(stderr, "shape %u failed: %d\n", k, rc); return 1; }
    }
    if (oracle_out_dim(224, 7, 2, 0) != 109 || oracle_out_dim(4, 5, 1, 0) != -1 || oracle_out_dim(4, 2, 0, 0) != -1) return 2;
    printf("oracle sanitizer run ok\n");
    return 0;
}
"""

HOST_DRIVER = r"""
#include "im2win.h"
#include "im2win_probe.h"
#include <limits.h>
#include <stdio.h>
#include <string.h>

static int known(int rc) { return rc <= 0 && rc >= -5; }

int main()
{
    static const int vals[] = {1, 2, 3, 7, 8, 11, 64, 227, 1 << 16, 1 << 26, INT_MAX};
    const int nv = (int)(sizeof vals / sizeof vals[0]);
    im2win_launch_info info;
    long planned = 0, rejected = 0;
    /* every combination of a few ordinary and extreme values for the image, filter, stride and padding */
    for (int a = 0; a < nv; ++a) for (int b = 0; b < nv; ++b) for (int c = 0; c < 6; ++c) for (int d = 0; d < 6; ++d)
    for (int e = 0; e < nv; ++e) for (int f = 0; f < 4; ++f) {
        const int Hi = vals[a], Wi = vals[b], Hf = vals[c], Wf = vals[d], s = vals[e], p = f == 3 ? INT_MAX : f;
        for (int ci = 1; ci <= 64; ci *= 8) {
            int Ho, Wo; size_t ws, col;
            int r1 = im2win_out_shape(Hi, Wi, Hf, Wf, s, p, &Ho, &Wo);
            int r2 = im2win_workspace_bytes(3, ci, Hi, Wi, Hf, Wf, s, p, &ws);
            int r3 = im2col_footprint_bytes(3, ci, Hi, Wi, Hf, Wf, s, p, &col);
            int r4 = im2win_transform_launch_info(3, ci, Hi, Wi, Hf, Wf, s, p, &info);
            if (!known(r1) || !known(r2) || !known(r3) || !known(r4)) return 1;
            if (r4 == IM2WIN_OK && (info.grid_x < 1 || info.block < 64 || info.lds_bytes > 160 * 1024 || !info.kernel[0])) return 2;
            for (int wf = 0; wf < 2; ++wf) {
                int r5 = conv2d_im2win_fwd_launch_info(3, ci, Hi, Wi, 70, Hf, Wf, s, p, 0, wf, &info);
                if (!known(r5)) return 3;
                if (r5 == IM2WIN_OK) {
                    ++planned;
                    if (info.grid_x < 1 || info.grid_y < 1 || info.block < 64 || info.block > 1024 ||
                        info.lds_bytes > 160 * 1024 || !memchr(info.kernel, 0, sizeof info.kernel) || !info.kernel[0]) return 4;
                } else ++rejected;
            }
        }
    }
    /* the benchmark layers and every variant */
    static const int layers[][9] = {{1, 3, 32, 32, 16, 3, 3, 1, 0}, {32, 64, 56, 56, 64, 3, 3, 1, 1},
        {128, 256, 14, 14, 256, 3, 3, 1, 1}, {128, 3, 224, 224, 64, 7, 7, 2, 3}, {128, 3, 227, 227, 96, 11, 11, 4, 0},
        {128, 64, 224, 224, 64, 7, 7, 2, 0}, {128, 96, 24, 24, 256, 5, 5, 1, 0}, {128, 60, 56, 56, 64, 3, 3, 1, 1}};
    for (unsigned k = 0; k < sizeof layers / sizeof layers[0]; ++k) {
        const int *q = layers[k];
        for (int v = 0; v <= IM2WIN_VARIANT_LAST; ++v)
            if (conv2d_im2win_fwd_launch_info(q[0], q[1], q[2], q[3], q[4], q[5], q[6], q[7], q[8], v, 0, &info) != IM2WIN_OK) return 5;
        if (conv2d_im2win_fwd_launch_info(q[0], q[1], q[2], q[3], q[4], q[5], q[6], q[7], q[8], 0, 1, &info) != IM2WIN_OK) return 6;
    }
    /* argument checks of the launching calls (all fail before any launch) */
    float *one = (float *)16;
    if (im2win_transform(0, one, 1, 1, 4, 4, 2, 2, 1, 0, 0) != IM2WIN_ERR_NULL) return 7;
    if (conv2d_im2win_fwd(one, one, one, 1, 1, 4, 4, 1, 5, 5, 1, 0, 0) != IM2WIN_ERR_SHAPE) return 8;
    if (conv2d_im2win_fwd(one, one, one, 128, 3, 1024, 1024, 64, 1, 1, 1, 0, 0) != IM2WIN_ERR_OVERFLOW) return 9;
    if (conv2d_im2col_fwd(one, one, one, 512, 256, 112, 112, 8, 3, 3, 1, 1, 0) != IM2WIN_ERR_OVERFLOW) return 10;
    if (im2win_probe_stream(0, one, one, 1000, 0) != IM2WIN_ERR_SHAPE) return 11;
    if (!im2win_status_str(IM2WIN_ERR_HIP)[0] || !im2win_status_str(IM2WIN_OK)[0]) return 12;
    printf("host sanitizer run ok: %ld plans, %ld rejections\n", planned, rejected);
    return planned > 100 && rejected > 100 ? 0 : 13;
}
"""


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, "%s\n%s\n%s" % (" ".join(map(str, cmd)), r.stdout[-3000:], r.stderr[-6000:])
    return r


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "oracle_driver.c"
    src.write_text(ORACLE_DRIVER)
    exe = tmp_path / "oracle_driver"
    _run([gcc, "-std=c11", "-Wall", "-Wextra", "-fopenmp", *SAN, "-static-libasan", "-I", os.path.join(ROOT, "oracle"),
          str(src), "-o", str(exe), "-lm"])
    out = _run([str(exe)], env=dict(ENV, OMP_NUM_THREADS="2"), timeout=300)
    assert "oracle sanitizer run ok" in out.stdout


def test_library_host_side_under_sanitizers(tmp_path):
    from paper_2306_14316_amd import build
    hipcc = build._hipcc()
    if shutil.which(hipcc) is None and not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    # host-only compilation: the device side of every source is replaced by an empty code-object bundle
    bundle = tmp_path / "empty.hipfb"
    bundle.write_bytes(b"__CLANG_OFFLOAD_BUNDLE__" + struct.pack("<Q", 0))
    objs = []
    procs = []
    for name in build.SOURCES:
        obj = tmp_path / (os.path.splitext(name)[0] + ".o")
        objs.append(str(obj))
        procs.append(subprocess.Popen(
            [hipcc, "--offload-arch=gfx950", "-std=c++17", "--offload-host-only", "-Xclang", "-fcuda-include-gpubinary",
             "-Xclang", str(bundle), *SAN, "-c", os.path.join(build.CSRC, name), "-o", str(obj)],
            stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True))
    for pr in procs:
        _, err = pr.communicate(timeout=600)
        assert pr.returncode == 0, err[-4000:]
    src = tmp_path / "host_driver.cpp"
    src.write_text(HOST_DRIVER)
    exe = tmp_path / "host_driver"
    _run([hipcc, "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"), "-x", "c++", str(src), "-x", "none", *objs,
          "-o", str(exe)])
    out = _run([str(exe)], env=ENV, timeout=600)
    assert "host sanitizer run ok" in out.stdout
