"""The boundary is a C ABI: a plain C program that includes include/im2win.h, links
libim2win.so and calls the host-side entry points must compile and run (no GPU needed)."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

C_SOURCE = r"""
#include <stdio.h>
#include <string.h>
#include "im2win.h"

int main(void)
{
    int Ho = 0, Wo = 0;
    size_t ws = 0, col = 0;
    /* Table 2, Conv4: 224, 7x7, stride 2, no padding -> 109 */
    if (im2win_out_shape(224, 224, 7, 7, 2, 0, &Ho, &Wo) != IM2WIN_OK || Ho != 109 || Wo != 109) return 1;
    /* Fig. 1: three 3x3 channels, 2x2 filter: 36 im2win elements, 48 im2col elements */
    if (im2win_workspace_bytes(1, 3, 3, 3, 2, 2, 1, 0, &ws) != IM2WIN_OK || ws != 4 * 36) return 2;
    if (im2col_footprint_bytes(1, 3, 3, 3, 2, 2, 1, 0, &col) != IM2WIN_OK || col != 4 * 48) return 3;
    if (im2win_out_shape(4, 4, 5, 5, 1, 0, &Ho, &Wo) != IM2WIN_ERR_SHAPE) return 4;
    if (im2win_transform(NULL, NULL, 1, 1, 4, 4, 2, 2, 1, 0, NULL) != IM2WIN_ERR_NULL) return 5;
    if (conv2d_im2win_fwd_variant((const float *)16, (const float *)16, (float *)16, 1, 1, 4, 4, 1, 2, 2, 1, 0,
                                  IM2WIN_VARIANT_LAST + 1, NULL) != IM2WIN_ERR_UNSUPPORTED) return 6;
    if (strlen(im2win_status_str(IM2WIN_ERR_OVERFLOW)) == 0) return 7;
    printf("c abi ok\n");
    return 0;
}
"""


def test_c_program_links_and_runs(tmp_path):
    import paper_2306_14316_amd as im2win
    lib = im2win.lib_path()
    if not os.path.exists(lib):
        pytest.skip("library not built")
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_abi.c"
    src.write_text(C_SOURCE)
    exe = tmp_path / "use_abi"
    libdir = os.path.dirname(lib)
    cmd = [gcc, "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
           "-L", libdir, "-lim2win", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"]
    subprocess.run(cmd, check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True, timeout=120)
    assert "c abi ok" in out.stdout


# A plain C99 program that allocates device memory through the HIP runtime's C API, runs the two
# calls of the path on the tiny benchmark layer and checks the result against oracle values read
# from a text file (written beforehand by tests/golden/make_cfg1_expected.py, which calls only
# the oracle).  argv: input.bin filter.bin expected.txt output.bin
C_GPU_SOURCE = r"""
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include "im2win.h"

enum { N = 1, CI = 3, HI = 32, WI = 32, CO = 16, HF = 3, WF = 3, S = 1, PAD = 0 };

static float *read_floats(const char *path, size_t count)
{
    float *p = (float *)malloc(count * sizeof(float));
    FILE *f = fopen(path, "rb");
    if (!p || !f || fread(p, sizeof(float), count, f) != count) { fprintf(stderr, "cannot read %s\n", path); exit(20); }
    fclose(f);
    return p;
}

int main(int argc, char **argv)
{
    int Ho = 0, Wo = 0;
    size_t ws = 0;
    if (argc != 5) return 21;
    if (im2win_out_shape(HI, WI, HF, WF, S, PAD, &Ho, &Wo) != IM2WIN_OK || Ho != 30 || Wo != 30) return 1;
    if (im2win_workspace_bytes(N, CI, HI, WI, HF, WF, S, PAD, &ws) != IM2WIN_OK || ws != 34560) return 2;
    const size_t n_in = (size_t)N * CI * HI * WI, n_f = (size_t)CO * CI * HF * WF, n_out = (size_t)N * CO * Ho * Wo;
    float *in = read_floats(argv[1], n_in), *flt = read_floats(argv[2], n_f);
    float *out = (float *)malloc(n_out * sizeof(float));
    float *d_in, *d_f, *d_w, *d_o;
    hipStream_t st;
    if (hipMalloc((void **)&d_in, n_in * 4) || hipMalloc((void **)&d_f, n_f * 4) || hipMalloc((void **)&d_w, ws) ||
        hipMalloc((void **)&d_o, n_out * 4) || hipStreamCreate(&st)) return 3;
    if (hipMemcpy(d_in, in, n_in * 4, hipMemcpyHostToDevice) || hipMemcpy(d_f, flt, n_f * 4, hipMemcpyHostToDevice)) return 4;
    if (hipMemset(d_w, 0xff, ws) || hipMemset(d_o, 0xff, n_out * 4)) return 5;   /* NaN patterns */
    printf("launching from C\n"); fflush(stdout);
    if (im2win_transform(d_in, d_w, N, CI, HI, WI, HF, WF, S, PAD, st) != IM2WIN_OK) return 6;
    if (conv2d_im2win_fwd(d_w, d_f, d_o, N, CI, HI, WI, CO, HF, WF, S, PAD, st) != IM2WIN_OK) return 7;
    if (hipStreamSynchronize(st)) return 8;
    if (hipMemcpy(out, d_o, n_out * 4, hipMemcpyDeviceToHost)) return 9;

    FILE *e = fopen(argv[3], "r");
    if (!e) return 22;
    char line[256];
    long checked = 0;
    double worst = 0.0;
    while (fgets(line, sizeof line, e)) {
        long idx; double want, bound;
        if (line[0] == '#') continue;
        if (sscanf(line, "%ld %la %la", &idx, &want, &bound) != 3 || idx < 0 || (size_t)idx >= n_out) return 23;
        const double err = fabs((double)out[idx] - want);
        if (!(err <= 1e-4 * bound)) { fprintf(stderr, "output %ld: got %g want %g\n", idx, out[idx], want); return 10; }
        if (bound > 0 && err / bound > worst) worst = err / bound;
        ++checked;
    }
    fclose(e);
    if (checked < 1000) return 24;
    FILE *o = fopen(argv[4], "wb");
    if (!o || fwrite(out, sizeof(float), n_out, o) != n_out) return 25;
    fclose(o);
    hipFree(d_in); hipFree(d_f); hipFree(d_w); hipFree(d_o); hipStreamDestroy(st);
    printf("c gpu ok: %ld outputs checked, max |err|/sum|x||w| = %.3e\n", checked, worst);
    return 0;
}
"""


@pytest.mark.gpu
def test_c_program_runs_the_path_on_the_gpu(tmp_path):
    """The whole path driven from C, no Python between the caller and the library: device buffers
    from hipMalloc, a stream from hipStreamCreate, results against stored oracle values (and, back
    in Python, every output element against the oracle)."""
    import numpy as np

    import oracle
    import paper_2306_14316_amd as im2win
    from paper_2306_14316_amd import workloads
    from parity_util import assert_conv_close

    lib = im2win.lib_path()
    assert os.path.exists(lib), "library not built"
    gcc = shutil.which("gcc")
    assert gcc is not None
    L = workloads.layer(1)
    I, F = workloads.make_inputs(L)
    I.numpy().tofile(tmp_path / "input.bin")
    F.numpy().tofile(tmp_path / "filter.bin")
    src = tmp_path / "run_path.c"
    src.write_text(C_GPU_SOURCE)
    exe = tmp_path / "run_path"
    libdir = os.path.dirname(lib)
    cmd = [gcc, "-std=c99", "-Wall", "-Werror", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
           "-I", "/opt/rocm/include", str(src), "-o", str(exe), "-L", libdir, "-lim2win", "-L", "/opt/rocm/lib",
           "-lamdhip64", "-lm", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"]
    subprocess.run(cmd, check=True)
    print("running the C program", flush=True)
    out = subprocess.run([str(exe), str(tmp_path / "input.bin"), str(tmp_path / "filter.bin"),
                          os.path.join(ROOT, "tests", "golden", "cfg1_expected_samples.txt"),
                          str(tmp_path / "output.bin")], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, (out.returncode, out.stdout, out.stderr)
    assert "c gpu ok" in out.stdout
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), L.stride, L.pad)
    got = np.fromfile(tmp_path / "output.bin", dtype=np.float32).reshape(O_ref.shape)
    assert_conv_close(got, O_ref, B_ref)
