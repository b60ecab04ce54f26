"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, derives shapes as the oracle does, and turns every invalid
argument into an error code without launching anything."""
import ctypes
import os
import re

import pytest

import oracle
import paper_2306_14316_amd as im2win
from paper_2306_14316_amd import binding, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(im2win.lib_path()):
        from paper_2306_14316_amd import build
        build.build()
    return im2win.load_library()


def test_header_symbols_are_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "im2win.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(im2win_\w+|conv2d_\w+|im2col_\w+)\s*\(", hdr))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    probes = open(os.path.join(ROOT, "include", "im2win_probe.h")).read()
    probes = re.sub(r"/\*.*?\*/", "", probes, flags=re.S)
    declared = set(re.findall(r"\b(im2win_\w+)\s*\(", probes))
    assert declared == set(binding.PROBE_EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_shapes_and_footprints_match_oracle(lib, golden_dir):
    for L in workloads.LAYERS:
        assert im2win.im2win_out_shape(L.Hi, L.Wi, L.Hf, L.Wf, L.stride, L.pad) == \
            oracle.out_shape(L.Hi, L.Wi, L.Hf, L.Wf, L.stride, L.pad)
        a = (L.N, L.Ci, L.Hi, L.Wi, L.Hf, L.Wf, L.stride, L.pad)
        assert im2win.im2win_workspace_bytes(*a) == 4 * oracle.im2win_elems(*a)
        assert im2win.im2col_footprint_bytes(*a) == 4 * oracle.im2col_elems(*a)
    # the paper's worked example and Table 2
    assert im2win.im2win_workspace_bytes(1, 3, 3, 3, 2, 2, 1, 0) == 4 * 36
    assert im2win.im2col_footprint_bytes(1, 3, 3, 3, 2, 2, 1, 0) == 4 * 48
    for ln in open(os.path.join(golden_dir, "table2_layers.txt")):
        if ln.startswith("#") or not ln.strip():
            continue
        _, Ci, Hi, Wi, Co, Hf, Wf, s, Ho, Wo = ln.split()
        assert im2win.im2win_out_shape(int(Hi), int(Wi), int(Hf), int(Wf), int(s), 0) == (int(Ho), int(Wo))


def test_workspace_bytes_of_the_five_layers(lib):
    want = [34560, 79822848, 88080384, 276971520, 210946560]
    got = [im2win.im2win_workspace_bytes(L.N, L.Ci, L.Hi, L.Wi, L.Hf, L.Wf, L.stride, L.pad)
           for L in workloads.LAYERS]
    assert got == want


BAD_SHAPES = [
    dict(N=0), dict(Ci=0), dict(Hi=0), dict(Wi=-1), dict(Co=0), dict(Hf=0), dict(Wf=0),
    dict(stride=0), dict(pad=-1), dict(Hf=9), dict(Wf=9),
]


@pytest.mark.parametrize("bad", BAD_SHAPES)
def test_invalid_shapes_are_rejected_before_any_launch(lib, bad):
    a = dict(N=1, Ci=2, Hi=8, Wi=8, Co=3, Hf=3, Wf=3, stride=1, pad=0)
    a.update(bad)
    one = ctypes.c_void_p(16)   # non-NULL dummy: validation must fail before it is touched
    rc = lib.im2win_transform(one, one, a["N"], a["Ci"], a["Hi"], a["Wi"], a["Hf"], a["Wf"],
                              a["stride"], a["pad"], None)
    if "Co" not in bad:
        assert rc == -2
    for fn in (lib.conv2d_im2win_fwd, lib.conv2d_im2win_fwd_basic):
        assert fn(one, one, one, a["N"], a["Ci"], a["Hi"], a["Wi"], a["Co"], a["Hf"], a["Wf"],
                  a["stride"], a["pad"], None) == -2
    assert lib.conv2d_im2win_fwd_variant(one, one, one, a["N"], a["Ci"], a["Hi"], a["Wi"], a["Co"], a["Hf"],
                                         a["Wf"], a["stride"], a["pad"], 1, None) == -2


def test_null_pointers_and_overflow(lib):
    one = ctypes.c_void_p(16)
    assert lib.im2win_transform(None, one, 1, 1, 4, 4, 2, 2, 1, 0, None) == -1
    assert lib.im2win_transform(one, None, 1, 1, 4, 4, 2, 2, 1, 0, None) == -1
    assert lib.conv2d_im2win_fwd(one, None, one, 1, 1, 4, 4, 1, 2, 2, 1, 0, None) == -1
    assert lib.conv2d_im2win_fwd(one, one, None, 1, 1, 4, 4, 1, 2, 2, 1, 0, None) == -1
    assert lib.conv2d_im2win_fwd_basic(None, one, one, 1, 1, 4, 4, 1, 2, 2, 1, 0, None) == -1
    assert lib.im2win_out_shape(4, 4, 2, 2, 1, 0, None, None) == -1
    assert lib.conv2d_im2win_fwd_variant(one, one, None, 1, 1, 4, 4, 1, 2, 2, 1, 0, 0, None) == -1
    assert lib.conv2d_im2win_fwd_variant(one, one, one, 1, 1, 4, 4, 1, 2, 2, 1, 0, 7, None) == -4
    assert lib.conv2d_im2win_fwd_variant(one, one, one, 1, 1, 4, 4, 1, 2, 2, 1, 0, -1, None) == -4
    # 2^31 or more elements in the im2win tensor / the output
    assert lib.im2win_transform(one, one, 4096, 64, 224, 224, 7, 7, 2, 0, None) == -3
    assert lib.conv2d_im2win_fwd(one, one, one, 128, 3, 1024, 1024, 64, 1, 1, 1, 0, None) == -3
    # the baselines: NULL pointers, and an im2col matrix of 2^31 or more groups of four floats
    assert lib.conv2d_direct_fwd(one, None, one, 1, 1, 4, 4, 1, 2, 2, 1, 0, None) == -1
    assert lib.conv2d_im2win_implicit_fwd(None, one, one, 1, 8, 4, 4, 1, 3, 3, 1, 0, None) == -1
    assert lib.im2col_transform(one, None, 1, 1, 4, 4, 2, 2, 1, 0, None) == -1
    assert lib.conv2d_im2col_fwd(None, one, one, 1, 1, 4, 4, 1, 2, 2, 1, 0, None) == -1
    assert lib.im2col_transform(one, one, 512, 256, 112, 112, 3, 3, 1, 1, None) == -3
    assert lib.conv2d_im2col_fwd(one, one, one, 512, 256, 112, 112, 8, 3, 3, 1, 1, None) == -3
    b = ctypes.c_size_t()
    assert lib.im2win_workspace_bytes(4096, 64, 224, 224, 7, 7, 2, 0, ctypes.byref(b)) == -3
    for code in (0, -1, -2, -3, -4, -5, 77):
        assert im2win.status_str(code)


def test_filter_as_large_as_padded_input_is_valid(lib):
    assert im2win.im2win_out_shape(6, 6, 8, 8, 1, 1) == (1, 1)
    with pytest.raises(im2win.Im2winError):
        im2win.im2win_out_shape(6, 6, 9, 8, 1, 1)


def test_binding_rejects_host_tensors(lib):
    import torch
    x = torch.zeros(1, 1, 4, 4)
    w = torch.zeros(1, 1, 3, 8)
    with pytest.raises(TypeError):
        im2win.im2win_transform(x, w, 1, 1, 4, 4, 2, 2, 1, 0)


def test_launch_info_names_the_dispatch(lib):
    """The planning calls run the library's own dispatch and launch nothing (no GPU needed: the
    grid is then planned for 256 compute units)."""
    want = {1: "conv_mfma_kernel<9, false>", 2: "conv_mfma_fast_kernel<3, 3, 8,", 3: "conv_mfma_fast_kernel<3, 3, 8,",
            4: "conv_mfma_shallow_kernel<7, 7, 3,", 5: "conv_mfma_shallow_kernel<11, 11, 3,"}
    for idx, prefix in want.items():
        L = workloads.layer(idx)
        info = im2win.conv2d_im2win_fwd_launch_info(*L.dims)
        assert info["kernel"].startswith(prefix), info
        assert info["grid"][0] >= 1 and info["block"] in (256, 512, 768)
        t = im2win.im2win_transform_launch_info(L.N, L.Ci, L.Hi, L.Wi, L.Hf, L.Wf, L.stride, L.pad)
        assert t["kernel"].startswith("transform_assemble_kernel<%d, %d, " % (L.Hf, L.stride)), t
        assert t["kernel"].endswith("true>" if idx in (1, 3) else "false>"), t   # small planes go in groups
    assert im2win.im2win_transform_launch_info(1, 1, 12, 1100, 9, 1, 1, 1)["kernel"] == "transform_kernel<4>"
    assert im2win.im2win_transform_launch_info(1, 1, 4, 3, 2, 2, 1, 0)["kernel"] == "transform_kernel<4>"
    for L in workloads.TABLE2:
        t = im2win.im2win_transform_launch_info(L.N, L.Ci, L.Hi, L.Wi, L.Hf, L.Wf, L.stride, L.pad)
        assert t["kernel"].startswith("transform_assemble_kernel<") and t["lds_bytes"] <= 24 * 1024 + 32, t
    L = workloads.layer(2)
    assert im2win.conv2d_im2win_fwd_launch_info(*L.dims, variant=im2win.VARIANT_NO_MFMA)["kernel"] == "conv_basic_kernel"
    assert im2win.conv2d_im2win_fwd_launch_info(*L.dims, variant=im2win.VARIANT_NO_PIPELINE)["kernel"] == "conv_mfma_kernel<9, false>"
    assert im2win.conv2d_im2win_fwd_launch_info(*L.dims, variant=im2win.VARIANT_VALU_MICROKERNEL)["kernel"] == "conv_mfma_kernel<9, true>"
    for v, cw in ((im2win.VARIANT_DEFAULT, 4), (im2win.VARIANT_NARROW_LOADS, 2), (im2win.VARIANT_SCALAR_LOADS, 1)):
        assert im2win.conv2d_im2win_fwd_launch_info(*L.dims, variant=v)["kernel"].startswith(
            "conv_mfma_fast_kernel<3, 3, 8, 1, %d, 3," % cw)
    assert ", true, " in im2win.conv2d_im2win_fwd_launch_info(*L.dims, workspace_free=True)["kernel"]
    # a channel count off the K block still takes the pipelined kernel (its ragged instance)
    assert im2win.conv2d_im2win_fwd_launch_info(128, 60, 56, 56, 64, 3, 3, 1, 1)["kernel"] == \
        "conv_mfma_fast_kernel<3, 3, 8, 1, 4, 3, false, false, false, false, true>"
    assert im2win.conv2d_im2win_fwd_launch_info(8, 7, 56, 56, 64, 3, 3, 1, 1)["kernel"] == "conv_mfma_kernel<9, false>"
    # 1x1 layers: their own kernel; 1x7 / 7x1 / 1x3 / 3x1: instances of the pipelined kernel; other asymmetric filters:
    # the pipelined generic kernel, its single-stage form when two stages do not fit LDS
    assert im2win.conv2d_im2win_fwd_launch_info(64, 256, 28, 28, 256, 1, 1, 1, 0)["kernel"] == "conv_mfma_1x1_kernel<32, false, 2, 1>"
    assert im2win.conv2d_im2win_fwd_launch_info(64, 256, 28, 28, 256, 1, 1, 1, 0, workspace_free=True)["kernel"] == "conv_mfma_1x1_kernel<32, false, 2, 1>"
    assert im2win.conv2d_im2win_fwd_launch_info(64, 256, 28, 28, 256, 1, 1, 2, 0)["kernel"] == "conv_mfma_1x1_kernel<32, true, 2, 1>"   # strided
    assert im2win.conv2d_im2win_fwd_launch_info(64, 252, 28, 28, 256, 1, 1, 1, 0)["kernel"] == "conv_mfma_pipe_kernel<1, 1>"
    assert im2win.conv2d_im2win_fwd_launch_info(64, 64, 28, 28, 64, 1, 7, 1, 0)["kernel"].startswith("conv_mfma_fast_kernel<1, 7, 8, 1, 4, 3, false,")
    assert im2win.conv2d_im2win_fwd_launch_info(64, 64, 28, 28, 64, 7, 1, 1, 3, workspace_free=True)["kernel"].startswith("conv_mfma_fast_kernel<7, 1, 8, 2, 4, 2, true,")
    # 11x11 on three channels: 16-byte operand reads on the two-call path when the stride is a multiple of four
    assert im2win.conv2d_im2win_fwd_launch_info(128, 3, 227, 227, 96, 11, 11, 4, 0)["kernel"] == "conv_mfma_shallow_kernel<11, 11, 3, 3, 2, 4, false, 1, false, true>"
    assert im2win.conv2d_im2win_fwd_launch_info(128, 3, 227, 227, 96, 11, 11, 4, 0, workspace_free=True)["kernel"] == "conv_mfma_shallow_kernel<11, 11, 3, 3, 2, 4, true, 1, false, false>"
    assert im2win.conv2d_im2win_fwd_launch_info(32, 3, 227, 227, 96, 11, 11, 2, 0)["kernel"].endswith(", false, 1, false, false>")
    assert im2win.conv2d_im2win_fwd_launch_info(64, 64, 28, 28, 64, 1, 5, 1, 0)["kernel"] == "conv_mfma_pipe_kernel<0, 0>"
    assert im2win.conv2d_im2win_fwd_launch_info(2, 3, 35, 35, 96, 11, 11, 4, 0)["kernel"] == "conv_mfma_kernel<121, false>"
    assert im2win.conv2d_im2win_fwd_launch_info(2, 10, 35, 35, 96, 9, 9, 2, 0)["kernel"] == "conv_mfma_pipe_kernel<0, 0>"
    assert im2win.conv2d_im2win_fwd_launch_info(1, 2, 40, 40, 8, 17, 17, 1, 0)["kernel"] == "conv_mfma_kernel<0, false>"
    assert im2win.conv2d_im2win_fwd_launch_info(8, 7, 56, 56, 64, 3, 3, 1, 1, workspace_free=True)["kernel"] == "conv_mfma_kernel<9, false>"
    # layers that no tiled kernel takes go to the one-thread-per-output kernels instead of failing
    assert im2win.conv2d_im2win_fwd_launch_info(1, 2, 30, 28, 6, 25, 25, 1, 0)["kernel"] == "conv_basic_kernel"
    assert im2win.conv2d_im2win_fwd_launch_info(1, 2, 30, 28, 6, 25, 25, 1, 0, workspace_free=True)["kernel"] == "conv_direct_kernel"
    # a stride far beyond the image, one output per image: the strips of a tile are 64 windows
    info = im2win.conv2d_im2win_fwd_launch_info(3, 8, 3, 3, 5, 3, 3, 1 << 26, 0)
    assert info["kernel"] == "conv_mfma_kernel<9, false>" and info["lds_bytes"] <= 160 * 1024
    # ... and with two outputs per row the window step no longer fits the tiled kernels' indices
    assert im2win.conv2d_im2win_fwd_launch_info(1, 1, 1, (1 << 28) + 1, 1, 1, 1, 1 << 28, 0)["kernel"] == "conv_basic_kernel"
    # errors as for the calls they describe
    info = binding.LaunchInfo()
    assert lib.conv2d_im2win_fwd_launch_info(1, 1, 4, 4, 1, 5, 5, 1, 0, 0, 0, ctypes.byref(info)) == -2
    assert lib.conv2d_im2win_fwd_launch_info(1, 1, 4, 4, 1, 2, 2, 1, 0, 9, 0, ctypes.byref(info)) == -4
    assert lib.conv2d_im2win_fwd_launch_info(1, 1, 4, 4, 1, 2, 2, 1, 0, 1, 1, ctypes.byref(info)) == -4
    assert lib.conv2d_im2win_fwd_launch_info(1, 1, 4, 4, 1, 2, 2, 1, 0, 0, 0, None) == -1
    assert lib.im2win_transform_launch_info(1, 1, 4, 4, 2, 2, 1, 0, None) == -1


def test_probe_arguments_are_validated(lib):
    one = ctypes.c_void_p(16)
    fl = ctypes.c_double()
    assert lib.im2win_probe_mfma_f32(None, 64, ctypes.byref(fl), None) == -1
    assert lib.im2win_probe_mfma_f32(one, 2, ctypes.byref(fl), None) == -2
    assert lib.im2win_probe_stream(3, one, one, 1024, None) == -4
    assert lib.im2win_probe_stream(0, None, one, 1024, None) == -1
    assert lib.im2win_probe_stream(0, one, one, 1000, None) == -2
    assert lib.im2win_probe_stream(2, None, ctypes.c_void_p(20), 1024, None) == -2


def test_bench_traffic_constants_are_the_profiled_ones():
    """bench.py reports HBM traffic per launch from constants; they must be the figures of the
    kept rocprofv3 summary, not numbers from some other run."""
    import bench
    path = os.path.join(ROOT, "profiles", "all_layers_default_bench.md")
    got = {"conv": {}, "transform": {}}
    for ln in open(path):
        m = re.match(r"\s+TRAFFIC_BYTES (\w+) (\w+) (\d+)", ln)
        if m:
            got[m.group(1)][m.group(2)] = int(m.group(3))
    assert got["conv"] == bench.MEASURED_CONV_TRAFFIC_BYTES
    assert got["transform"] == bench.MEASURED_TRANSFORM_TRAFFIC_BYTES
    assert set(got["conv"]) == {L.name for L in workloads.LAYERS}
