"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs -- bit-exact im2win tensors, convolution outputs within
the stated tolerance -- on the five benchmark layers at full size and on small
shapes that exercise ragged tiles and the degenerate cases."""
import numpy as np
import pytest
import torch

import oracle
import paper_2306_14316_amd as im2win
from paper_2306_14316_amd import workloads

from parity_util import (assert_bitwise_equal, assert_conv_close, check_layer, run_conv,
                         run_transform)

pytestmark = pytest.mark.gpu

# (N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
EDGE_SHAPES = [
    (1, 1, 5, 5, 1, 3, 3, 1, 0),       # a single channel, 9 pixels
    (2, 3, 7, 9, 4, 3, 2, 1, 0),       # asymmetric filter, odd channel count
    (2, 3, 9, 7, 5, 2, 3, 2, 1),
    (1, 2, 11, 13, 3, 5, 3, 3, 3),     # pad as large as the filter allows
    (3, 4, 12, 10, 2, 4, 1, 4, 0),     # stride wider than the filter (gaps between windows)
    (1, 5, 6, 8, 3, 6, 2, 1, 0),       # Hf == Hi: one output row
    (2, 2, 6, 6, 3, 8, 8, 1, 1),       # filter == padded input: 1x1 output per image
    (1, 3, 10, 10, 6, 1, 1, 2, 0),     # 1x1 strided
    (2, 6, 8, 8, 7, 3, 3, 2, 1),
    (5, 8, 9, 9, 65, 3, 3, 1, 1),      # Co one past a tile; 405 pixels (ragged last tile)
    (3, 13, 12, 12, 96, 3, 3, 1, 0),   # Ci not a multiple of the K block, odd tail channel
    (2, 20, 10, 17, 33, 3, 3, 1, 1),   # Ci = 2.5 K blocks
    (70, 4, 3, 3, 8, 3, 3, 1, 0),      # one pixel per image: a tile spans 64 images
    (9, 5, 5, 6, 10, 2, 2, 1, 0),      # 20 pixels per image: tiles straddle images
    (1, 3, 40, 40, 16, 7, 7, 2, 3),    # the 7x7 stride-2 window, small
    (2, 3, 35, 35, 96, 11, 11, 4, 0),  # the 11x11 stride-4 window, small
    (1, 4, 6, 70, 8, 1, 9, 1, 0),      # 1x9 filter: 9-element windows from one row
    (1, 4, 70, 6, 8, 9, 1, 1, 0),      # 9x1 filter
    (1, 2, 4, 300, 4, 3, 3, 1, 1),     # one very wide row
    # multi-channel 5x5 and 7x7 layers: the pipelined kernel's other instances
    (2, 8, 12, 12, 40, 5, 5, 1, 2),
    (1, 12, 24, 24, 70, 5, 5, 1, 0),
    (2, 4, 16, 100, 64, 7, 7, 2, 0),
    (1, 2, 9, 140, 8, 7, 7, 2, 3),
    (1, 6, 30, 70, 33, 7, 7, 2, 3),
    # three-channel layers with wide rows: the filter-stationary kernel
    (2, 3, 70, 150, 40, 7, 7, 2, 3),   # 7x7 s2, Co not a multiple of 32
    (3, 3, 20, 140, 64, 7, 7, 2, 0),
    (1, 3, 40, 260, 96, 7, 7, 2, 3),   # three 32-row filter blocks per workgroup
    (1, 3, 9, 400, 8, 7, 7, 2, 3),     # fewer tiles than workgroups
    (1, 3, 100, 300, 96, 11, 11, 4, 0),  # 11x11 s4: K split between two waves
    (1, 3, 60, 300, 20, 11, 11, 4, 2),
    (2, 3, 50, 290, 64, 11, 11, 4, 0),
    (1, 3, 30, 200, 16, 3, 3, 1, 1),   # 3x3 on three channels
    (1, 3, 36, 280, 100, 3, 3, 1, 1),  # Co = 100: two filter groups in the grid
    # channel counts that are not a multiple of the pipelined kernel's K block: zero-filled last block
    (2, 9, 14, 14, 70, 3, 3, 1, 1),      # 3x3, 9 channels: one real channel in the second block
    (2, 12, 30, 30, 64, 3, 3, 1, 1),
    (1, 60, 56, 56, 64, 3, 3, 1, 1),     # the headline layer's shape with 60 channels
    (1, 15, 20, 150, 40, 3, 3, 2, 0),    # wide rows (two strip words per thread), stride 2
    (2, 6, 16, 16, 40, 5, 5, 1, 2),      # 5x5, 6 channels (K block of 4)
    (1, 5, 30, 70, 33, 7, 7, 2, 3),      # 7x7, 5 channels (K block of 2): odd K, 8-byte fetches at 4-byte alignment
    (1, 256 + 8 + 1, 7, 7, 64, 3, 3, 1, 1),   # 33 whole K blocks and one channel
    # the generic kernel, pipelined (two LDS stages) and, for the largest windows, single-stage
    (2, 256, 14, 14, 70, 1, 1, 1, 0),    # 1x1, four blocks of 64 channels
    (2, 64, 14, 14, 70, 1, 1, 1, 0),     # 1x1, one block: single-stage kernel
    (1, 230, 9, 9, 40, 1, 1, 2, 0),      # 1x1 strided, 64 + 64 + 64 + 38 channels
    (1, 193, 12, 12, 20, 1, 1, 1, 1),    # 1x1 padded, odd channel count: a split step in the last block
    (2, 50, 9, 30, 40, 1, 5, 1, 0),      # 1x5: twelve channels per block, five blocks, the last with two
    (2, 43, 30, 9, 40, 6, 1, 1, 3),      # 6x1 padded, odd channel count: a split step in the last block
    (1, 37, 12, 14, 24, 2, 4, 2, 1),     # 2x4 stride 2: eight channels per block, five blocks, the last with five
    (1, 7, 24, 24, 12, 9, 9, 1, 0),      # 9x9: two channels per block, four blocks, a split step in the last
    (1, 3, 24, 24, 12, 9, 9, 1, 0),      # 9x9 with three channels: too few blocks, single-stage kernel
    (2, 7, 12, 14, 24, 2, 4, 1, 1),      # 2x4, seven channels: one block, single-stage kernel
    (1, 2, 40, 40, 8, 17, 17, 1, 0),     # 17x17: two stages do not fit LDS, single-stage kernel
    # layers no tiled kernel takes: computed by the one-thread-per-output kernels
    (3, 8, 3, 3, 5, 3, 3, 1 << 26, 0),   # a stride far beyond the image (one output per image)
    (2, 8, 5, 3, 5, 3, 3, 2, 0),         # ... and an ordinary one on the same tiny image
    (1, 2, 30, 28, 6, 25, 25, 1, 0),     # a 25x25 window: too large for an LDS filter tile
    (1, 1, 26, 40, 3, 26, 23, 2, 1),
]


@pytest.mark.parametrize("shape", EDGE_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("basic", [False, True], ids=["mfma", "basic"])
def test_edge_shapes(shape, basic):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = workloads.random_layer_inputs(7000 + sum(shape), N, Ci, Hi, Wi, Co, Hf, Wf)
    print("shape", shape, "basic", basic, flush=True)
    check_layer(I, F, s, p, basic=basic)


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_benchmark_layers_full_size(idx):
    """All five layers at their full size, every output element against the oracle."""
    L = workloads.layer(idx)
    print("layer", L.name, flush=True)
    I, F = workloads.make_inputs(L)
    elem, l2 = check_layer(I, F, L.stride, L.pad, basic=False)
    print("layer %s: max|err|/sum|x||w| = %.3e, rel L2 = %.3e" % (L.name, elem, l2), flush=True)


@pytest.mark.parametrize("L", workloads.TABLE2, ids=lambda l: l.name)
def test_table2_layers_small_batch(L):
    """The twelve layers of the paper's Table 2 (unpadded), at batch 3, every element."""
    Ls = workloads.with_batch(L, 3)
    print("layer", Ls.name, flush=True)
    I, F = workloads.make_inputs(Ls)
    check_layer(I, F, Ls.stride, Ls.pad, basic=False, twice=False)


@pytest.mark.parametrize("L", workloads.TABLE2, ids=lambda l: l.name)
def test_table2_layers_full_batch(L):
    """The twelve layers of Table 2 at the paper's batch of 128, in the launch configuration the
    benchmark times: the first and the last image in full (im2win tensor bit for bit, every
    output), 20000 sampled outputs anywhere, and the workspace-free call bit for bit."""
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = L.dims
    print("layer", L.name, flush=True)
    I, F = workloads.make_inputs(L)
    dW = run_transform(I, Hf, Wf, s, p)
    dO = run_conv(dW, F, N, Ci, Hi, Wi, s, p)
    for i in (0, N - 1):
        Ii = I[i:i + 1].numpy()
        assert_bitwise_equal(dW[i:i + 1], oracle.im2win(Ii, Hf, Wf, s, p))
        O_ref, B_ref = oracle.conv2d_direct(Ii, F.numpy(), s, p)
        assert_conv_close(dO[i:i + 1].cpu().numpy(), O_ref, B_ref)
    print("layer", L.name, "samples", flush=True)
    Ho, Wo = im2win.im2win_out_shape(Hi, Wi, Hf, Wf, s, p)
    rng = np.random.default_rng(L.seed)
    idx = np.stack([rng.integers(0, N, 20000), rng.integers(0, Co, 20000),
                    rng.integers(0, Ho, 20000), rng.integers(0, Wo, 20000)], axis=1).astype(np.int32)
    O_s, B_s = oracle.conv2d_direct_at(I.numpy(), F.numpy(), s, p, idx)
    ti = torch.from_numpy(idx.astype(np.int64)).cuda()
    got = dO[ti[:, 0], ti[:, 1], ti[:, 2], ti[:, 3]].cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert (np.abs(got - O_s) <= 1e-4 * B_s).all()
    assert bool(torch.isfinite(dO).all())
    del dW
    print("layer", L.name, "workspace-free", flush=True)
    dO2 = torch.full_like(dO, float("nan"))
    im2win.conv2d_im2win_implicit_fwd(I.cuda(), F.cuda(), dO2, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    assert torch.equal(dO.view(torch.int32), dO2.view(torch.int32))


@pytest.mark.parametrize("Co,pad,Wi", [(64, 0, 224), (20, 1, 223), (96, 1, 223), (64, 0, 223), (40, 0, 221)])
def test_three_channel_3x3_layer_with_many_pixels(Co, pad, Wi):
    """Table 2's Conv7 shape at batch 16: enough pixels for the tiles of four 64-pixel groups
    (one, two and three 32-channel blocks per workgroup; ragged last tile with padding).  The first
    three have output planes of a multiple of four pixels (16-byte stores), the last two do not."""
    I, F = workloads.random_layer_inputs(7700 + Co + Wi, 16, 3, 224, Wi, Co, 3, 3)
    print("conv7-like", Co, pad, Wi, flush=True)
    check_layer(I, F, 1, pad, basic=False, twice=False)


# (N, Ci, Hi, Wi, Co, stride): 1x1 layers without padding, and the form of the dedicated 1x1 kernel that takes
# each: "x4" (pixels by 16-byte loads: stride 1, planes of a multiple of four pixels), "gather" (one word per
# pixel lane: strided layers, other plane sizes) or None (Ci not a multiple of eight, Co not of four)
ONE_BY_ONE_SHAPES = [
    ((2, 64, 8, 8, 64, 1), "x4"),        # one K block, one tile per image
    ((3, 128, 14, 14, 100, 1), "x4"),    # ragged last tile, a partial block of output channels, K blocks of 64
    ((5, 64, 6, 6, 68, 1), "x4"),        # planes of 36 pixels: a tile spans three images
    ((1, 192, 10, 10, 8, 1), "x4"),      # eight output channels
    ((8, 256, 28, 28, 256, 1), "x4"),    # eight K blocks, four channel blocks
    ((2, 64, 2, 2, 64, 1), "x4"),        # planes of four pixels, one ragged tile over both images
    ((2, 96, 8, 8, 64, 1), "x4"),        # 96 input channels
    ((4, 8, 16, 16, 32, 1), "x4"),       # eight input channels: one short block
    ((2, 200, 12, 12, 72, 1), "x4"),     # 200 = 6 * 32 + 8
    ((3, 64, 7, 7, 64, 1), "gather"),    # 49 pixels per plane
    ((4, 128, 28, 28, 256, 2), "gather"),    # stride 2: every second row and column
    ((3, 64, 15, 13, 36, 2), "gather"),      # stride 2 on odd sizes, K blocks of 64
    ((2, 72, 17, 9, 16, 3), "gather"),       # stride 3, a short last K block
    ((70, 64, 3, 3, 64, 2), "gather"),       # planes of four output pixels: a tile spans sixteen images
    ((70, 16, 3, 3, 8, 1 << 26), "gather"),  # a stride far beyond the image: one output pixel per image
    ((2, 64, 8, 8, 66, 1), None),        # 66 output channels
    ((2, 100, 8, 8, 64, 1), None),       # 100 input channels
]


@pytest.mark.parametrize("dims,form", ONE_BY_ONE_SHAPES, ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_one_by_one_layers(dims, form):
    """1x1 convolutions: a plain GEMM over the channel planes (with stride 1 the im2win tensor is the
    input's own layout); both calls and the workspace-free call, every element, bit-identical between
    the two where the dedicated kernel runs."""
    N, Ci, Hi, Wi, Co, st = dims
    shape = (N, Ci, Hi, Wi, Co, 1, 1, st, 0)
    name = im2win.conv2d_im2win_fwd_launch_info(*shape)["kernel"]
    want = {"x4": ", false, ", "gather": ", true, "}
    if form is None:
        assert not name.startswith("conv_mfma_1x1_kernel<"), name
    else:
        assert name.startswith("conv_mfma_1x1_kernel<") and want[form] in name, name
    I, F = workloads.random_layer_inputs(8800 + sum(dims), N, Ci, Hi, Wi, Co, 1, 1)
    print("1x1", dims, name, flush=True)
    check_layer(I, F, st, 0, basic=False)
    dW = run_transform(I, 1, 1, st, 0)
    dO = run_conv(dW, F, N, Ci, Hi, Wi, st, 0)
    dO2 = torch.full_like(dO, float("nan"))
    im2win.conv2d_im2win_implicit_fwd(I.cuda(), F.cuda(), dO2, N, Ci, Hi, Wi, Co, 1, 1, st, 0)
    torch.cuda.synchronize()
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), st, 0)
    assert_conv_close(dO2.cpu().numpy(), O_ref, B_ref)
    if form is not None:
        assert torch.equal(dO.view(torch.int32), dO2.view(torch.int32))


def test_three_channel_3x3_layer_output_off_16_byte_alignment():
    """The Conv7 shape again with an output buffer that starts 4 bytes past a 16-byte boundary: the
    16-byte stores are not used then, and the result is the same bit for bit."""
    N, Co = 16, 64
    I, F = workloads.random_layer_inputs(7790, N, 3, 224, 224, Co, 3, 3)
    dW = run_transform(I, 3, 3, 1, 0)
    dO = run_conv(dW, F, N, 3, 224, 224, 1, 0)
    Ho, Wo = im2win.im2win_out_shape(224, 224, 3, 3, 1, 0)
    buf = torch.full((N * Co * Ho * Wo + 1,), float("nan"), dtype=torch.float32, device="cuda")
    dO2 = buf[1:].view(N, Co, Ho, Wo)
    assert dO2.data_ptr() % 16 == 4
    im2win.conv2d_im2win_fwd(dW, F.cuda(), dO2, N, 3, 224, 224, Co, 3, 3, 1, 0)
    torch.cuda.synchronize()
    assert torch.equal(dO.view(torch.int32), dO2.contiguous().view(torch.int32))
    assert bool(torch.isnan(buf[0]))


# (N, Ci, Hi, Wi, Co, Hf, Wf, s, p): short K loops and at least 2304 tiles, so that the pipelined
# kernel gives every workgroup several tiles and runs its pipeline across tile boundaries
MANY_TILE_SHAPES = [
    (48, 16, 56, 56, 64, 3, 3, 1, 1),    # two K blocks per tile
    (46, 64, 57, 57, 64, 3, 3, 1, 1),    # eight K blocks; ragged last tile; rows of 57 pixels
    (24, 32, 56, 56, 128, 3, 3, 1, 1),   # two M tiles per pixel tile
    (42, 8, 64, 64, 64, 5, 5, 1, 0),     # 5x5 instance
    (40, 4, 128, 128, 64, 7, 7, 2, 0),   # 7x7 stride-2 instance
]


@pytest.mark.parametrize("shape", MANY_TILE_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_many_tiles_per_workgroup(shape):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = workloads.random_layer_inputs(7300 + sum(shape), N, Ci, Hi, Wi, Co, Hf, Wf)
    print("many tiles", shape, flush=True)
    check_layer(I, F, s, p, basic=False, twice=False)
    # the workspace-free variant runs the same pipeline from the input: same bits
    dW = run_transform(I, Hf, Wf, s, p)
    dO = run_conv(dW, F, N, Ci, Hi, Wi, s, p)
    dO2 = torch.full_like(dO, float("nan"))
    im2win.conv2d_im2win_implicit_fwd(I.cuda(), F.cuda(), dO2, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    assert torch.equal(dO.view(torch.int32), dO2.view(torch.int32))


# Filters other than 3x3 / 5x5 / 7x7 with instances of the pipelined kernel (1x7 / 7x1 with eight channels per
# K block, 1x3 / 3x1 / 2x2 with sixteen, 4x4 with four; 5x5 at stride 2), and the neighbours that stay with the
# generic kernels.
ASYMMETRIC_SHAPES = [
    ((4, 16, 20, 40, 70, 1, 7, 1, 0), True),     # 1x7, two K blocks, a partial block of output channels
    ((2, 24, 17, 150, 64, 1, 7, 2, 3), True),    # 1x7 stride 2, padded
    ((2, 8, 9, 300, 16, 1, 7, 4, 0), True),      # 1x7 stride 4: two strip words per thread
    ((2, 34, 9, 30, 40, 1, 7, 1, 0), True),      # 1x7, 34 channels: a last K block with two
    ((3, 16, 40, 20, 70, 7, 1, 1, 3), True),     # 7x1 padded
    ((2, 27, 30, 9, 40, 7, 1, 1, 3), True),      # 7x1, 27 channels: a last K block with three
    ((2, 8, 60, 9, 24, 7, 1, 2, 0), False),      # 7x1 stride 2: a tile's strips are longer than the instance's
    ((2, 32, 14, 30, 40, 1, 3, 1, 1), True),     # 1x3 padded, two K blocks of sixteen channels
    ((2, 40, 14, 30, 40, 1, 3, 1, 1), True),     # 1x3, 40 channels: half a K block left over
    ((2, 48, 30, 14, 40, 3, 1, 1, 0), True),     # 3x1
    ((1, 17, 30, 14, 72, 3, 1, 2, 1), False),    # 3x1 stride 2: strips longer than the instance's
    ((1, 17, 30, 14, 72, 1, 3, 2, 1), True),     # 1x3 stride 2, 17 channels
    ((2, 12, 14, 30, 40, 1, 3, 1, 1), False),    # 1x3 with fewer channels than a K block
    ((48, 16, 56, 56, 64, 1, 7, 1, 3), True),    # 1x7: several tiles per workgroup
    ((32, 32, 56, 56, 64, 3, 1, 1, 1), True),    # 3x1: several tiles per workgroup
    ((2, 8, 20, 20, 40, 4, 4, 2, 1), True),      # 4x4 stride 2: a tile spans seven rows
    ((2, 64, 64, 64, 64, 4, 4, 2, 1), True),     # 4x4 stride 2, sixteen K blocks, two rows per tile
    ((1, 16, 16, 130, 16, 4, 4, 2, 1), True),    # 4x4 stride 2, rows of 65 pixels
    ((2, 12, 12, 30, 24, 4, 4, 1, 0), True),     # 4x4 stride 1, three K blocks
    ((2, 6, 12, 30, 24, 4, 4, 1, 2), True),      # 4x4, six channels: half a K block left over
    ((2, 8, 32, 32, 96, 4, 4, 4, 0), False),     # 4x4 stride 4: strips longer than the instances'
    ((32, 8, 112, 112, 64, 4, 4, 2, 1), True),   # 4x4 stride 2: several tiles per workgroup
    ((2, 16, 20, 20, 40, 2, 2, 2, 0), True),     # 2x2 stride 2, one K block of sixteen channels
    ((2, 48, 33, 31, 70, 2, 2, 2, 1), True),     # 2x2 stride 2 padded, odd sizes
    ((2, 40, 16, 16, 24, 2, 2, 1, 0), True),     # 2x2 stride 1, 40 channels: half a K block left over
    ((32, 32, 112, 112, 64, 2, 2, 2, 0), True),  # 2x2 stride 2: several tiles per workgroup
    ((2, 8, 24, 100, 40, 5, 5, 2, 2), True),     # 5x5 stride 2: three strip words per thread
    ((1, 10, 30, 110, 70, 5, 5, 2, 0), True),    # 5x5 stride 2, ten channels: half a K block left over
]


@pytest.mark.parametrize("shape,pipelined", ASYMMETRIC_SHAPES, ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_asymmetric_filters(shape, pipelined):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    name = im2win.conv2d_im2win_fwd_launch_info(*shape)["kernel"]
    assert name.startswith("conv_mfma_fast_kernel<%d, %d," % (Hf, Wf)) == pipelined, name
    I, F = workloads.random_layer_inputs(7700 + sum(shape), N, Ci, Hi, Wi, Co, Hf, Wf)
    print("asymmetric", shape, name, flush=True)
    check_layer(I, F, s, p, basic=False, twice=False)
    dW = run_transform(I, Hf, Wf, s, p)
    dO = run_conv(dW, F, N, Ci, Hi, Wi, s, p)
    dO2 = torch.full_like(dO, float("nan"))
    im2win.conv2d_im2win_implicit_fwd(I.cuda(), F.cuda(), dO2, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    if pipelined:   # the workspace-free variant runs the same pipeline from the input: same bits
        assert torch.equal(dO.view(torch.int32), dO2.view(torch.int32))
    else:
        O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), s, p)
        assert_conv_close(dO2.cpu().numpy(), O_ref, B_ref)


# Layers whose tile count leaves a few tiles (at most an eighth of the compute units) after the
# last full round of the grid: the pipelined 3x3 kernel computes those in sixteen 16x16 pieces,
# the four waves of a workgroup splitting the channels (a multiple of 16).  Tile counts are for
# 256 compute units.
LEFTOVER_TILE_SHAPES = [
    (1, 16, 130, 130, 64, 3, 3, 1, 1),   # 265 tiles: 9 left; one channel group per wave; last tile has 4 pixels
    (1, 48, 96, 96, 88, 3, 3, 1, 0),     # 278 tiles: 22 left; 3 groups per wave; second M tile: 24 of 64 rows
    (11, 128, 78, 78, 40, 3, 3, 2, 1),   # 262 tiles: 6 left; 8 groups per wave (one refill); stride 2; tiles cross rows and images
    (7, 32, 50, 50, 64, 3, 3, 1, 1),     # 274 tiles: 18 left
]


@pytest.mark.parametrize("shape", LEFTOVER_TILE_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_leftover_tiles_in_pieces(shape):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = workloads.random_layer_inputs(7900 + sum(shape), N, Ci, Hi, Wi, Co, Hf, Wf)
    print("leftover tiles", shape, flush=True)
    check_layer(I, F, s, p, basic=False, twice=False)
    dW = run_transform(I, Hf, Wf, s, p)
    dO = run_conv(dW, F, N, Ci, Hi, Wi, s, p)
    dO2 = torch.full_like(dO, float("nan"))
    im2win.conv2d_im2win_implicit_fwd(I.cuda(), F.cuda(), dO2, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    assert torch.equal(dO.view(torch.int32), dO2.view(torch.int32))


# Leftovers of up to half of the compute units that do not qualify for the sixteenths (more than
# an eighth of the compute units, or channels not a multiple of 16): two half tiles of 32 pixels
# each, two waves per block of outputs splitting the channel pairs of every K block.
HALF_TILE_SHAPES = [
    (1, 8, 130, 130, 64, 3, 3, 1, 1),    # 265 tiles: 9 left; one K block; the last tile's second half is empty
    (1, 24, 96, 96, 88, 3, 3, 1, 0),     # 278 tiles: 22 left; three K blocks; second M tile: 24 of 64 rows
    (11, 40, 78, 78, 40, 3, 3, 2, 1),    # 262 tiles: 6 left; five K blocks; stride 2; tiles cross rows and images
    (7, 64, 56, 56, 64, 3, 3, 1, 1),     # 343 tiles: 87 left; eight K blocks
    (9, 32, 50, 50, 128, 3, 3, 1, 0),    # 648 tiles (two M tiles each): 136 left -> 128 in halves, 8 in sixteenths
    (8, 32, 42, 42, 128, 3, 3, 1, 0),    # 400 tiles: 144 left -> 128 in halves, 16 in sixteenths
    (8, 24, 42, 42, 128, 3, 3, 1, 0),    # the same with 24 channels: no sixteenths, the 144 stay whole
    (9, 32, 53, 53, 128, 3, 3, 1, 0),    # 732 tiles: 220 left: too many, all whole
    (5, 8, 68, 68, 64, 5, 5, 1, 0),      # the 5x5 instance: 320 tiles, 64 left, two K blocks
    (3, 12, 60, 60, 70, 5, 5, 1, 2),     # 5x5: 338 tiles, 82 left, three K blocks, second M tile: 6 of 64 rows
]


@pytest.mark.parametrize("shape", HALF_TILE_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_leftover_tiles_in_halves(shape):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = workloads.random_layer_inputs(7950 + sum(shape), N, Ci, Hi, Wi, Co, Hf, Wf)
    print("half tiles", shape, flush=True)
    check_layer(I, F, s, p, basic=False, twice=True)
    dW = run_transform(I, Hf, Wf, s, p)
    dO = run_conv(dW, F, N, Ci, Hi, Wi, s, p)
    dO2 = torch.full_like(dO, float("nan"))
    im2win.conv2d_im2win_implicit_fwd(I.cuda(), F.cuda(), dO2, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    assert torch.equal(dO.view(torch.int32), dO2.view(torch.int32))


def test_im2win_tensor_larger_than_4_gib():
    """A 5 GB im2win tensor (byte offsets pass 2^32): images at both ends and in the
    middle are checked in full, plus sampled outputs anywhere."""
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = 512, 64, 112, 112, 16, 3, 3, 1, 1
    g = torch.Generator(device="cpu")
    g.manual_seed(4242)
    I = torch.rand((N, Ci, Hi, Wi), generator=g, dtype=torch.float32)
    F = torch.randn((Co, Ci, Hf, Wf), generator=g, dtype=torch.float32) * 0.06
    Ho, Wo = im2win.im2win_out_shape(Hi, Wi, Hf, Wf, s, p)
    assert im2win.im2win_workspace_bytes(N, Ci, Hi, Wi, Hf, Wf, s, p) > 2 ** 32
    print("large tensor: transform", flush=True)
    dW = run_transform(I, Hf, Wf, s, p)
    print("large tensor: convolution", flush=True)
    dO = run_conv(dW, F, N, Ci, Hi, Wi, s, p)
    for i in (0, 255, 511):
        Ii = I[i:i + 1].numpy()
        assert_bitwise_equal(dW[i:i + 1], oracle.im2win(Ii, Hf, Wf, s, p))
        O_ref, B_ref = oracle.conv2d_direct(Ii, F.numpy(), s, p)
        assert_conv_close(dO[i:i + 1].cpu().numpy(), O_ref, B_ref)
    rng = np.random.default_rng(7)
    idx = np.stack([rng.integers(0, N, 20000), rng.integers(0, Co, 20000),
                    rng.integers(0, Ho, 20000), rng.integers(0, Wo, 20000)], axis=1).astype(np.int32)
    O_s, B_s = oracle.conv2d_direct_at(I.numpy(), F.numpy(), s, p, idx)
    got = dO.cpu().numpy()[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].astype(np.float64)
    assert np.isfinite(got).all()
    assert (np.abs(got - O_s) <= 1e-4 * B_s).all()
    assert not bool(torch.isnan(dO).any())


@pytest.mark.parametrize("Ci", [8, 3])
def test_output_planes_beyond_32_bit_offsets(Ci):
    """One 2900x2900 image, 64 output channels: an output tile's channels lie more than 4 GiB
    apart, past the 32-bit offsets of the stores of the pipelined kernel (8 input channels)
    and of the filter-stationary kernel (3 input channels), so the layer must take a kernel
    that addresses its output with full pointers.  Sampled outputs, plus the first and the last
    output rows of every channel (the ends of the 2.1 GB output)."""
    N, Hi, Wi, Co, Hf, Wf, s, p = 1, 2900, 2900, 64, 3, 3, 1, 0
    g = torch.Generator(device="cpu")
    g.manual_seed(4343 + Ci)
    I = torch.rand((N, Ci, Hi, Wi), generator=g, dtype=torch.float32)
    F = torch.randn((Co, Ci, Hf, Wf), generator=g, dtype=torch.float32) * 0.15
    Ho, Wo = im2win.im2win_out_shape(Hi, Wi, Hf, Wf, s, p)
    assert 4 * Co * Ho * Wo > 2 ** 31
    print("huge image: transform + convolution", flush=True)
    dW = run_transform(I, Hf, Wf, s, p)
    dO = run_conv(dW, F, N, Ci, Hi, Wi, s, p)
    assert bool(torch.isfinite(dO).all())
    rng = np.random.default_rng(11)
    idx = np.stack([np.zeros(20000, dtype=np.int64), rng.integers(0, Co, 20000),
                    rng.integers(0, Ho, 20000), rng.integers(0, Wo, 20000)], axis=1)
    rows = np.array([(0, j, m, n) for j in range(Co) for m in (0, Ho - 1) for n in range(0, Wo, 7)])
    idx = np.concatenate([idx, rows]).astype(np.int32)
    O_s, B_s = oracle.conv2d_direct_at(I.numpy(), F.numpy(), s, p, idx)
    ti = torch.from_numpy(idx.astype(np.int64)).cuda()
    got = dO[ti[:, 0], ti[:, 1], ti[:, 2], ti[:, 3]].cpu().numpy().astype(np.float64)
    assert (np.abs(got - O_s) <= 1e-4 * B_s).all()
    del dW
    print("huge image: workspace-free", flush=True)
    dO2 = torch.full_like(dO, float("nan"))
    im2win.conv2d_im2win_implicit_fwd(I.cuda(), F.cuda(), dO2, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    got2 = dO2[ti[:, 0], ti[:, 1], ti[:, 2], ti[:, 3]].cpu().numpy().astype(np.float64)
    assert (np.abs(got2 - O_s) <= 1e-4 * B_s).all()
    assert bool(torch.isfinite(dO2).all())


@pytest.mark.parametrize("idx", [1, 2])
def test_basic_kernel_on_benchmark_layers(idx):
    L = workloads.layer(idx)
    I, F = workloads.make_inputs(L)
    check_layer(I, F, L.stride, L.pad, basic=True, twice=False)


VARIANT_SHAPES = [
    (1, 3, 32, 32, 16, 3, 3, 1, 0),      # the tiny benchmark layer
    (4, 64, 56, 56, 64, 3, 3, 1, 1),     # the headline layer at batch 4
    (2, 16, 20, 20, 40, 3, 3, 1, 1),     # ragged Co
    (1, 3, 40, 260, 64, 7, 7, 2, 3),     # a three-channel 7x7 layer
    (2, 5, 9, 9, 7, 2, 3, 2, 1),         # a small odd layer
    (2, 16, 30, 150, 70, 3, 3, 1, 1),    # wide rows: two strip words per thread in the 3x3 instances
    (3, 13, 12, 12, 96, 5, 5, 1, 2),     # odd channel count, 5x5
]


@pytest.mark.parametrize("shape", VARIANT_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 5])
def test_ablation_variants(shape, variant):
    """Every ablation variant computes the same convolution."""
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = workloads.random_layer_inputs(9000 + sum(shape), N, Ci, Hi, Wi, Co, Hf, Wf)
    dW = run_transform(I, Hf, Wf, s, p)
    Ho, Wo = im2win.im2win_out_shape(Hi, Wi, Hf, Wf, s, p)
    dO = torch.full((N, Co, Ho, Wo), float("nan"), dtype=torch.float32, device="cuda")
    im2win.conv2d_im2win_fwd_variant(dW, F.cuda(), dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p, variant)
    torch.cuda.synchronize()
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), s, p)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)


def test_unknown_variant_is_rejected():
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = 1, 2, 6, 6, 3, 3, 3, 1, 0
    I, F = workloads.random_layer_inputs(5, N, Ci, Hi, Wi, Co, Hf, Wf)
    dW = run_transform(I, Hf, Wf, s, p)
    dO = torch.zeros((N, Co, 4, 4), dtype=torch.float32, device="cuda")
    for bad in (-1, 6, 99):
        with pytest.raises(im2win.Im2winError):
            im2win.conv2d_im2win_fwd_variant(dW, F.cuda(), dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p, bad)
    assert not bool(dO.any())      # nothing was launched


def test_transform_copies_bit_patterns():
    """NaN payloads, infinities, -0.0 and denormals pass through untouched; padding is +0.0."""
    bits = np.array([0x7FC00001, 0xFFC12345, 0x7F800001, 0x80000000, 0x00000001, 0x807FFFFF,
                     0x7F800000, 0xFF800000, 0x3F800000], dtype=np.uint32)
    I = torch.from_numpy(np.resize(bits, 3 * 2 * 9 * 11).view(np.float32).reshape(3, 2, 9, 11).copy())
    for (Hf, Wf, s, p) in [(2, 2, 1, 1), (3, 3, 2, 0), (4, 1, 3, 2)]:
        dW = run_transform(I, Hf, Wf, s, p)
        assert_bitwise_equal(dW, oracle.im2win(I.numpy(), Hf, Wf, s, p))


# (N, Ci, Hi, Wi, Hf, s, p): the transform kernel that assembles a workgroup's stretch of the
# tensor in LDS (row blocks of one plane, or groups of whole small planes), and its fallbacks
TALL_WINDOW_SHAPES = [
    (2, 3, 37, 65, 5, 1, 0),     # odd row length: workgroup stretches start at every word offset mod 4
    (1, 2, 50, 71, 7, 2, 3),     # Ho not a multiple of the rows per workgroup; the 7/2 instance with padding
    (3, 1, 23, 64, 5, 6, 0),     # stride wider than the window: input rows that no window uses
    (1, 2, 9, 90, 9, 1, 0),      # one output row per plane
    (1, 1, 30, 500, 11, 4, 5),   # wide rows: one or two output rows per workgroup; the 11/4 instance
    (1, 1, 12, 1100, 9, 1, 1),   # more than 256 sixteen-byte pieces per input row: falls back to the gather
    (1, 1, 20, 1000, 17, 1, 0),  # an im2win row too long for LDS: falls back to the gather
    (1, 1, 5, 64, 5, 1, 0),      # a single output row, fewer words than threads
    (5, 13, 9, 7, 3, 1, 0),      # small planes in groups: 65 planes of 147 words, a ragged last group
    (3, 7, 6, 6, 3, 1, 1),       # ... all planes in one workgroup, padded
    (4, 6, 5, 9, 3, 1, 2),       # ... padding wider than the reach of the filter
    (2, 9, 11, 5, 4, 1, 0),      # rows of five words: the second piece overlaps the first; generic instance
    (2, 5, 10, 4, 2, 2, 1),      # rows of exactly one piece
    (1, 3, 40, 6, 1, 1, 0),      # Hf = 1: the identity copy
    (2, 2, 33, 130, 3, 2, 1),    # 3-row windows at stride 2: generic instance, row blocks
    (1, 2, 300, 31, 5, 1, 2),    # tall narrow planes, 5/1 instance, many row blocks
    (1, 1, 4, 3, 2, 1, 0),       # rows shorter than one piece: the gather
]


@pytest.mark.parametrize("shape", TALL_WINDOW_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_transform_tall_windows(shape):
    N, Ci, Hi, Wi, Hf, s, p = shape
    I, _ = workloads.random_layer_inputs(8000 + sum(shape), N, Ci, Hi, Wi, 1, Hf, 1)
    print("transform shape", shape, flush=True)
    Ho, _ = im2win.im2win_out_shape(Hi, Wi, Hf, 1, s, p)
    n = N * Ci * Ho * (Wi + 2 * p) * Hf
    buf = torch.full((n + 64,), float("nan"), dtype=torch.float32, device="cuda")
    win = buf[32:32 + n]                                   # 128-byte offset: stays 16-byte aligned
    im2win.im2win_transform(I.cuda(), win, N, Ci, Hi, Wi, Hf, 1, s, p)
    torch.cuda.synchronize()
    assert_bitwise_equal(win.reshape(N, Ci, Ho, -1), oracle.im2win(I.numpy(), Hf, 1, s, p))
    assert torch.isnan(buf[:32]).all() and torch.isnan(buf[32 + n:]).all()   # nothing written outside


# (N, Ci, Hi, Wi, Hf, s, p): short windows on large tensors (input + im2win tensor of 192 MiB or more)
LARGE_SHORT_WINDOW_SHAPES = [
    (64, 20, 150, 131, 3, 1, 1),   # odd row length (399 words): stretches start at every word offset mod 4
    (96, 24, 150, 131, 3, 2, 2),   # stride 2, two rows and columns of padding
    (40, 16, 161, 190, 4, 1, 0),   # a four-row window
]


@pytest.mark.parametrize("shape", LARGE_SHORT_WINDOW_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_transform_short_windows_large_tensors(shape):
    N, Ci, Hi, Wi, Hf, s, p = shape
    Ho, _ = im2win.im2win_out_shape(Hi, Wi, Hf, 1, s, p)
    n = N * Ci * Ho * (Wi + 2 * p) * Hf
    assert 4 * (N * Ci * Hi * Wi + n) >= 192 * 2 ** 20 and Wi + 2 * p >= 48
    g = torch.Generator(device="cpu")
    g.manual_seed(8100 + sum(shape))
    I = torch.randn((N, Ci, Hi, Wi), generator=g, dtype=torch.float32)
    print("transform shape", shape, flush=True)
    buf = torch.full((n + 64,), float("nan"), dtype=torch.float32, device="cuda")
    win = buf[32:32 + n]
    im2win.im2win_transform(I.cuda(), win, N, Ci, Hi, Wi, Hf, 1, s, p)
    torch.cuda.synchronize()
    assert_bitwise_equal(win.reshape(N, Ci, Ho, -1), oracle.im2win(I.numpy(), Hf, 1, s, p))
    assert torch.isnan(buf[:32]).all() and torch.isnan(buf[32 + n:]).all()   # nothing written outside


def test_transform_unaligned_output_pointer():
    """A window buffer that is only 4-byte aligned takes the scalar-store path."""
    N, Ci, Hi, Wi, Hf, Wf, s, p = 2, 3, 9, 10, 3, 3, 1, 1
    I, _ = workloads.random_layer_inputs(11, N, Ci, Hi, Wi, 1, Hf, Wf)
    Ho, _ = im2win.im2win_out_shape(Hi, Wi, Hf, Wf, s, p)
    n = N * Ci * Ho * (Wi + 2 * p) * Hf
    buf = torch.full((n + 8,), float("nan"), dtype=torch.float32, device="cuda")
    win = buf[1:1 + n]
    im2win.im2win_transform(I.cuda(), win, N, Ci, Hi, Wi, Hf, Wf, s, p)
    torch.cuda.synchronize()
    assert_bitwise_equal(win.reshape(N, Ci, Ho, -1), oracle.im2win(I.numpy(), Hf, Wf, s, p))
    assert torch.isnan(buf[0]) and torch.isnan(buf[1 + n:]).all()      # nothing written outside


def test_unaligned_filter_pointer_takes_scalar_staging():
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = 2, 8, 10, 10, 20, 3, 3, 1, 1
    I, F = workloads.random_layer_inputs(12, N, Ci, Hi, Wi, Co, Hf, Wf)
    dW = run_transform(I, Hf, Wf, s, p)
    fbuf = torch.zeros(F.numel() + 4, dtype=torch.float32, device="cuda")
    dF = fbuf[1:1 + F.numel()]
    dF.copy_(F.reshape(-1))
    Ho, Wo = im2win.im2win_out_shape(Hi, Wi, Hf, Wf, s, p)
    dO = torch.full((N, Co, Ho, Wo), float("nan"), dtype=torch.float32, device="cuda")
    im2win.conv2d_im2win_fwd(dW, dF, dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), s, p)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)


def test_outputs_do_not_spill_outside_their_buffers():
    """Guard bands around the output stay untouched."""
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = 3, 5, 9, 9, 37, 3, 3, 2, 1
    I, F = workloads.random_layer_inputs(13, N, Ci, Hi, Wi, Co, Hf, Wf)
    dW = run_transform(I, Hf, Wf, s, p)
    Ho, Wo = im2win.im2win_out_shape(Hi, Wi, Hf, Wf, s, p)
    n = N * Co * Ho * Wo
    for fn in (im2win.conv2d_im2win_fwd, im2win.conv2d_im2win_fwd_basic):
        buf = torch.full((n + 512,), float("nan"), dtype=torch.float32, device="cuda")
        out = buf[256:256 + n]
        fn(dW, F.cuda(), out, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
        torch.cuda.synchronize()
        assert torch.isnan(buf[:256]).all() and torch.isnan(buf[256 + n:]).all()
        O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), s, p)
        assert_conv_close(out.reshape(N, Co, Ho, Wo).cpu().numpy(), O_ref, B_ref)


def test_runs_on_a_side_stream():
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = 2, 4, 12, 12, 8, 3, 3, 1, 1
    I, F = workloads.random_layer_inputs(14, N, Ci, Hi, Wi, Co, Hf, Wf)
    Ho, Wo = im2win.im2win_out_shape(Hi, Wi, Hf, Wf, s, p)
    dI, dF = I.cuda(), F.cuda()
    dW = torch.empty((N, Ci, Ho, (Wi + 2 * p) * Hf), dtype=torch.float32, device="cuda")
    dO = torch.empty((N, Co, Ho, Wo), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        im2win.im2win_transform(dI, dW, N, Ci, Hi, Wi, Hf, Wf, s, p)
        im2win.conv2d_im2win_fwd(dW, dF, dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    st.synchronize()
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), s, p)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)
