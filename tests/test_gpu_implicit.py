"""GPU tests of the workspace-free variant (im2win strips built in LDS from the
NCHW input) against the CPU oracle, through the C ABI."""
import pytest
import torch

import oracle
import paper_2306_14316_amd as im2win
from paper_2306_14316_amd import workloads
from parity_util import POISON, assert_conv_close

pytestmark = pytest.mark.gpu

# (N, Ci, Hi, Wi, Co, Hf, Wf, s, p): layers the pipelined kernel takes
SHAPES = [
    (5, 8, 9, 9, 65, 3, 3, 1, 1),        # padding on all sides; Co one past a tile; ragged last tile
    (3, 16, 12, 12, 96, 3, 3, 1, 0),     # no padding
    (2, 24, 10, 17, 33, 3, 3, 2, 1),     # stride 2
    (70, 8, 4, 4, 8, 3, 3, 1, 0),        # four pixels per image: a tile spans 16 images
    (9, 8, 5, 6, 10, 3, 3, 1, 1),        # tiles straddle images
    (1, 8, 4, 300, 4, 3, 3, 1, 1),       # one very wide row (two strip words per thread)
    (2, 8, 7, 7, 16, 3, 3, 1, 3),        # padding wider than the filter's reach: all-zero windows
    (2, 8, 12, 12, 40, 5, 5, 1, 2),      # 5x5
    (1, 12, 24, 24, 70, 5, 5, 1, 0),
    (2, 4, 16, 100, 64, 7, 7, 2, 0),     # 7x7 stride 2
    (1, 2, 9, 140, 8, 7, 7, 2, 3),
    (1, 6, 30, 70, 33, 7, 7, 2, 3),
    (3, 8, 11, 13, 20, 3, 3, 2, 2),      # stride 2, padding 2: tiles of nine short rows
    (2, 9, 14, 14, 70, 3, 3, 1, 1),      # channel counts off the K block: zero-filled last block
    (1, 60, 56, 56, 64, 3, 3, 1, 1),
    (2, 6, 16, 16, 40, 5, 5, 1, 2),
    (1, 5, 30, 70, 33, 7, 7, 2, 3),
]


def _run(I, F, s, p):
    N, Ci, Hi, Wi = I.shape
    Co, _, Hf, Wf = F.shape
    Ho, Wo = im2win.im2win_out_shape(Hi, Wi, Hf, Wf, s, p)
    dO = torch.full((N, Co, Ho, Wo), POISON, dtype=torch.float32, device="cuda")
    im2win.conv2d_im2win_implicit_fwd(I.cuda(), F.cuda(), dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    return dO


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_implicit_edge_shapes(shape):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = workloads.random_layer_inputs(5000 + sum(shape), N, Ci, Hi, Wi, Co, Hf, Wf)
    print("implicit", shape, flush=True)
    dO = _run(I, F, s, p)
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), s, p)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)
    dO2 = _run(I, F, s, p)   # a second run reproduces the first bit for bit
    assert torch.equal(dO.view(torch.int32), dO2.view(torch.int32))


@pytest.mark.parametrize("idx", [2, 3])
def test_implicit_benchmark_layers_full_size(idx):
    L = workloads.layer(idx)
    print("implicit layer", L.name, flush=True)
    I, F = workloads.make_inputs(L)
    dO = _run(I, F, L.stride, L.pad)
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), L.stride, L.pad)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)


def test_implicit_matches_two_call_path_bitwise():
    """Same strips in LDS, same MFMA order: the result equals the transform + convolution path's."""
    L = workloads.with_batch(workloads.layer(2), 4)
    I, F = workloads.make_inputs(L)
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = L.dims
    dO = _run(I, F, s, p)
    dW = torch.empty(oracle.im2win_elems(N, Ci, Hi, Wi, Hf, Wf, s, p), dtype=torch.float32, device="cuda")
    dO2 = torch.full_like(dO, POISON)
    im2win.im2win_transform(I.cuda(), dW, N, Ci, Hi, Wi, Hf, Wf, s, p)
    im2win.conv2d_im2win_fwd(dW, F.cuda(), dO2, *L.dims)
    torch.cuda.synchronize()
    assert torch.equal(dO.view(torch.int32), dO2.view(torch.int32))


@pytest.mark.parametrize("L", [l for l in workloads.TABLE2 if l.Ci > 3], ids=lambda l: l.name)
def test_implicit_table2_layers_small_batch(L):
    Ls = workloads.with_batch(L, 3)
    I, F = workloads.make_inputs(Ls)
    print("implicit", Ls.name, flush=True)
    dO = _run(I, F, Ls.stride, Ls.pad)
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), Ls.stride, Ls.pad)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)


# layers outside the pipelined kernel's shapes: the generic kernel builds the strips from the input
OTHER_SHAPES = [
    (1, 1, 5, 5, 1, 3, 3, 1, 0),
    (2, 3, 7, 9, 4, 3, 2, 1, 0),       # asymmetric filter, odd channel count
    (2, 3, 9, 7, 5, 2, 3, 2, 1),
    (1, 2, 11, 13, 3, 5, 3, 3, 3),     # pad as large as the filter allows
    (3, 4, 12, 10, 2, 4, 1, 4, 0),     # stride wider than the filter
    (1, 5, 6, 8, 3, 6, 2, 1, 0),       # Hf == Hi
    (2, 2, 6, 6, 3, 8, 8, 1, 1),       # filter == padded input
    (1, 3, 10, 10, 6, 1, 1, 2, 0),     # 1x1 strided
    (3, 13, 12, 12, 96, 3, 3, 1, 0),   # Ci not a multiple of the K block
    (70, 4, 3, 3, 8, 3, 3, 1, 0),      # one pixel per image
    (1, 3, 40, 40, 16, 7, 7, 2, 3),    # three-channel 7x7 stride 2
    (2, 3, 35, 35, 96, 11, 11, 4, 0),  # three-channel 11x11 stride 4
    (1, 4, 6, 70, 8, 1, 9, 1, 0),      # 1x9
    # three-channel layers with wide rows: the filter-stationary kernel gathers from the input
    (2, 3, 70, 150, 40, 7, 7, 2, 3),
    (3, 3, 20, 140, 64, 7, 7, 2, 0),
    (1, 3, 40, 260, 96, 7, 7, 2, 3),
    (1, 3, 9, 400, 8, 7, 7, 2, 3),
    (1, 3, 100, 300, 96, 11, 11, 4, 0),
    (1, 3, 60, 300, 20, 11, 11, 4, 2),
    (2, 3, 50, 290, 64, 11, 11, 4, 0),
    (1, 3, 30, 200, 16, 3, 3, 1, 1),
    (1, 3, 36, 280, 100, 3, 3, 1, 1),
    (4, 3, 3, 70, 8, 3, 3, 1, 1),      # short images: a tile spans three images
    (1, 4, 70, 6, 8, 9, 1, 1, 2),      # 9x1, padded
    # layers no tiled kernel takes: the direct one-thread-per-output kernel computes them
    (3, 8, 3, 3, 5, 3, 3, 1 << 26, 0),   # a stride far beyond the image
    (1, 2, 30, 28, 6, 25, 25, 1, 0),     # a 25x25 window
]


@pytest.mark.parametrize("shape", OTHER_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_implicit_other_shapes(shape):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = workloads.random_layer_inputs(5500 + sum(shape), N, Ci, Hi, Wi, Co, Hf, Wf)
    print("implicit (generic)", shape, flush=True)
    dO = _run(I, F, s, p)
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), s, p)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)


@pytest.mark.parametrize("pad", [1, 0])
def test_implicit_three_channel_3x3_layer_with_many_pixels(pad):
    """Conv7's shape at batch 16 (tiles of four pixel groups), gathered from the input; output planes
    of 224x223 pixels (a multiple of four: 16-byte stores) and of 222x221."""
    I, F = workloads.random_layer_inputs(7801 + pad, 16, 3, 224, 223, 64, 3, 3)
    dO = _run(I, F, 1, pad)
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), 1, pad)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)


def test_implicit_three_channel_layers_small_batch():
    for idx in (1, 4, 5):
        L = workloads.layer(idx)
        Ls = workloads.with_batch(L, min(L.N, 2))
        I, F = workloads.make_inputs(Ls)
        print("implicit", Ls.name, flush=True)
        dO = _run(I, F, Ls.stride, Ls.pad)
        O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), Ls.stride, Ls.pad)
        assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)
