"""Seeded random layer shapes through every route of the library (two-call im2win path,
workspace-free variant, im2col + GEMM, direct) against the CPU oracle.  The generator is
biased towards the boundaries the kernels care about: channel counts around the K blocks,
rows around the 64-pixel tile, three-channel wide rows, strides and paddings up to the
filter size."""
import numpy as np
import pytest
import torch

import oracle
import paper_2306_14316_amd as im2win
from paper_2306_14316_amd import workloads
from parity_util import POISON, assert_bitwise_equal, assert_conv_close, run_conv, run_transform

pytestmark = pytest.mark.gpu


def _shapes(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        kind = rng.integers(0, 4)
        if kind == 0:      # multi-channel square filters: the pipelined kernel's territory
            Hf = Wf = int(rng.choice([3, 3, 5, 7]))
            Ci = int(rng.choice([2, 4, 6, 8, 12, 16, 24, 40]))
            Hi, Wi = int(rng.integers(Hf, 30)), int(rng.integers(Hf, 90))
        elif kind == 1:    # three channels, wide rows: the filter-stationary kernel's territory
            Hf = Wf = int(rng.choice([3, 7, 11]))
            Ci = 3
            Hi, Wi = int(rng.integers(Hf, 40)), int(rng.integers(120, 420))
        elif kind == 2:    # anything: asymmetric filters, odd channel counts
            Hf, Wf = int(rng.integers(1, 8)), int(rng.integers(1, 8))
            Ci = int(rng.integers(1, 21))
            Hi, Wi = int(rng.integers(Hf, 26)), int(rng.integers(Wf, 40))
        else:              # tiny images, many of them: tiles straddle images
            Hf = Wf = int(rng.choice([1, 2, 3]))
            Ci = int(rng.choice([3, 8, 16]))
            Hi, Wi = int(rng.integers(Hf, 8)), int(rng.integers(Wf, 8))
        s = min(int(rng.choice([1, 1, 1, 2, 2, 3, 4])), min(Hf, Wf) + 1)
        p = int(rng.integers(0, min(Hf, Wf) + 1))
        N = int(rng.integers(1, 6)) if kind != 3 else int(rng.integers(8, 80))
        Co = int(rng.choice([1, 5, 16, 31, 32, 33, 64, 65, 96, 100]))
        Ho, Wo = (Hi + 2 * p - Hf) // s + 1, (Wi + 2 * p - Wf) // s + 1
        if Ho < 1 or Wo < 1:
            continue
        if N * Co * Ho * Wo * Ci * Hf * Wf > 4e8:      # keep the oracle to a fraction of a second
            continue
        out.append((N, Ci, Hi, Wi, Co, Hf, Wf, s, p))
    return out


SHAPES = _shapes(20230614, 48)


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_random_shape_all_routes(shape):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = workloads.random_layer_inputs(4000 + sum(shape), N, Ci, Hi, Wi, Co, Hf, Wf)
    print("random shape", shape, flush=True)
    In, Fn = I.numpy(), F.numpy()
    O_ref, B_ref = oracle.conv2d_direct(In, Fn, s, p)
    Ho, Wo = O_ref.shape[2:]
    dI, dF = I.cuda(), F.cuda()

    # the paper's path: transform, then convolution over the im2win tensor
    dW = run_transform(I, Hf, Wf, s, p)
    assert_bitwise_equal(dW, oracle.im2win(In, Hf, Wf, s, p))
    dO = run_conv(dW, F, N, Ci, Hi, Wi, s, p)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)

    # workspace-free variant: same strips, same summation order -> same bits (where the two-call path
    # takes the two-stage generic kernel, which has no workspace-free form, the K blocks differ)
    dO2 = torch.full_like(dO, POISON)
    im2win.conv2d_im2win_implicit_fwd(dI, dF, dO2, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    assert_conv_close(dO2.cpu().numpy(), O_ref, B_ref)
    if not im2win.conv2d_im2win_fwd_launch_info(*shape)["kernel"].startswith("conv_mfma_pipe_kernel"):
        assert torch.equal(dO.view(torch.int32), dO2.view(torch.int32))

    # baselines
    dO3 = torch.full_like(dO, POISON)
    im2win.conv2d_direct_fwd(dI, dF, dO3, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    col = torch.full((N * Ho * Wo * Ci * Hf * Wf,), POISON, dtype=torch.float32, device="cuda")
    dO4 = torch.full_like(dO, POISON)
    im2win.im2col_transform(dI, col, N, Ci, Hi, Wi, Hf, Wf, s, p)
    im2win.conv2d_im2col_fwd(col, dF, dO4, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    assert_conv_close(dO3.cpu().numpy(), O_ref, B_ref)
    assert_conv_close(dO4.cpu().numpy(), O_ref, B_ref)


def _leftover_shapes(seed, count):
    """3x3 and 5x5 multi-channel layers with 150 to 700 tiles: every way the pipelined kernel
    cuts the tiles left after the last full round of 256 (sixteenths, halves, both, none)."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        Hf = Wf = int(rng.choice([3, 3, 3, 5]))
        Ci = int(rng.choice([8, 16, 24, 32, 48, 64])) if Hf == 3 else int(rng.choice([4, 8, 12, 16]))
        s = int(rng.choice([1, 1, 2]))
        p = int(rng.integers(0, 3))
        Hi, Wi = int(rng.integers(20, 90)), int(rng.integers(20, 90))
        Co = int(rng.choice([24, 64, 64, 100, 128]))
        Ho, Wo = (Hi + 2 * p - Hf) // s + 1, (Wi + 2 * p - Wf) // s + 1
        if Ho < 1 or Wo < 1:
            continue
        want = int(rng.integers(150, 700))                      # tiles
        N = max(1, round(want * 64 / ((Co + 63) // 64) / (Ho * Wo)))
        tiles = ((N * Ho * Wo + 63) // 64) * ((Co + 63) // 64)
        if not 150 <= tiles <= 700 or N * Co * Ho * Wo * Ci * Hf * Wf > 8e8:
            continue
        out.append((N, Ci, Hi, Wi, Co, Hf, Wf, s, p))
    return out


LEFTOVER_SHAPES = _leftover_shapes(20230615, 20)


@pytest.mark.parametrize("shape", LEFTOVER_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_random_shape_leftover_tiles(shape):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = workloads.random_layer_inputs(4100 + sum(shape), N, Ci, Hi, Wi, Co, Hf, Wf)
    print("random leftover shape", shape, flush=True)
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), s, p)
    dW = run_transform(I, Hf, Wf, s, p)
    dO = run_conv(dW, F, N, Ci, Hi, Wi, s, p)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)
    dO2 = torch.full_like(dO, POISON)
    im2win.conv2d_im2win_implicit_fwd(I.cuda(), F.cuda(), dO2, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    assert torch.equal(dO.view(torch.int32), dO2.view(torch.int32))


def _other_filter_shapes(seed, count):
    """Row, column, 2x2, 4x4 and 1x1 filters with enough channels for their instances of the pipelined
    kernel (and the 1x1 kernel), strides 1 to 3, paddings up to the filter's reach, ragged channel counts."""
    rng = np.random.default_rng(seed)
    filters = [(1, 7), (7, 1), (1, 3), (3, 1), (2, 2), (4, 4), (1, 1), (5, 5)]
    out = []
    while len(out) < count:
        Hf, Wf = filters[int(rng.integers(0, len(filters)))]
        Ci = int(rng.choice([8, 16, 17, 24, 32, 40, 64, 72]))
        s = int(rng.choice([1, 1, 2, 2, 3]))
        p = 0 if Hf == Wf == 1 else int(rng.integers(0, min(Hf, Wf) + 1))
        Hi, Wi = int(rng.integers(max(Hf, 2), 40)), int(rng.integers(max(Wf, 2), 80))
        Co = int(rng.choice([8, 20, 36, 64, 64, 72, 100, 128]))
        N = int(rng.integers(1, 12))
        Ho, Wo = (Hi + 2 * p - Hf) // s + 1, (Wi + 2 * p - Wf) // s + 1
        if Ho < 1 or Wo < 1 or N * Co * Ho * Wo * Ci * Hf * Wf > 6e8:
            continue
        out.append((N, Ci, Hi, Wi, Co, Hf, Wf, s, p))
    return out


OTHER_FILTER_SHAPES = _other_filter_shapes(20230616, 40)


@pytest.mark.parametrize("shape", OTHER_FILTER_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_random_shape_other_filters(shape):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = workloads.random_layer_inputs(4200 + sum(shape), N, Ci, Hi, Wi, Co, Hf, Wf)
    name = im2win.conv2d_im2win_fwd_launch_info(*shape)["kernel"]
    print("random other-filter shape", shape, name, flush=True)
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), s, p)
    dW = run_transform(I, Hf, Wf, s, p)
    assert_bitwise_equal(dW, oracle.im2win(I.numpy(), Hf, Wf, s, p))
    dO = run_conv(dW, F, N, Ci, Hi, Wi, s, p)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)
    dO2 = torch.full_like(dO, POISON)
    im2win.conv2d_im2win_implicit_fwd(I.cuda(), F.cuda(), dO2, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    assert_conv_close(dO2.cpu().numpy(), O_ref, B_ref)
    if not name.startswith("conv_mfma_pipe_kernel"):
        assert torch.equal(dO.view(torch.int32), dO2.view(torch.int32))
