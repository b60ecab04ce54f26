"""GPU tests of the comparison baselines (direct convolution; im2col + GEMM)
against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2306_14316_amd as im2win
from paper_2306_14316_amd import workloads
from parity_util import POISON, assert_conv_close

pytestmark = pytest.mark.gpu

# (N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
SHAPES = [
    (1, 1, 5, 5, 1, 3, 3, 1, 0),
    (2, 3, 7, 9, 4, 3, 2, 1, 0),       # K = 18: not a multiple of four (scalar accesses)
    (1, 2, 11, 13, 3, 5, 3, 3, 3),     # pad as large as the filter allows
    (3, 4, 12, 10, 2, 4, 1, 4, 0),     # K = 16, stride wider than the filter
    (5, 8, 9, 9, 65, 3, 3, 1, 1),      # K = 72; Co one past a tile; ragged last pixel tile
    (2, 20, 10, 17, 33, 3, 3, 1, 1),   # K = 180 = 5.6 K blocks
    (70, 4, 3, 3, 8, 3, 3, 1, 0),      # one pixel per image
    (1, 3, 40, 40, 16, 7, 7, 2, 3),    # K = 147
    (2, 3, 35, 35, 96, 11, 11, 4, 0),  # K = 363
    (1, 16, 20, 20, 130, 2, 2, 1, 0),  # K = 64 exactly two K blocks; three M tiles
]


def _outputs(shape):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = workloads.random_layer_inputs(6000 + sum(shape), N, Ci, Hi, Wi, Co, Hf, Wf)
    Ho, Wo = im2win.im2win_out_shape(Hi, Wi, Hf, Wf, s, p)
    dO = torch.full((N, Co, Ho, Wo), POISON, dtype=torch.float32, device="cuda")
    return I, F, Ho, Wo, dO


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_direct_convolution(shape):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F, Ho, Wo, dO = _outputs(shape)
    print("direct", shape, flush=True)
    im2win.conv2d_direct_fwd(I.cuda(), F.cuda(), dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), s, p)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_im2col_then_gemm(shape):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F, Ho, Wo, dO = _outputs(shape)
    print("im2col+gemm", shape, flush=True)
    K = Ci * Hf * Wf
    buf = torch.full((N * Ho * Wo * K + 8,), POISON, dtype=torch.float32, device="cuda")
    col = buf[4:4 + N * Ho * Wo * K]             # 16-byte aligned, guard words on both sides
    im2win.im2col_transform(I.cuda(), col, N, Ci, Hi, Wi, Hf, Wf, s, p)
    torch.cuda.synchronize()
    assert torch.isnan(buf[:4]).all() and torch.isnan(buf[4 + N * Ho * Wo * K:]).all()
    got = col.cpu().numpy().reshape(N, Ho * Wo, K)
    for i in range(N):   # the oracle's matrix holds the same fp32 values, widened to fp64
        want = oracle.im2col(I[i].numpy(), Hf, Wf, s, p).astype(np.float32)
        assert np.array_equal(got[i].view(np.uint32), want.view(np.uint32)), "im2col matrix of image %d" % i
    im2win.conv2d_im2col_fwd(col, F.cuda(), dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), s, p)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)


def test_im2col_unaligned_buffers():
    """Buffers that are only 4-byte aligned take the scalar paths."""
    shape = (2, 8, 10, 10, 20, 3, 3, 1, 1)    # K = 72, a multiple of four
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F, Ho, Wo, dO = _outputs(shape)
    K = Ci * Hf * Wf
    buf = torch.full((N * Ho * Wo * K + 8,), POISON, dtype=torch.float32, device="cuda")
    col = buf[1:1 + N * Ho * Wo * K]
    fbuf = torch.empty(F.numel() + 1, dtype=torch.float32, device="cuda")
    dF = fbuf[1:]
    dF.copy_(F.reshape(-1))
    im2win.im2col_transform(I.cuda(), col, N, Ci, Hi, Wi, Hf, Wf, s, p)
    im2win.conv2d_im2col_fwd(col, dF, dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    assert torch.isnan(buf[0]) and torch.isnan(buf[1 + N * Ho * Wo * K:]).all()
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), s, p)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)


def test_baselines_on_headline_layer_small_batch():
    """The headline 3x3 layer at batch 2: all three routes agree with the oracle."""
    L = workloads.with_batch(workloads.layer(2), 2)
    I, F = workloads.make_inputs(L)
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = L.dims
    O_ref, B_ref = oracle.conv2d_direct(I.numpy(), F.numpy(), s, p)
    dI, dF = I.cuda(), F.cuda()
    Ho, Wo = oracle.out_shape(Hi, Wi, Hf, Wf, s, p)
    dO = torch.full((N, Co, Ho, Wo), POISON, dtype=torch.float32, device="cuda")
    im2win.conv2d_direct_fwd(dI, dF, dO, *L.dims)
    torch.cuda.synchronize()
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)
    col = torch.full((N * Ho * Wo * Ci * Hf * Wf,), POISON, dtype=torch.float32, device="cuda")
    dO.fill_(POISON)
    im2win.im2col_transform(dI, col, N, Ci, Hi, Wi, Hf, Wf, s, p)
    im2win.conv2d_im2col_fwd(col, dF, dO, *L.dims)
    torch.cuda.synchronize()
    assert col.numel() * 4 == im2win.im2col_footprint_bytes(N, Ci, Hi, Wi, Hf, Wf, s, p)
    assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)
