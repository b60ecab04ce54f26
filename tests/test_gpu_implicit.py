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
    dW = torch.empty((N, Ci, L.Ho, L.Wp * Hf), dtype=torch.float32, device="cuda")
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


def test_implicit_rejects_layers_it_does_not_take():
    for shape in [(1, 3, 32, 32, 16, 3, 3, 1, 0), (1, 8, 16, 16, 8, 3, 2, 1, 0), (1, 8, 40, 40, 8, 11, 11, 4, 0)]:
        N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
        I, F = workloads.random_layer_inputs(3, N, Ci, Hi, Wi, Co, Hf, Wf)
        Ho, Wo = im2win.im2win_out_shape(Hi, Wi, Hf, Wf, s, p)
        dO = torch.full((N, Co, Ho, Wo), POISON, dtype=torch.float32, device="cuda")
        with pytest.raises(im2win.Im2winError) as e:
            im2win.conv2d_im2win_implicit_fwd(I.cuda(), F.cuda(), dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
        assert e.value.status == -4
        torch.cuda.synchronize()
        assert torch.isnan(dO).all()      # nothing was launched
