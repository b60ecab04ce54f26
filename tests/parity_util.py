"""Shared helpers for the GPU parity tests: run the library through its C ABI
on device tensors and compare with the CPU oracle."""
import numpy as np
import torch

import oracle
import paper_2306_14316_amd as im2win

# Acceptance bar for the fp32 convolution (fp32 multiply/accumulate on the
# matrix cores, any summation order) against the fp64 oracle:
#   every element: |O_gpu - O_ref| <= 1e-4 * sum|x||w|   and   relative L2 <= 1e-5.
# The expected error is about sqrt(K)*2^-24 relative (3e-6 at K = 2304).
ELEM_TOL = 1e-4
L2_TOL = 1e-5

POISON = float("nan")


def run_transform(I, Hf, Wf, s, p):
    N, Ci, Hi, Wi = I.shape
    Ho, _ = im2win.im2win_out_shape(Hi, Wi, Hf, Wf, s, p)
    dI = I.cuda()
    dW = torch.full((N, Ci, Ho, (Wi + 2 * p) * Hf), POISON, dtype=torch.float32, device="cuda")
    im2win.im2win_transform(dI, dW, N, Ci, Hi, Wi, Hf, Wf, s, p)
    torch.cuda.synchronize()
    return dW


def run_conv(dW, F, N, Ci, Hi, Wi, s, p, basic=False):
    Co, _, Hf, Wf = F.shape
    Ho, Wo = im2win.im2win_out_shape(Hi, Wi, Hf, Wf, s, p)
    dF = F.cuda()
    dO = torch.full((N, Co, Ho, Wo), POISON, dtype=torch.float32, device="cuda")
    fn = im2win.conv2d_im2win_fwd_basic if basic else im2win.conv2d_im2win_fwd
    fn(dW, dF, dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    torch.cuda.synchronize()
    return dO


def assert_bitwise_equal(dW, W_ref):
    got = dW.cpu().numpy().view(np.uint32)
    want = np.ascontiguousarray(W_ref).view(np.uint32)
    assert got.shape == want.shape
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        raise AssertionError("im2win tensor differs at %d of %d words, first at %s"
                             % (len(bad), got.size, bad[0]))


def conv_errors(O_gpu, O_ref, B_ref):
    """(max |err| / sum|x||w|, relative L2 error); O_gpu fp32 array, references fp64."""
    got = np.asarray(O_gpu, dtype=np.float64)
    assert got.shape == O_ref.shape
    assert np.isfinite(got).all(), "output holds NaN/Inf (an element was never written?)"
    err = np.abs(got - O_ref)
    scale = np.where(B_ref > 0, B_ref, 1.0)
    elem = float((err / scale).max())
    # where the bound is zero every term is zero and the output must be exactly zero
    assert not err[B_ref == 0].any()
    l2 = float(np.sqrt((err ** 2).sum()) / max(np.sqrt((O_ref ** 2).sum()), 1e-300))
    return elem, l2


def assert_conv_close(O_gpu, O_ref, B_ref):
    elem, l2 = conv_errors(O_gpu, O_ref, B_ref)
    assert elem <= ELEM_TOL, "max |err|/sum|x||w| = %.3e" % elem
    assert l2 <= L2_TOL, "relative L2 error = %.3e" % l2
    return elem, l2


def check_layer(I, F, s, p, basic=False, twice=True):
    """Transform + convolution of one layer against the oracle; returns the error norms."""
    N, Ci, Hi, Wi = I.shape
    Co, _, Hf, Wf = F.shape
    In, Fn = I.numpy(), F.numpy()
    dW = run_transform(I, Hf, Wf, s, p)
    assert_bitwise_equal(dW, oracle.im2win(In, Hf, Wf, s, p))
    O_ref, B_ref = oracle.conv2d_direct(In, Fn, s, p)
    dO = run_conv(dW, F, N, Ci, Hi, Wi, s, p, basic=basic)
    res = assert_conv_close(dO.cpu().numpy(), O_ref, B_ref)
    if twice:   # a second run must reproduce the first bit for bit (no races on LDS)
        dO2 = run_conv(dW, F, N, Ci, Hi, Wi, s, p, basic=basic)
        assert torch.equal(dO.view(torch.int32), dO2.view(torch.int32))
    return res
