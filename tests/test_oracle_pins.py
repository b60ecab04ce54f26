"""Pins for the CPU oracle: each check ties an oracle routine to something other
than itself -- numbers the paper prints (Fig. 1 counts, Table 2 sizes), library
routines (scipy's 2-D cross-correlation, torch's fp64 conv2d, numpy matmul and
transpose), closed forms and structural invariants of the im2win layout.
CPU only; tiny shapes.
"""
import itertools
import os

import numpy as np
import pytest
import scipy.signal
import torch

import oracle

RNG = np.random.default_rng(20230614)

# (N, Ci, Hi, Wi, Co, Hf, Wf, s, p): asymmetric filters, strides 1-4, pads 0-3,
# a filter as tall as the padded input, Ci = 1 and odd channel counts.
TINY_SHAPES = [
    (1, 1, 5, 5, 1, 3, 3, 1, 0),
    (2, 3, 7, 9, 4, 3, 2, 1, 0),
    (2, 3, 9, 7, 5, 2, 3, 2, 1),
    (1, 2, 11, 13, 3, 5, 3, 3, 3),
    (3, 4, 12, 10, 2, 4, 1, 4, 0),
    (1, 5, 6, 8, 3, 6, 2, 1, 0),    # Hf == Hi  -> Ho == 1
    (2, 2, 6, 6, 3, 8, 8, 1, 1),    # filter == padded input -> 1x1 output
    (1, 3, 10, 10, 6, 1, 1, 2, 0),  # 1x1 strided
    (2, 6, 8, 8, 7, 3, 3, 2, 1),
]


def rand_pair(N, Ci, Hi, Wi, Co, Hf, Wf):
    I = RNG.uniform(-1, 1, size=(N, Ci, Hi, Wi)).astype(np.float32)
    F = RNG.uniform(-1, 1, size=(Co, Ci, Hf, Wf)).astype(np.float32)
    return I, F


def pad_np(I, p):
    return np.pad(I, ((0, 0), (0, 0), (p, p), (p, p)))


# --------------------------------------------------------------------------- #
# numbers the paper prints
# --------------------------------------------------------------------------- #
def _rows(path):
    with open(path) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_fig1_element_counts(golden_dir):
    (row,) = _rows(os.path.join(golden_dir, "fig1_counts.txt"))
    N, Ci, Hi, Wi, Hf, Wf, s, p, n_col, n_win = map(int, row)
    assert oracle.im2col_elems(N, Ci, Hi, Wi, Hf, Wf, s, p) == n_col == 48
    assert oracle.im2win_elems(N, Ci, Hi, Wi, Hf, Wf, s, p) == n_win == 36
    I = RNG.uniform(-1, 1, size=(N, Ci, Hi, Wi)).astype(np.float32)
    assert oracle.im2win(I, Hf, Wf, s, p).size == n_win
    assert oracle.im2col(I[0], Hf, Wf, s, p).size == n_col


def test_table2_output_sizes(golden_dir):
    rows = _rows(os.path.join(golden_dir, "table2_layers.txt"))
    assert len(rows) == 12
    for name, *vals in rows:
        Ci, Hi, Wi, Co, Hf, Wf, s, Ho, Wo = map(int, vals)
        assert oracle.out_shape(Hi, Wi, Hf, Wf, s, 0) == (Ho, Wo), name


def test_out_dim_rejects_bad_arguments():
    assert oracle.out_dim(5, 6, 1, 0) == -1      # filter larger than input
    assert oracle.out_dim(5, 6, 1, 1) == 2       # ... but fits once padded
    assert oracle.out_dim(5, 3, 0, 0) == -1
    assert oracle.out_dim(5, 3, 1, -1) == -1
    assert oracle.out_dim(0, 1, 1, 0) == -1


# --------------------------------------------------------------------------- #
# direct convolution against library routines
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("shape", TINY_SHAPES)
def test_direct_matches_scipy_correlate2d(shape):
    """Unit stride is a textbook 'valid' 2-D cross-correlation per channel pair;
    a stride subsamples it."""
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = rand_pair(N, Ci, Hi, Wi, Co, Hf, Wf)
    O, _ = oracle.conv2d_direct(I, F, s, p)
    Ip = pad_np(I, p).astype(np.float64)
    ref = np.zeros_like(O)
    for i, j in itertools.product(range(N), range(Co)):
        full = sum(scipy.signal.correlate2d(Ip[i, r], F[j, r].astype(np.float64), mode="valid")
                   for r in range(Ci))
        ref[i, j] = full[::s, ::s]
    assert O.shape == ref.shape
    np.testing.assert_allclose(O, ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("shape", TINY_SHAPES)
def test_direct_and_bound_match_torch_fp64(shape):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = rand_pair(N, Ci, Hi, Wi, Co, Hf, Wf)
    O, B = oracle.conv2d_direct(I, F, s, p)
    tI, tF = torch.from_numpy(I).double(), torch.from_numpy(F).double()
    ref = torch.nn.functional.conv2d(tI, tF, stride=s, padding=p).numpy()
    refB = torch.nn.functional.conv2d(tI.abs(), tF.abs(), stride=s, padding=p).numpy()
    np.testing.assert_allclose(O, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(B, refB, rtol=0, atol=1e-12)
    assert np.all(np.abs(O) <= B + 1e-12)


def test_sampled_outputs_equal_full_pass():
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = 2, 3, 9, 11, 4, 3, 5, 2, 2
    I, F = rand_pair(N, Ci, Hi, Wi, Co, Hf, Wf)
    O, B = oracle.conv2d_direct(I, F, s, p)
    idx = np.array(list(itertools.product(*[range(d) for d in O.shape])), dtype=np.int32)
    Os, Bs = oracle.conv2d_direct_at(I, F, s, p, idx)
    assert np.array_equal(Os, O.reshape(-1))
    assert np.array_equal(Bs, B.reshape(-1))
    with pytest.raises(ValueError):
        oracle.conv2d_direct_at(I, F, s, p, np.array([[0, 0, O.shape[2], 0]]))


def test_delta_filter_reproduces_strided_shifted_input():
    """F = one-hot at (r0,u0,v0): the output is the padded input sampled at
    (m*s+u0, n*s+v0) -- exact, and fixes stride, padding offset and no flip."""
    N, Ci, Hi, Wi, Co, Hf, Wf = 2, 3, 9, 8, 4, 3, 4
    I = RNG.uniform(-1, 1, size=(N, Ci, Hi, Wi)).astype(np.float32)
    for s, p in [(1, 0), (2, 1), (3, 2)]:
        Ho, Wo = oracle.out_shape(Hi, Wi, Hf, Wf, s, p)
        Ip = pad_np(I, p)
        for (r0, u0, v0) in [(0, 0, 0), (2, 2, 3), (1, 0, 3), (1, 2, 0)]:
            F = np.zeros((Co, Ci, Hf, Wf), dtype=np.float32)
            F[1, r0, u0, v0] = 1.0
            O, _ = oracle.conv2d_direct(I, F, s, p)
            want = Ip[:, r0, u0:u0 + (Ho - 1) * s + 1:s, v0:v0 + (Wo - 1) * s + 1:s]
            assert np.array_equal(O[:, 1], want.astype(np.float64))
            assert not O[:, [0, 2, 3]].any()


def test_one_by_one_filter_is_a_gemm():
    N, Ci, Hi, Wi, Co = 2, 5, 6, 7, 4
    I, F = rand_pair(N, Ci, Hi, Wi, Co, 1, 1)
    for s in (1, 2, 3):
        O, _ = oracle.conv2d_direct(I, F, s, 0)
        X = I[:, :, ::s, ::s].astype(np.float64)
        ref = np.matmul(F[:, :, 0, 0].astype(np.float64)[None], X.reshape(N, Ci, -1)).reshape(O.shape)
        np.testing.assert_allclose(O, ref, rtol=0, atol=1e-13)


def test_linearity_in_input_and_filter():
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = 2, 3, 8, 9, 3, 3, 2, 2, 1
    # dyadic values: every combination below is exact in fp32 and fp64
    def dy(shape):
        return (RNG.integers(-8, 9, size=shape) / 8.0).astype(np.float32)
    I1, I2 = dy((N, Ci, Hi, Wi)), dy((N, Ci, Hi, Wi))
    F1, F2 = dy((Co, Ci, Hf, Wf)), dy((Co, Ci, Hf, Wf))
    a, b = 2.0, -0.5
    c = lambda I, F: oracle.conv2d_direct(I, F, s, p)[0]
    assert np.array_equal(c((a * I1 + b * I2).astype(np.float32), F1), a * c(I1, F1) + b * c(I2, F1))
    assert np.array_equal(c(I1, (a * F1 + b * F2).astype(np.float32)), a * c(I1, F1) + b * c(I1, F2))


def test_all_ones_counts_unpadded_taps():
    """I = 1, F = 1: each output counts the taps that fall inside the image."""
    N, Ci, Hi, Wi, Co, Hf, Wf = 1, 3, 7, 6, 2, 3, 4
    for s, p in [(1, 0), (1, 2), (2, 3), (3, 1)]:
        I = np.ones((N, Ci, Hi, Wi), dtype=np.float32)
        F = np.ones((Co, Ci, Hf, Wf), dtype=np.float32)
        O, B = oracle.conv2d_direct(I, F, s, p)
        Ho, Wo = oracle.out_shape(Hi, Wi, Hf, Wf, s, p)
        rows = np.array([sum(0 <= m * s + u - p < Hi for u in range(Hf)) for m in range(Ho)])
        cols = np.array([sum(0 <= n * s + v - p < Wi for v in range(Wf)) for n in range(Wo)])
        want = Ci * rows[:, None] * cols[None, :]
        assert np.array_equal(O[0, 0], want.astype(np.float64))
        assert np.array_equal(O, B)


# --------------------------------------------------------------------------- #
# the other routes of the paper agree with the definition
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("shape", TINY_SHAPES)
def test_im2col_gemm_route_agrees(shape):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = rand_pair(N, Ci, Hi, Wi, Co, Hf, Wf)
    O, _ = oracle.conv2d_direct(I, F, s, p)
    np.testing.assert_allclose(oracle.conv2d_im2col_gemm(I, F, s, p), O, rtol=0, atol=1e-12)


@pytest.mark.parametrize("shape", TINY_SHAPES)
def test_im2col_matrix_rows_are_flattened_windows(shape):
    """Library check of the im2col matrix: numpy's sliding windows, flattened
    (r,u,v) with v fastest, one row per output pixel in (m,n) order."""
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, _ = rand_pair(N, Ci, Hi, Wi, Co, Hf, Wf)
    Ip = pad_np(I, p)[0]
    win = np.lib.stride_tricks.sliding_window_view(Ip, (Hf, Wf), axis=(1, 2))[:, ::s, ::s]
    ref = win.transpose(1, 2, 0, 3, 4).reshape(win.shape[1] * win.shape[2], Ci * Hf * Wf)
    assert np.array_equal(oracle.im2col(I[0], Hf, Wf, s, p), ref.astype(np.float64))


@pytest.mark.parametrize("shape", TINY_SHAPES)
def test_convolution_over_im2win_agrees(shape):
    """Dot products over the contiguous windows of the im2win tensor reach the
    definition's result: fixes the element order inside a row of the tensor
    (column after column) and the window start n*s*Hf together."""
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, F = rand_pair(N, Ci, Hi, Wi, Co, Hf, Wf)
    O, _ = oracle.conv2d_direct(I, F, s, p)
    W = oracle.im2win(I, Hf, Wf, s, p)
    np.testing.assert_allclose(oracle.conv2d_over_im2win(W, F, Hi, Wi, s, p), O, rtol=0, atol=1e-12)


# --------------------------------------------------------------------------- #
# structure of the im2win tensor
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("shape", TINY_SHAPES)
def test_im2win_windows_are_contiguous_column_major_patches(shape):
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = shape
    I, _ = rand_pair(N, Ci, Hi, Wi, Co, Hf, Wf)
    W = oracle.im2win(I, Hf, Wf, s, p)
    Ho, Wo = oracle.out_shape(Hi, Wi, Hf, Wf, s, p)
    Wp = Wi + 2 * p
    assert W.shape == (N, Ci, Ho, Wp * Hf)
    assert W.size == oracle.im2win_elems(N, Ci, Hi, Wi, Hf, Wf, s, p)
    Ip = pad_np(I, p)
    for i, r, m, n in itertools.product(range(N), range(Ci), range(Ho), range(Wo)):
        run = W[i, r, m, n * s * Hf:n * s * Hf + Hf * Wf]
        patch = Ip[i, r, m * s:m * s + Hf, n * s:n * s + Wf]
        assert np.array_equal(run.reshape(Wf, Hf).T, patch)
    # whole rows: row m of the tensor is the Hf x Wp strip starting at input row m*s, transposed
    for m in range(Ho):
        strip = Ip[:, :, m * s:m * s + Hf, :]                       # [N,Ci,Hf,Wp]
        assert np.array_equal(W[:, :, m, :].reshape(N, Ci, Wp, Hf), strip.transpose(0, 1, 3, 2))


def test_im2win_row_overlap_and_multiplicity():
    N, Ci, Hi, Wi, Hf, Wf, s, p = 1, 2, 10, 7, 4, 3, 2, 1
    I = np.arange(N * Ci * Hi * Wi, dtype=np.float32).reshape(N, Ci, Hi, Wi) + 1.0  # all distinct, non-zero
    W = oracle.im2win(I, Hf, Wf, s, p)
    Ho, _ = oracle.out_shape(Hi, Wi, Hf, Wf, s, p)
    Wp = Wi + 2 * p
    Wv = W.reshape(N, Ci, Ho, Wp, Hf)
    # consecutive rows share the strip rows they both cover
    for m in range(Ho - 1):
        assert np.array_equal(Wv[:, :, m + 1, :, :Hf - s], Wv[:, :, m, :, s:])
    # each input element appears once per (m,u) with m*s+u equal to its padded row
    vals, counts = np.unique(W[W != 0], return_counts=True)
    got = dict(zip(vals.tolist(), counts.tolist()))
    for h in range(Hi):
        mult = sum(1 for m in range(Ho) for u in range(Hf) if m * s + u == h + p)
        for w in range(Wi):
            assert got.get(float(I[0, 0, h, w]), 0) == mult
    # zeros are exactly the padding
    n_pad = sum(1 for m in range(Ho) for u in range(Hf) for k in range(Wp)
                if not (0 <= m * s + u - p < Hi and 0 <= k - p < Wi))
    assert int((W == 0).sum()) == N * Ci * n_pad


def test_im2win_special_cases_reduce_to_copy_and_transpose():
    I = RNG.uniform(-1, 1, size=(2, 3, 5, 6)).astype(np.float32)
    # Hf = 1, s = 1, p = 0: the tensor is the input itself
    assert np.array_equal(oracle.im2win(I, 1, 1, 1, 0), I)
    assert np.array_equal(oracle.im2win(I, 1, 3, 1, 0), I)
    # Hf = Hi, p = 0: one output row whose content is the transposed plane
    W = oracle.im2win(I, 5, 2, 1, 0)
    assert W.shape == (2, 3, 1, 6 * 5)
    assert np.array_equal(W.reshape(2, 3, 6, 5), I.transpose(0, 1, 3, 2))


def test_im2win_copies_bit_patterns():
    bits = np.array([0x7FC00001, 0xFFC12345, 0x7F800001, 0x80000000, 0x00000001, 0x807FFFFF,
                     0x7F800000, 0xFF800000, 0x3F800000], dtype=np.uint32)
    I = np.resize(bits, 2 * 1 * 4 * 5).view(np.float32).reshape(2, 1, 4, 5)
    W = oracle.im2win(I, 2, 2, 1, 1)
    Ho, _ = oracle.out_shape(4, 5, 2, 2, 1, 1)
    Ipb = np.pad(I.view(np.uint32), ((0, 0), (0, 0), (1, 1), (1, 1)))
    Wb = W.view(np.uint32).reshape(2, 1, Ho, 7, 2)
    for m in range(Ho):
        assert np.array_equal(Wb[:, :, m], Ipb[:, :, m:m + 2, :].transpose(0, 1, 3, 2))


def test_footprint_ratio_closed_form():
    for (N, Ci, Hi, Wi, Co, Hf, Wf, s, p) in TINY_SHAPES:
        Ho, Wo = oracle.out_shape(Hi, Wi, Hf, Wf, s, p)
        win = oracle.im2win_elems(N, Ci, Hi, Wi, Hf, Wf, s, p)
        col = oracle.im2col_elems(N, Ci, Hi, Wi, Hf, Wf, s, p)
        assert win == N * Ci * Ho * Hf * (Wi + 2 * p)
        assert col == N * Ho * Wo * Ci * Hf * Wf
        assert win * Wo * Wf == col * (Wi + 2 * p)
