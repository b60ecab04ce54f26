/*
 * CPU oracle for the im2win window-order convolution (arXiv 2306.14316).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path and nothing in the product path may call it.
 *
 * Every routine is the definition written out, in the paper's notation:
 *   I[Ni][Ci][Hi][Wi]  input,  F[Co][Ci][Hf][Wf]  filter,
 *   O[Ni][Co][Ho][Wo]  output, all NCHW (Section 2.1), one stride s for both
 *   axes.  Zero padding p (not in the paper, whose Table 2 layers are all
 *   unpadded) is added on all four sides: Ipad(i,r,h,w) = I(i,r,h-p,w-p) when
 *   that index is inside the image and 0 otherwise.
 *
 * Floating point: inputs are fp32; every product and every running sum is
 * taken in fp64 and the result is returned in fp64.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_pins.py
 * (library cross-correlation, closed forms, the paper's Fig. 1 counts and
 * Table 2 sizes, structural invariants).  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Output extent along one axis: floor((in + 2p - f) / s) + 1 (Table 2 fixes the
 * floor: 224 wide, 7 wide filter, stride 2 gives 109).  Returns -1 when the
 * filter does not fit or an argument is out of range. */
int oracle_out_dim(int in, int f, int s, int p)
{
    if (in <= 0 || f <= 0 || s <= 0 || p < 0) return -1;
    int span = in + 2 * p - f;
    if (span < 0) return -1;
    return span / s + 1;
}

/* Number of elements of the im2win tensor, (Ni, Ci, Ho, Wp*Hf) with Wp = Wi+2p
 * (Section 3.1: size (Ni, Ci, Ho, Wi x Hf)). */
int64_t oracle_im2win_elems(int N, int Ci, int Hi, int Wi, int Hf, int Wf, int s, int p)
{
    int Ho = oracle_out_dim(Hi, Hf, s, p);
    int Wo = oracle_out_dim(Wi, Wf, s, p);
    if (Ho < 0 || Wo < 0 || N <= 0 || Ci <= 0) return -1;
    return (int64_t)N * Ci * Ho * ((int64_t)(Wi + 2 * p) * Hf);
}

/* Number of elements of the im2col matrices of all images: each image gives a
 * (Ho*Wo) x (Ci*Hf*Wf) matrix (Section 2.3). */
int64_t oracle_im2col_elems(int N, int Ci, int Hi, int Wi, int Hf, int Wf, int s, int p)
{
    int Ho = oracle_out_dim(Hi, Hf, s, p);
    int Wo = oracle_out_dim(Wi, Wf, s, p);
    if (Ho < 0 || Wo < 0 || N <= 0 || Ci <= 0) return -1;
    return (int64_t)N * Ho * Wo * ((int64_t)Ci * Hf * Wf);
}

/* Padded-input read, as raw 32-bit words so that a copy never touches the
 * value (NaN payloads, -0.0 and denormals survive); padding is +0.0. */
static inline uint32_t ipad_bits(const uint32_t *I, int Ci, int Hi, int Wi,
                                 int i, int r, int h, int w, int p)
{
    int hh = h - p, ww = w - p;
    if (hh < 0 || hh >= Hi || ww < 0 || ww >= Wi) return 0u;
    return I[(((size_t)i * Ci + r) * Hi + hh) * Wi + ww];
}

static inline double ipad_val(const float *I, int Ci, int Hi, int Wi,
                              int i, int r, int h, int w, int p)
{
    int hh = h - p, ww = w - p;
    if (hh < 0 || hh >= Hi || ww < 0 || ww >= Wi) return 0.0;
    return (double)I[(((size_t)i * Ci + r) * Hi + hh) * Wi + ww];
}

/*
 * Direct convolution, Eq. 1 (Section 2.1) read as a cross-correlation:
 *   O(i,j,m,n) = sum_r sum_u sum_v Ipad(i,r,m*s+u,n*s+v) * F(j,r,u,v)
 * as the seven nested loops of Section 2.2 (outer four over O, inner three
 * over F and I).  Bnd, when not NULL, receives sum |Ipad|*|F| over the same
 * terms: the scale of the per-element error bound.
 */
int oracle_conv2d_direct(const float *I, const float *F,
                         int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf,
                         int s, int p, double *O, double *Bnd)
{
    int Ho = oracle_out_dim(Hi, Hf, s, p);
    int Wo = oracle_out_dim(Wi, Wf, s, p);
    if (Ho < 0 || Wo < 0 || N <= 0 || Ci <= 0 || Co <= 0) return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < Co; ++j)
            for (int m = 0; m < Ho; ++m)
                for (int n = 0; n < Wo; ++n) {
                    double acc = 0.0, bnd = 0.0;
                    for (int r = 0; r < Ci; ++r)
                        for (int u = 0; u < Hf; ++u)
                            for (int v = 0; v < Wf; ++v) {
                                double x = ipad_val(I, Ci, Hi, Wi, i, r, m * s + u, n * s + v, p);
                                double w = (double)F[(((size_t)j * Ci + r) * Hf + u) * Wf + v];
                                acc += x * w;
                                bnd += fabs(x) * fabs(w);
                            }
                    size_t o = (((size_t)i * Co + j) * Ho + m) * Wo + n;
                    O[o] = acc;
                    if (Bnd) Bnd[o] = bnd;
                }
    return 0;
}

/* The same definition evaluated one output element at a time, for sampled
 * checks at sizes where the full seven-loop pass is too slow.  idx holds
 * count quadruples (i,j,m,n). */
int oracle_conv2d_direct_at(const float *I, const float *F,
                            int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf,
                            int s, int p, const int32_t *idx, int64_t count,
                            double *O, double *Bnd)
{
    int Ho = oracle_out_dim(Hi, Hf, s, p);
    int Wo = oracle_out_dim(Wi, Wf, s, p);
    if (Ho < 0 || Wo < 0 || N <= 0 || Ci <= 0 || Co <= 0) return -1;
    for (int64_t q = 0; q < count; ++q) {
        int i = idx[4 * q], j = idx[4 * q + 1], m = idx[4 * q + 2], n = idx[4 * q + 3];
        if (i < 0 || i >= N || j < 0 || j >= Co || m < 0 || m >= Ho || n < 0 || n >= Wo) return -2;
    }
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < count; ++q) {
        int i = idx[4 * q], j = idx[4 * q + 1], m = idx[4 * q + 2], n = idx[4 * q + 3];
        double acc = 0.0, bnd = 0.0;
        for (int r = 0; r < Ci; ++r)
            for (int u = 0; u < Hf; ++u)
                for (int v = 0; v < Wf; ++v) {
                    double x = ipad_val(I, Ci, Hi, Wi, i, r, m * s + u, n * s + v, p);
                    double w = (double)F[(((size_t)j * Ci + r) * Hf + u) * Wf + v];
                    acc += x * w;
                    bnd += fabs(x) * fabs(w);
                }
        O[q] = acc;
        if (Bnd) Bnd[q] = bnd;
    }
    return 0;
}

/*
 * im2win data transformation, Eq. 2 (Section 3.1).  The printed equation is
 * for s = 1 and leaves k unexplained; the reading taken here is that k is the
 * (padded) input column and u the row inside the window, so that
 *   What(i, r, m, k*Hf + u) = Ipad(i, r, m*s + u, k),  0<=k<Wp, 0<=u<Hf,
 * which gives the stated size (Ni, Ci, Ho, Wi x Hf) and puts the Wo windows
 * of output row m side by side, each one contiguous (column after column).
 * Values are copied as 32-bit words.
 */
int oracle_im2win(const float *I, float *What,
                  int N, int Ci, int Hi, int Wi, int Hf, int Wf, int s, int p)
{
    int Ho = oracle_out_dim(Hi, Hf, s, p);
    int Wo = oracle_out_dim(Wi, Wf, s, p);
    if (Ho < 0 || Wo < 0 || N <= 0 || Ci <= 0) return -1;
    const uint32_t *src = (const uint32_t *)I;
    uint32_t *dst = (uint32_t *)What;
    int Wp = Wi + 2 * p;
#pragma omp parallel for collapse(2) schedule(static)
    for (int i = 0; i < N; ++i)
        for (int r = 0; r < Ci; ++r)
            for (int m = 0; m < Ho; ++m)
                for (int k = 0; k < Wp; ++k)
                    for (int u = 0; u < Hf; ++u)
                        dst[((((size_t)i * Ci + r) * Ho + m) * Wp + k) * Hf + u] =
                            ipad_bits(src, Ci, Hi, Wi, i, r, m * s + u, k, p);
    return 0;
}

/*
 * im2col matrix of ONE image I' (Section 2.3), with the stride and padding
 * written in:  M(m*Wo + n, (r*Hf + u)*Wf + v) = I'pad(r, m*s + u, n*s + v).
 * M is (Ho*Wo) x (Ci*Hf*Wf), row-major, fp64.
 */
int oracle_im2col(const float *Iimg, double *M,
                  int Ci, int Hi, int Wi, int Hf, int Wf, int s, int p)
{
    int Ho = oracle_out_dim(Hi, Hf, s, p);
    int Wo = oracle_out_dim(Wi, Wf, s, p);
    if (Ho < 0 || Wo < 0 || Ci <= 0) return -1;
    size_t K = (size_t)Ci * Hf * Wf;
    for (int m = 0; m < Ho; ++m)
        for (int n = 0; n < Wo; ++n)
            for (int r = 0; r < Ci; ++r)
                for (int u = 0; u < Hf; ++u)
                    for (int v = 0; v < Wf; ++v)
                        M[((size_t)m * Wo + n) * K + ((size_t)r * Hf + u) * Wf + v] =
                            ipad_val(Iimg, Ci, Hi, Wi, 0, r, m * s + u, n * s + v, p);
    return 0;
}

/*
 * GEMM-based convolution (Section 2.3): per image, M as above, filter matrix
 * Nf((r*Hf+u)*Wf+v, j) = F(j,r,u,v), R' = M x Nf, R(j,m,n) = R'(m*Wo+n, j).
 * A second, differently structured route to the same numbers.
 */
int oracle_conv2d_im2col_gemm(const float *I, const float *F,
                              int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf,
                              int s, int p, double *O)
{
    int Ho = oracle_out_dim(Hi, Hf, s, p);
    int Wo = oracle_out_dim(Wi, Wf, s, p);
    if (Ho < 0 || Wo < 0 || N <= 0 || Ci <= 0 || Co <= 0) return -1;
    size_t K = (size_t)Ci * Hf * Wf, P = (size_t)Ho * Wo;
    double *M = (double *)malloc(P * K * sizeof(double));
    double *Nf = (double *)malloc(K * Co * sizeof(double));
    double *R = (double *)malloc(P * Co * sizeof(double));
    if (!M || !Nf || !R) { free(M); free(Nf); free(R); return -3; }
    for (int j = 0; j < Co; ++j)
        for (int r = 0; r < Ci; ++r)
            for (int u = 0; u < Hf; ++u)
                for (int v = 0; v < Wf; ++v)
                    Nf[(((size_t)r * Hf + u) * Wf + v) * Co + j] =
                        (double)F[(((size_t)j * Ci + r) * Hf + u) * Wf + v];
    for (int i = 0; i < N; ++i) {
        oracle_im2col(I + (size_t)i * Ci * Hi * Wi, M, Ci, Hi, Wi, Hf, Wf, s, p);
        for (size_t a = 0; a < P; ++a)
            for (int j = 0; j < Co; ++j) {
                double acc = 0.0;
                for (size_t k = 0; k < K; ++k) acc += M[a * K + k] * Nf[k * Co + j];
                R[a * Co + j] = acc;
            }
        for (int j = 0; j < Co; ++j)
            for (int m = 0; m < Ho; ++m)
                for (int n = 0; n < Wo; ++n)
                    O[(((size_t)i * Co + j) * Ho + m) * Wo + n] = R[((size_t)m * Wo + n) * Co + j];
    }
    free(M); free(Nf); free(R);
    return 0;
}

/*
 * Convolution read off the im2win tensor (Section 3.1-3.2).  The property the
 * method rests on: for output pixel (i, m, n) and channel r, the Hf x Wf patch
 * of the padded input is ONE contiguous run of What, Hf*Wf floats long, that
 * starts at column n*s*Hf of row What[i][r][m][.] and holds the patch column
 * after column (element v*Hf + u is patch row u, patch column v).  Each output
 * is therefore the sum, over the channels, of the dot product of that run with
 * the channel's filter taps taken in the same column-major order.  Plain nested
 * loops over the output and over (r, v, u); no flattened-index decoding.  A
 * differently structured third route to Eq. 1's numbers: it pins the element
 * order inside a row of What and the way the convolution must index it.
 */
int oracle_conv2d_over_im2win(const float *What, const float *F,
                              int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf,
                              int s, int p, double *O)
{
    int Ho = oracle_out_dim(Hi, Hf, s, p);
    int Wo = oracle_out_dim(Wi, Wf, s, p);
    if (Ho < 0 || Wo < 0 || N <= 0 || Ci <= 0 || Co <= 0) return -1;
    size_t rowlen = (size_t)(Wi + 2 * p) * Hf;   /* floats in one row of What */
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < Co; ++j)
            for (int m = 0; m < Ho; ++m)
                for (int n = 0; n < Wo; ++n) {
                    double acc = 0.0;
                    for (int r = 0; r < Ci; ++r) {
                        const float *row = What + (((size_t)i * Ci + r) * Ho + m) * rowlen;
                        const float *window = row + (size_t)n * s * Hf;   /* contiguous Hf*Wf floats */
                        const float *taps = F + ((size_t)j * Ci + r) * Hf * Wf;
                        for (int v = 0; v < Wf; ++v)
                            for (int u = 0; u < Hf; ++u)
                                acc += (double)window[v * Hf + u] * (double)taps[u * Wf + v];
                    }
                    O[(((size_t)i * Co + j) * Ho + m) * Wo + n] = acc;
                }
    return 0;
}
