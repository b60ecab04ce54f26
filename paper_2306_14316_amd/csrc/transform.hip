// im2win data transformation (Section 3.1, Eq. 2) for gfx950:
//   What(i, r, m, k*Hf + u) = Ipad(i, r, m*s + u, k),  0<=k<Wp, 0<=u<Hf.
// A pure gather-copy, bound by HBM traffic: the input is read (each row about
// Hf/s times, re-reads served by the caches) and the tensor is written once.
// Values move as 32-bit words, so bit patterns survive; padding is +0.0.
#include "common.h"

namespace im2win {

struct TransformParams {
    const uint32_t *in;
    uint32_t *win;
    int Ci, Hi, Wi, Ho, Hf, s, p, Wp;
    uint32_t rowlen;      // Wp*Hf
    uint32_t total;       // N*Ci*Ho*rowlen
    uint32_t plane_in;    // Hi*Wi
    FastDiv d_rowlen, d_ho, d_hf;
};

// One thread writes VEC consecutive words of the tensor (one 16-byte store
// when VEC == 4).  The first word's coordinates come from three reciprocal
// divisions; the following ones are stepped with carries (u fastest, then the
// column k, then the row m, then the plane).
template <int VEC>
__global__ __launch_bounds__(256) void transform_kernel(TransformParams P)
{
    uint32_t y0 = (blockIdx.x * 256u + threadIdx.x) * VEC;
    if (y0 >= P.total) return;

    uint32_t row = fdiv(y0, P.d_rowlen);          // (i*Ci + r)*Ho + m
    uint32_t x = y0 - row * P.rowlen;             // k*Hf + u
    uint32_t plane = fdiv(row, P.d_ho);           // i*Ci + r
    int m = (int)(row - plane * (uint32_t)P.Ho);
    int k = (int)fdiv(x, P.d_hf);
    int u = (int)(x - (uint32_t)k * (uint32_t)P.Hf);
    const uint32_t *src = P.in + (size_t)plane * P.plane_in;

    uint32_t v[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        int h = m * P.s + u - P.p;
        int w = k - P.p;
        bool inside = (h >= 0) & (h < P.Hi) & (w >= 0) & (w < P.Wi) & (y0 + e < P.total);
        v[e] = inside ? src[h * P.Wi + w] : 0u;
        // step to the next word of the tensor
        if (++u == P.Hf) {
            u = 0;
            if (++k == P.Wp) {
                k = 0;
                if (++m == P.Ho) {
                    m = 0;
                    src += P.plane_in;
                }
            }
        }
    }

    if (VEC == 4) {
        if (y0 + 4 <= P.total) {
            *reinterpret_cast<uint4 *>(P.win + y0) = make_uint4(v[0], v[1], v[2], v[3]);
        } else {
            for (int e = 0; e < VEC; ++e)
                if (y0 + e < P.total) P.win[y0 + e] = v[e];
        }
    } else {
        P.win[y0] = v[0];
    }
}

hipError_t launch_transform(const float *in, float *win, const Shape &sh, hipStream_t st)
{
    TransformParams P;
    P.in = reinterpret_cast<const uint32_t *>(in);
    P.win = reinterpret_cast<uint32_t *>(win);
    P.Ci = sh.Ci; P.Hi = sh.Hi; P.Wi = sh.Wi; P.Ho = sh.Ho; P.Hf = sh.Hf;
    P.s = sh.s; P.p = sh.p; P.Wp = sh.Wp;
    P.rowlen = (uint32_t)sh.rowlen;
    P.total = (uint32_t)((size_t)sh.N * sh.Ci * sh.Ho * sh.rowlen);
    P.plane_in = (uint32_t)(sh.Hi * sh.Wi);
    P.d_rowlen = make_fastdiv(P.rowlen);
    P.d_ho = make_fastdiv((uint32_t)sh.Ho);
    P.d_hf = make_fastdiv((uint32_t)sh.Hf);

    bool vec4 = (reinterpret_cast<uintptr_t>(win) & 15u) == 0;
    if (vec4) {
        uint32_t chunks = (P.total + 3u) / 4u;
        uint32_t blocks = (chunks + 255u) / 256u;
        hipLaunchKernelGGL(transform_kernel<4>, dim3(blocks), dim3(256), 0, st, P);
    } else {
        uint32_t blocks = (P.total + 255u) / 256u;
        hipLaunchKernelGGL(transform_kernel<1>, dim3(blocks), dim3(256), 0, st, P);
    }
    return hipGetLastError();
}

}  // namespace im2win
