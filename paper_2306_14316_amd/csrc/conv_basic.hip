// Basic im2win convolution (Section 3.2, Algorithm 2) for gfx950: one thread
// per output element, a K loop of scalar fp32 multiply-adds that reads the
// im2win tensor and the filter straight from global memory.  Slow by design:
// it is the in-library reference the MFMA kernel is developed against and the
// "no micro-kernel, no LDS" end of the ablation (Section 4.4).
#include "common.h"

namespace im2win {

struct BasicParams {
    const float *win;
    const float *flt;
    float *out;
    int Ci, Ho, Wo, Co, Hf, Wf, s;
    uint32_t rowlen, khw, total;   // total = N*Co*Ho*Wo
    FastDiv d_wo, d_ho, d_co;
};

__global__ __launch_bounds__(256) void conv_basic_kernel(BasicParams P)
{
    uint32_t o = blockIdx.x * 256u + threadIdx.x;   // flat NCHW output index
    if (o >= P.total) return;
    uint32_t t = fdiv(o, P.d_wo);
    uint32_t n = o - t * (uint32_t)P.Wo;
    uint32_t t2 = fdiv(t, P.d_ho);
    uint32_t m = t - t2 * (uint32_t)P.Ho;
    uint32_t i = fdiv(t2, P.d_co);
    uint32_t j = t2 - i * (uint32_t)P.Co;

    // Window of channel r for this output: a contiguous run of Hf*Wf floats that
    // starts at column n*s of row (i, r, m), ordered column after column.
    const float *wrow = P.win + ((size_t)i * P.Ci * P.Ho + m) * P.rowlen + (size_t)n * P.s * P.Hf;
    const float *f = P.flt + (size_t)j * P.Ci * P.khw;
    size_t chan_stride = (size_t)P.Ho * P.rowlen;
    float acc = 0.0f;
    for (int r = 0; r < P.Ci; ++r) {
        for (int u = 0; u < P.Hf; ++u)
            for (int v = 0; v < P.Wf; ++v)
                acc = fmaf(wrow[v * P.Hf + u], f[u * P.Wf + v], acc);
        wrow += chan_stride;
        f += P.khw;
    }
    P.out[o] = acc;
}

hipError_t launch_conv_basic(const float *win, const float *flt, float *out, const Shape &sh,
                             hipStream_t st, LaunchPlan *plan)
{
    BasicParams P;
    P.win = win; P.flt = flt; P.out = out;
    P.Ci = sh.Ci; P.Ho = sh.Ho; P.Wo = sh.Wo; P.Co = sh.Co; P.Hf = sh.Hf; P.Wf = sh.Wf; P.s = sh.s;
    P.rowlen = (uint32_t)sh.rowlen;
    P.khw = (uint32_t)sh.khw;
    P.total = (uint32_t)((size_t)sh.npix * sh.Co);
    P.d_wo = make_fastdiv((uint32_t)sh.Wo);
    P.d_ho = make_fastdiv((uint32_t)sh.Ho);
    P.d_co = make_fastdiv((uint32_t)sh.Co);
    uint32_t blocks = (P.total + 255u) / 256u;
    if (plan) { plan_record(plan, dim3(blocks), 256, 0, "conv_basic_kernel"); return hipSuccess; }
    hipLaunchKernelGGL(conv_basic_kernel, dim3(blocks), dim3(256), 0, st, P);
    return hipGetLastError();
}

}  // namespace im2win
