// C ABI of the library (see include/im2win.h): argument validation, shape
// derivation and dispatch to the gfx950 kernels.  Host code only.
#include "../../include/im2win.h"
#include "common.h"

#include <limits.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

using im2win::Shape;

namespace {

const long long kMaxElems = 2147483647LL;   // every tensor must stay below 2^31 elements

im2win_status derive(int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf, int stride, int pad,
                     Shape *sh)
{
    if (N <= 0 || Ci <= 0 || Hi <= 0 || Wi <= 0 || Co <= 0 || Hf <= 0 || Wf <= 0) return IM2WIN_ERR_SHAPE;
    if (stride < 1 || pad < 0) return IM2WIN_ERR_SHAPE;
    long long Hp = (long long)Hi + 2LL * pad, Wp = (long long)Wi + 2LL * pad;
    if (Hf > Hp || Wf > Wp) return IM2WIN_ERR_SHAPE;
    if (Hp > INT_MAX || Wp > INT_MAX) return IM2WIN_ERR_OVERFLOW;
    long long Ho = (Hp - Hf) / stride + 1, Wo = (Wp - Wf) / stride + 1;
    long long rowlen = Wp * Hf, khw = (long long)Hf * Wf, K = khw * Ci;
    long long n_in = (long long)N * Ci;
    // products are checked step by step so that nothing wraps
    auto mul_ok = [](long long a, long long b, long long *r) {
        if (a != 0 && b > kMaxElems / a) return false;
        *r = a * b;
        return *r <= kMaxElems;
    };
    // every tensor of the call: input, im2win tensor, output, filter
    long long t, in_e, win_e, out_e, flt_e;
    if (!mul_ok(n_in, Hi, &t) || !mul_ok(t, Wi, &in_e)) return IM2WIN_ERR_OVERFLOW;
    if (rowlen > kMaxElems || !mul_ok(n_in, Ho, &t) || !mul_ok(t, rowlen, &win_e)) return IM2WIN_ERR_OVERFLOW;
    if ((long long)N * Co > kMaxElems || !mul_ok((long long)N * Co, Ho, &t) || !mul_ok(t, Wo, &out_e))
        return IM2WIN_ERR_OVERFLOW;
    if (khw > kMaxElems || !mul_ok(khw, Ci, &t) || !mul_ok(t, Co, &flt_e)) return IM2WIN_ERR_OVERFLOW;
    sh->N = N; sh->Ci = Ci; sh->Hi = Hi; sh->Wi = Wi; sh->Co = Co; sh->Hf = Hf; sh->Wf = Wf;
    sh->s = stride; sh->p = pad;
    sh->Ho = (int)Ho; sh->Wo = (int)Wo; sh->Hp = (int)Hp; sh->Wp = (int)Wp;
    sh->rowlen = (int)rowlen; sh->khw = (int)khw; sh->K = (int)K;
    sh->npix = (int)((long long)N * Ho * Wo);
    return IM2WIN_OK;
}

im2win_status copy_plan(const im2win::LaunchPlan &plan, im2win_launch_info *info)
{
    static_assert(sizeof(info->kernel) == sizeof(plan.kernel), "same name capacity on both sides of the ABI");
    memcpy(info->kernel, plan.kernel, sizeof(info->kernel));
    info->grid_x = plan.grid_x; info->grid_y = plan.grid_y; info->block = plan.block;
    info->lds_bytes = plan.lds_bytes;
    return IM2WIN_OK;
}

// Stand-ins for the buffers of a planned call: never dereferenced, 16-byte aligned like the
// buffers the planning calls are documented to assume.
const float *const kAlignedIn = reinterpret_cast<const float *>(uintptr_t(256));
float *const kAlignedOut = reinterpret_cast<float *>(uintptr_t(512));

}  // namespace

void im2win::plan_record(LaunchPlan *plan, dim3 grid, unsigned block, size_t lds, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(plan->kernel, sizeof(plan->kernel), fmt, ap);
    va_end(ap);
    plan->grid_x = grid.x; plan->grid_y = grid.y; plan->block = block; plan->lds_bytes = lds;
}

extern "C" {

im2win_status im2win_out_shape(int Hi, int Wi, int Hf, int Wf, int stride, int pad, int *Ho, int *Wo)
{
    if (!Ho || !Wo) return IM2WIN_ERR_NULL;
    Shape sh;
    im2win_status st = derive(1, 1, Hi, Wi, 1, Hf, Wf, stride, pad, &sh);
    if (st != IM2WIN_OK) return st;
    *Ho = sh.Ho;
    *Wo = sh.Wo;
    return IM2WIN_OK;
}

im2win_status im2win_workspace_bytes(int N, int Ci, int Hi, int Wi, int Hf, int Wf, int stride, int pad,
                                     size_t *bytes)
{
    if (!bytes) return IM2WIN_ERR_NULL;
    Shape sh;
    im2win_status st = derive(N, Ci, Hi, Wi, 1, Hf, Wf, stride, pad, &sh);
    if (st != IM2WIN_OK) return st;
    *bytes = (size_t)4 * (size_t)N * Ci * sh.Ho * (size_t)sh.rowlen;
    return IM2WIN_OK;
}

im2win_status im2col_footprint_bytes(int N, int Ci, int Hi, int Wi, int Hf, int Wf, int stride, int pad,
                                     size_t *bytes)
{
    if (!bytes) return IM2WIN_ERR_NULL;
    Shape sh;
    im2win_status st = derive(N, Ci, Hi, Wi, 1, Hf, Wf, stride, pad, &sh);
    if (st != IM2WIN_OK) return st;
    *bytes = (size_t)4 * (size_t)N * sh.Ho * sh.Wo * (size_t)Ci * Hf * Wf;   // reporting only: may exceed 2^31 elements
    return IM2WIN_OK;
}

im2win_status im2win_transform(const float *input_dev, float *window_dev, int N, int Ci, int Hi, int Wi,
                               int Hf, int Wf, int stride, int pad, void *stream)
{
    if (!input_dev || !window_dev) return IM2WIN_ERR_NULL;
    Shape sh;
    im2win_status st = derive(N, Ci, Hi, Wi, 1, Hf, Wf, stride, pad, &sh);
    if (st != IM2WIN_OK) return st;
    hipError_t e = im2win::launch_transform(input_dev, window_dev, sh, (hipStream_t)stream);
    return e == hipSuccess ? IM2WIN_OK : IM2WIN_ERR_HIP;
}

im2win_status conv2d_im2win_fwd(const float *window_dev, const float *filter_dev, float *output_dev,
                                int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf, int stride, int pad,
                                void *stream)
{
    if (!window_dev || !filter_dev || !output_dev) return IM2WIN_ERR_NULL;
    Shape sh;
    im2win_status st = derive(N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, &sh);
    if (st != IM2WIN_OK) return st;
    hipError_t e = im2win::launch_conv_mfma(window_dev, filter_dev, output_dev, sh, (hipStream_t)stream);
    if (e == hipErrorInvalidConfiguration) return IM2WIN_ERR_UNSUPPORTED;
    return e == hipSuccess ? IM2WIN_OK : IM2WIN_ERR_HIP;
}

im2win_status conv2d_im2win_fwd_variant(const float *window_dev, const float *filter_dev, float *output_dev,
                                        int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf, int stride,
                                        int pad, int variant, void *stream)
{
    if (!window_dev || !filter_dev || !output_dev) return IM2WIN_ERR_NULL;
    if (variant < IM2WIN_VARIANT_DEFAULT || variant > IM2WIN_VARIANT_LAST) return IM2WIN_ERR_UNSUPPORTED;
    Shape sh;
    im2win_status st = derive(N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, &sh);
    if (st != IM2WIN_OK) return st;
    hipError_t e = im2win::launch_conv_mfma(window_dev, filter_dev, output_dev, sh, (hipStream_t)stream, variant);
    if (e == hipErrorInvalidConfiguration || e == hipErrorNotSupported) return IM2WIN_ERR_UNSUPPORTED;
    return e == hipSuccess ? IM2WIN_OK : IM2WIN_ERR_HIP;
}

im2win_status conv2d_im2win_fwd_basic(const float *window_dev, const float *filter_dev, float *output_dev,
                                      int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf, int stride,
                                      int pad, void *stream)
{
    if (!window_dev || !filter_dev || !output_dev) return IM2WIN_ERR_NULL;
    Shape sh;
    im2win_status st = derive(N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, &sh);
    if (st != IM2WIN_OK) return st;
    hipError_t e = im2win::launch_conv_basic(window_dev, filter_dev, output_dev, sh, (hipStream_t)stream);
    return e == hipSuccess ? IM2WIN_OK : IM2WIN_ERR_HIP;
}

im2win_status conv2d_im2win_implicit_fwd(const float *input_dev, const float *filter_dev, float *output_dev,
                                         int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf, int stride, int pad,
                                         void *stream)
{
    if (!input_dev || !filter_dev || !output_dev) return IM2WIN_ERR_NULL;
    Shape sh;
    im2win_status st = derive(N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, &sh);
    if (st != IM2WIN_OK) return st;
    hipError_t e = im2win::launch_conv_implicit(input_dev, filter_dev, output_dev, sh, (hipStream_t)stream);
    if (e == hipErrorNotSupported || e == hipErrorInvalidConfiguration) return IM2WIN_ERR_UNSUPPORTED;
    return e == hipSuccess ? IM2WIN_OK : IM2WIN_ERR_HIP;
}

im2win_status conv2d_direct_fwd(const float *input_dev, const float *filter_dev, float *output_dev,
                                int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf, int stride, int pad,
                                void *stream)
{
    if (!input_dev || !filter_dev || !output_dev) return IM2WIN_ERR_NULL;
    Shape sh;
    im2win_status st = derive(N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, &sh);
    if (st != IM2WIN_OK) return st;
    hipError_t e = im2win::launch_conv_direct(input_dev, filter_dev, output_dev, sh, (hipStream_t)stream);
    return e == hipSuccess ? IM2WIN_OK : IM2WIN_ERR_HIP;
}

im2win_status im2col_transform(const float *input_dev, float *col_dev, int N, int Ci, int Hi, int Wi,
                               int Hf, int Wf, int stride, int pad, void *stream)
{
    if (!input_dev || !col_dev) return IM2WIN_ERR_NULL;
    Shape sh;
    im2win_status st = derive(N, Ci, Hi, Wi, 1, Hf, Wf, stride, pad, &sh);
    if (st != IM2WIN_OK) return st;
    hipError_t e = im2win::launch_im2col(input_dev, col_dev, sh, (hipStream_t)stream);
    if (e == hipErrorInvalidValue) return IM2WIN_ERR_OVERFLOW;
    return e == hipSuccess ? IM2WIN_OK : IM2WIN_ERR_HIP;
}

im2win_status conv2d_im2col_fwd(const float *col_dev, const float *filter_dev, float *output_dev,
                                int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf, int stride, int pad,
                                void *stream)
{
    if (!col_dev || !filter_dev || !output_dev) return IM2WIN_ERR_NULL;
    Shape sh;
    im2win_status st = derive(N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, &sh);
    if (st != IM2WIN_OK) return st;
    if ((unsigned long long)sh.npix * (unsigned long long)((sh.K + 3) / 4) >= (1ull << 31)) return IM2WIN_ERR_OVERFLOW;
    hipError_t e = im2win::launch_gemm_im2col(col_dev, filter_dev, output_dev, sh, (hipStream_t)stream);
    if (e == hipErrorInvalidValue) return IM2WIN_ERR_OVERFLOW;
    return e == hipSuccess ? IM2WIN_OK : IM2WIN_ERR_HIP;
}

im2win_status im2win_transform_launch_info(int N, int Ci, int Hi, int Wi, int Hf, int Wf, int stride, int pad,
                                           im2win_launch_info *info)
{
    if (!info) return IM2WIN_ERR_NULL;
    Shape sh;
    im2win_status st = derive(N, Ci, Hi, Wi, 1, Hf, Wf, stride, pad, &sh);
    if (st != IM2WIN_OK) return st;
    im2win::LaunchPlan plan;
    hipError_t e = im2win::launch_transform(kAlignedIn, kAlignedOut, sh, nullptr, &plan);
    return e == hipSuccess ? copy_plan(plan, info) : IM2WIN_ERR_HIP;
}

im2win_status conv2d_im2win_fwd_launch_info(int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf, int stride,
                                            int pad, int variant, int workspace_free, im2win_launch_info *info)
{
    if (!info) return IM2WIN_ERR_NULL;
    if (variant < IM2WIN_VARIANT_DEFAULT || variant > IM2WIN_VARIANT_LAST) return IM2WIN_ERR_UNSUPPORTED;
    if (workspace_free && variant != IM2WIN_VARIANT_DEFAULT) return IM2WIN_ERR_UNSUPPORTED;
    Shape sh;
    im2win_status st = derive(N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, &sh);
    if (st != IM2WIN_OK) return st;
    im2win::LaunchPlan plan;
    hipError_t e = workspace_free
        ? im2win::launch_conv_implicit(kAlignedIn, kAlignedIn, kAlignedOut, sh, nullptr, &plan)
        : im2win::launch_conv_mfma(kAlignedIn, kAlignedIn, kAlignedOut, sh, nullptr, variant, &plan);
    if (e == hipErrorInvalidConfiguration || e == hipErrorNotSupported) return IM2WIN_ERR_UNSUPPORTED;
    return e == hipSuccess ? copy_plan(plan, info) : IM2WIN_ERR_HIP;
}

const char *im2win_status_str(im2win_status status)
{
    switch (status) {
        case IM2WIN_OK: return "ok";
        case IM2WIN_ERR_NULL: return "a required pointer is NULL";
        case IM2WIN_ERR_SHAPE: return "invalid shape: non-positive dimension, stride < 1, pad < 0 or filter larger than padded input";
        case IM2WIN_ERR_OVERFLOW: return "a tensor has 2^31 or more elements (im2col matrix: 2^31 or more groups of four)";
        case IM2WIN_ERR_UNSUPPORTED: return "not supported: tile does not fit in LDS, or unknown kernel variant";
        case IM2WIN_ERR_HIP: return "HIP runtime error at launch";
        default: return "unknown status";
    }
}

}  // extern "C"
