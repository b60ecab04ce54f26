/*
 * im2win.h -- C ABI of the MI355X (gfx950) im2win convolution library.
 *
 * The library implements the forward path of "Im2win: An Efficient Convolution
 * Paradigm on GPU" (arXiv 2306.14316): the im2win data transformation
 * (Section 3.1, Eq. 2) and the forward convolution computed over the im2win
 * tensor (Section 3.2, Algorithms 2 and 3), in fp32.
 *
 * Notation and layouts (Section 2.1), all fp32, all dense and contiguous:
 *   input   I[N][Ci][Hi][Wi]                     (NCHW)
 *   filter  F[Co][Ci][Hf][Wf]
 *   output  O[N][Co][Ho][Wo]                     (NCHW)
 *   window  What[N][Ci][Ho][Wp*Hf], Wp = Wi+2*pad (the im2win tensor)
 * One stride applies to both axes, as in the paper.  Zero padding `pad` on all
 * four sides is an extension (every layer of the paper's Table 2 is unpadded);
 * it is materialised in the im2win tensor, whose rows are Wp*Hf long.
 *   Ho = floor((Hi + 2*pad - Hf)/stride) + 1,  Wo likewise (Table 2).
 *
 * Conventions for every entry point:
 *   - Pointers named *_dev are DEVICE pointers on the current HIP device; the
 *     caller owns all buffers and the library allocates nothing and keeps no
 *     state between calls.  Buffers must not overlap.  4-byte alignment is
 *     enough (16-byte alignment lets the kernels use wider accesses).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on it and never synchronise.
 *   - Outputs are overwritten in full (no accumulation into them).
 *   - Errors are returned, never thrown; on any error nothing is launched.
 *   - Every tensor must have fewer than 2^31 elements (IM2WIN_ERR_OVERFLOW);
 *     the baselines' im2col matrix alone may be larger (see there).
 */
#ifndef IM2WIN_H_
#define IM2WIN_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    IM2WIN_OK = 0,
    IM2WIN_ERR_NULL = -1,        /* a required pointer is NULL                           */
    IM2WIN_ERR_SHAPE = -2,       /* a dimension <= 0, stride < 1, pad < 0, or the filter */
                                 /* is larger than the padded input                      */
    IM2WIN_ERR_OVERFLOW = -3,    /* a tensor has 2^31 or more elements                   */
    IM2WIN_ERR_UNSUPPORTED = -4, /* shape needs more LDS than one workgroup can hold, or */
                                 /* an unknown kernel variant was requested              */
    IM2WIN_ERR_HIP = -5          /* the HIP runtime refused the launch                   */
} im2win_status;

/* Output extent of the convolution (size rule of Table 2, with padding). */
im2win_status im2win_out_shape(int Hi, int Wi, int Hf, int Wf, int stride, int pad,
                               int *Ho, int *Wo);

/* Bytes of the im2win tensor, 4*N*Ci*Ho*Hf*(Wi+2*pad): the workspace the caller
 * must provide between the two calls below (Section 3.1: size (Ni,Ci,Ho,Wi x Hf)). */
im2win_status im2win_workspace_bytes(int N, int Ci, int Hi, int Wi, int Hf, int Wf,
                                     int stride, int pad, size_t *bytes);

/* Bytes the im2col matrices of the same layer would take, 4*N*Ho*Wo*Ci*Hf*Wf
 * (Section 2.3); for reporting the footprint saving only. */
im2win_status im2col_footprint_bytes(int N, int Ci, int Hi, int Wi, int Hf, int Wf,
                                     int stride, int pad, size_t *bytes);

/*
 * im2win data transformation (Section 3.1, Eq. 2):
 *   window(i, r, m, k*Hf + u) = Ipad(i, r, m*stride + u, k)
 * for 0<=m<Ho, 0<=k<Wp, 0<=u<Hf, where Ipad is the input with `pad` zeros on
 * each side.  Values are copied bit for bit; padding is written as +0.0.
 *   input_dev   device, N*Ci*Hi*Wi floats, read only
 *   window_dev  device, N*Ci*Ho*Wp*Hf floats, fully overwritten
 */
im2win_status im2win_transform(const float *input_dev, float *window_dev,
                               int N, int Ci, int Hi, int Wi, int Hf, int Wf,
                               int stride, int pad, void *stream);

/*
 * Forward convolution over the im2win tensor (Section 3.2, Algorithm 3's role;
 * result defined by Eq. 1):
 *   O(i,j,m,n) = sum_{r,u,v} window(i, r, m, (n*stride+v)*Hf + u) * F(j,r,u,v)
 * computed as a GEMM with M = Co, N = N*Ho*Wo, K = Ci*Hf*Wf on the fp32 matrix
 * cores (fp32 multiply, fp32 accumulate; summation order is unspecified).
 * Hi, Wi and pad are those given to im2win_transform, so that both calls derive
 * the same shapes.
 *   window_dev  device, as written by im2win_transform, read only
 *   filter_dev  device, Co*Ci*Hf*Wf floats in the paper's [Co][Ci][Hf][Wf] order
 *   output_dev  device, N*Co*Ho*Wo floats, fully overwritten
 */
im2win_status conv2d_im2win_fwd(const float *window_dev, const float *filter_dev,
                                float *output_dev,
                                int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf,
                                int stride, int pad, void *stream);

/*
 * The basic im2win convolution of Algorithm 2 (Section 3.2): one thread per
 * output element, a K loop of scalar multiply-adds reading the im2win tensor
 * and the filter from global memory.  Same arguments and result as
 * conv2d_im2win_fwd; kept as the slow in-library reference kernel.
 */
im2win_status conv2d_im2win_fwd_basic(const float *window_dev, const float *filter_dev,
                                      float *output_dev,
                                      int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf,
                                      int stride, int pad, void *stream);

/*
 * Ablation variants of the convolution (Section 4.4 removes one optimisation
 * at a time; these are the CDNA4 counterparts).  Same arguments and result as
 * conv2d_im2win_fwd plus `variant` (any other value: IM2WIN_ERR_UNSUPPORTED):
 *   IM2WIN_VARIANT_DEFAULT           the kernel conv2d_im2win_fwd would pick;
 *   IM2WIN_VARIANT_NO_PIPELINE       no double buffer / prefetch: one LDS stage,
 *                                    staging outside the MFMA chain (any layer);
 *   IM2WIN_VARIANT_VALU_MICROKERNEL  no matrix cores: the tiling, LDS strips and
 *                                    filter tile of NO_PIPELINE, but every thread
 *                                    keeps a 4x4 register tile of outputs and advances
 *                                    it with scalar fused multiply-adds (the M_T x N_T
 *                                    micro-kernel of Section 3.3 on the vector ALUs);
 *                                    compare with NO_PIPELINE, which differs from it in
 *                                    the arithmetic unit only;
 *   IM2WIN_VARIANT_NARROW_LOADS,     the default kernel with the filter rows fetched in
 *   IM2WIN_VARIANT_SCALAR_LOADS      8-byte / 4-byte instead of 16-byte pieces (the vector
 *                                    loads of Section 3.3 at half and quarter width; the
 *                                    strips are staged in 4-byte words in every variant,
 *                                    their runs being 4-byte aligned only); the pipelined
 *                                    3x3 kernel alone has such instances, other layers
 *                                    run the default kernel;
 *   IM2WIN_VARIANT_NO_MFMA           none of the above at once -- no LDS, no register
 *                                    tile, no matrix cores: one thread per output
 *                                    (Algorithm 2, conv2d_im2win_fwd_basic).
 */
enum {
    IM2WIN_VARIANT_DEFAULT = 0,
    IM2WIN_VARIANT_NO_PIPELINE = 1,
    IM2WIN_VARIANT_NO_MFMA = 2,
    IM2WIN_VARIANT_NARROW_LOADS = 3,
    IM2WIN_VARIANT_VALU_MICROKERNEL = 4,
    IM2WIN_VARIANT_SCALAR_LOADS = 5,
    IM2WIN_VARIANT_LAST = IM2WIN_VARIANT_SCALAR_LOADS
};
im2win_status conv2d_im2win_fwd_variant(const float *window_dev, const float *filter_dev,
                                        float *output_dev,
                                        int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf,
                                        int stride, int pad, int variant, void *stream);

/*
 * Workspace-free variant: the same convolution computed straight from the NCHW
 * input.  Each workgroup builds the im2win strips of its tile (Section 3.1, Eq. 2)
 * in LDS instead of reading them from an im2win tensor, so no workspace and no
 * transform call are needed; the MFMA loop and the result are those of
 * conv2d_im2win_fwd.  Any layer is accepted.  Layers the pipelined kernel takes
 * (3x3 filters with Ci a multiple of 8, 5x5 with Ci a multiple of 4, 7x7 with
 * Ci even, filter_dev 16-byte aligned) run at the speed of conv2d_im2win_fwd
 * alone; the others (three-channel stem layers among them) take the generic,
 * unpipelined kernel and are slower than the two-call path.
 *   input_dev   device, N*Ci*Hi*Wi floats, read only
 *   filter_dev  device, Co*Ci*Hf*Wf floats, [Co][Ci][Hf][Wf]
 *   output_dev  device, N*Co*Ho*Wo floats, fully overwritten
 */
im2win_status conv2d_im2win_implicit_fwd(const float *input_dev, const float *filter_dev,
                                         float *output_dev,
                                         int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf,
                                         int stride, int pad, void *stream);

/*
 * Comparison baselines (not part of the im2win path; same conventions).
 *
 * conv2d_direct_fwd: the direct convolution of Section 2.2 -- one thread per
 * output element evaluates Eq. 1 from the NCHW input with no workspace.
 *   input_dev   device, N*Ci*Hi*Wi floats, read only
 *   filter_dev  device, Co*Ci*Hf*Wf floats, [Co][Ci][Hf][Wf]
 *   output_dev  device, N*Co*Ho*Wo floats, fully overwritten
 *
 * im2col_transform + conv2d_im2col_fwd: the GEMM-based convolution of
 * Section 2.3.  The im2col matrices of all images are stacked into
 *   col[(i*Ho + m)*Wo + n][(r*Hf + u)*Wf + v] = Ipad(i, r, m*stride + u, n*stride + v),
 * N*Ho*Wo rows of K = Ci*Hf*Wf floats, dense (im2col_footprint_bytes gives its
 * size, which may pass 2^31 elements: the limit is 2^31 groups of four floats,
 * IM2WIN_ERR_OVERFLOW beyond).  conv2d_im2col_fwd multiplies it with the filter
 * matrix on the fp32 matrix cores and writes NCHW output.
 *   col_dev     device, N*Ho*Wo*Ci*Hf*Wf floats; written by im2col_transform,
 *               read by conv2d_im2col_fwd
 */
im2win_status conv2d_direct_fwd(const float *input_dev, const float *filter_dev, float *output_dev,
                                int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf,
                                int stride, int pad, void *stream);
im2win_status im2col_transform(const float *input_dev, float *col_dev,
                               int N, int Ci, int Hi, int Wi, int Hf, int Wf,
                               int stride, int pad, void *stream);
im2win_status conv2d_im2col_fwd(const float *col_dev, const float *filter_dev, float *output_dev,
                                int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf,
                                int stride, int pad, void *stream);

/*
 * Which kernel a call would launch, and how: host-side queries that run the
 * library's own dispatch for the given layer and launch nothing (for reports and
 * for matching profiler output; they are not needed to use the path).  Buffers
 * are taken to be 16-byte aligned, as device allocations are.  The choice of
 * grid depends on the current device's number of compute units; with no device
 * present an MI355X's 256 are assumed.
 *   kernel     the kernel as a profiler prints it: function name and template
 *              arguments, without namespace and parameter list
 *   grid_x/y   workgroups, block: threads per workgroup, lds_bytes: dynamic LDS
 * im2win_transform_launch_info describes im2win_transform;
 * conv2d_im2win_fwd_launch_info describes conv2d_im2win_fwd_variant(variant), or,
 * with workspace_free != 0 (variant must then be IM2WIN_VARIANT_DEFAULT),
 * conv2d_im2win_implicit_fwd.  Errors as for the calls they describe.
 */
typedef struct {
    char kernel[160];
    unsigned grid_x, grid_y, block;
    size_t lds_bytes;
} im2win_launch_info;
im2win_status im2win_transform_launch_info(int N, int Ci, int Hi, int Wi, int Hf, int Wf,
                                           int stride, int pad, im2win_launch_info *info);
im2win_status conv2d_im2win_fwd_launch_info(int N, int Ci, int Hi, int Wi, int Co, int Hf, int Wf,
                                            int stride, int pad, int variant, int workspace_free,
                                            im2win_launch_info *info);

/* Static description of a status code (never NULL). */
const char *im2win_status_str(im2win_status status);

#ifdef __cplusplus
}
#endif
#endif /* IM2WIN_H_ */
