// Internal declarations shared by the library's translation units (host side
// and gfx950 device side).  Not part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace im2win {

// Division of a 32-bit n < 2^31 by a run-time constant d >= 1 with one
// multiply-high, one add and one shift (round-up reciprocal).
struct FastDiv {
    uint32_t mul;
    uint32_t shift;
    uint32_t d;
};

inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    f.d = d;
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    f.shift = l;
    f.mul = (uint32_t)((((1ull << l) - d) << 32) / d + 1);
    return f;
}

__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv &f)
{
    return (__umulhi(n, f.mul) + n) >> f.shift;
}

// Workgroups are handed to the 8 XCDs round-robin (block b runs on XCD b % 8)
// and each XCD has its own L2.  Remap so that each XCD works through one
// contiguous range of logical blocks: neighbouring items (the M tiles that share an
// im2win strip, neighbouring strips; the transform's neighbouring output rows, which read the
// same input rows) then meet in the same L2.
__device__ __forceinline__ uint32_t xcd_swizzle(uint32_t b, uint32_t nblocks)
{
    const uint32_t x = b & 7u, i = b >> 3;
    const uint32_t q = nblocks >> 3, r = nblocks & 7u;
    return x * q + min(x, r) + i;
}

// The same idea for streaming kernels, kept local: within each group of 64 consecutive blocks
// XCD x takes blocks 8x .. 8x+7, so neighbours meet in one L2 while the eight XCDs still write
// one compact front (remapping the whole grid, as above, slowed large transforms by 7-9 %).
__device__ __forceinline__ uint32_t xcd_swizzle64(uint32_t b, uint32_t nblocks)
{
    if (b >= (nblocks & ~63u)) return b;   // last partial group: as dealt
    return (b & ~63u) | ((b & 7u) << 3) | ((b >> 3) & 7u);
}

// Shapes derived once on the host from the ABI arguments.
struct Shape {
    int N, Ci, Hi, Wi, Co, Hf, Wf, s, p;
    int Ho, Wo, Hp, Wp;
    int rowlen;   // Wp*Hf : floats in one row of the im2win tensor
    int khw;      // Hf*Wf : floats in one dot-product window of one channel
    int K;        // Ci*Hf*Wf
    int npix;     // N*Ho*Wo : GEMM N dimension
};

// A launcher that is handed a LaunchPlan decides exactly as it would for a launch -- kernel
// instance, grid, LDS -- writes the decision down and launches nothing.  The kernel is named as
// a profiler prints it: function name and template arguments, without namespace or parameters.
struct LaunchPlan {
    char kernel[160];
    unsigned grid_x, grid_y, block;
    size_t lds_bytes;
};
void plan_record(LaunchPlan *plan, dim3 grid, unsigned block, size_t lds, const char *fmt, ...)
    __attribute__((format(printf, 5, 6)));
inline const char *tf(bool b) { return b ? "true" : "false"; }

// ---- launchers (defined in the .hip files) -------------------------------
hipError_t launch_transform(const float *in, float *win, const Shape &sh, hipStream_t st,
                            LaunchPlan *plan = nullptr);
hipError_t launch_conv_basic(const float *win, const float *flt, float *out, const Shape &sh,
                             hipStream_t st, LaunchPlan *plan = nullptr);
// Comparison baselines: direct convolution on the NCHW input; im2col matrix and GEMM over it.
// The im2col launchers return hipErrorInvalidValue when the matrix has 2^31 or more 16-byte groups.
hipError_t launch_conv_direct(const float *in, const float *flt, float *out, const Shape &sh,
                              hipStream_t st, LaunchPlan *plan = nullptr);
hipError_t launch_im2col(const float *in, float *col, const Shape &sh, hipStream_t st);
hipError_t launch_gemm_im2col(const float *col, const float *flt, float *out, const Shape &sh,
                              hipStream_t st);
// Workspace-free convolution from the NCHW input; hipErrorNotSupported when the layer is not one the
// pipelined kernel takes.
hipError_t launch_conv_implicit(const float *in, const float *flt, float *out, const Shape &sh,
                                hipStream_t st, LaunchPlan *plan = nullptr);
// Kernel selection for the MFMA convolution (the values of the public
// IM2WIN_VARIANT_* constants).
enum ConvVariant { kVariantDefault = 0, kVariantNoPipeline = 1, kVariantNoMfma = 2, kVariantNarrowLoads = 3,
                   kVariantValuMicrokernel = 4, kVariantScalarLoads = 5 };
// Returns hipErrorInvalidConfiguration when no tile configuration fits in LDS.
hipError_t launch_conv_mfma(const float *win, const float *flt, float *out, const Shape &sh,
                            hipStream_t st, int variant = kVariantDefault, LaunchPlan *plan = nullptr);

}  // namespace im2win
