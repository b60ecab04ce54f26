// Pieces shared by the MFMA convolution kernels: tile constants, the kernel
// parameter block, the XCD-aware block mapping and the output epilogue.
#pragma once
#include "common.h"

namespace im2win {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int MB = 64;   // tile rows (output channels) per workgroup
constexpr int NB = 64;   // tile columns (output pixels) per workgroup

struct MfmaParams {
    const float *win;
    const float *flt;
    float *out;
    int Ci, Ho, Wo, Co, Hf, Wf, s;
    int rowlen, khw, K;
    uint32_t npix, howo, chan_stride;
    size_t win_elems;   // floats in the whole im2win tensor
    // workspace-free variant only: `win` is then the NCHW input itself
    int implicit;       // 1: workspace-free variant
    int Hi, Wi, p;
    uint32_t in_plane;  // Hi*Wi
    int cb;          // channels per K block
    int S;           // LDS floats reserved per channel strip
    int rmax;        // output rows a tile may touch
    int fullseg;     // ((Wo-1)*s + Wf)*Hf : strip floats of a fully covered output row
    int tiles_m;
    uint32_t nblocks;   // tiles of the whole layer (the pipelined kernel may run fewer workgroups)
    uint32_t nmain;     // pipelined kernel: tiles below this one are computed whole, the rest in sixteenths
    int vec4;        // filter rows can be read as aligned float4 in every K block
    FastDiv d_wo, d_ho, d_howo, d_khw, d_wf, d_cpr, d_tm;
};

__host__ __device__ inline int round4(int x) { return (x + 3) & ~3; }

// Epilogue: accumulator register v of lane (h, l32) holds output channel
// 8*(v/4) + 4*h + v%4 of the wave's 32 and pixel l32 of the wave's 32.  Pixels
// are contiguous in NCHW for a fixed (image, channel), so every store
// instruction writes runs of up to 128 bytes.
__device__ __forceinline__ void store_tile(const MfmaParams &P, const floatx16 &acc, uint32_t P0,
                                           uint32_t Pend, int m0, int wm, int wn, int h, int l32)
{
    const uint32_t Pm = P0 + (uint32_t)(wn * 32 + l32);
    if (Pm <= Pend) {
        const uint32_t img = fdiv(Pm, P.d_howo);
        const uint32_t pin = Pm - img * P.howo;
        float *o = P.out + (size_t)img * P.Co * P.howo + pin;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int j = m0 + wm * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
            if (j < P.Co) o[(size_t)j * P.howo] = acc[v];
        }
    }
}

hipError_t launch_conv_mfma_fast(MfmaParams P, const Shape &sh, uint32_t blocks, hipStream_t st,
                                 bool implicit = false, bool narrow = false);
hipError_t launch_conv_mfma_shallow(const float *win, const float *flt, float *out, const Shape &sh,
                                    hipStream_t st, bool implicit = false);

}  // namespace im2win
