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
    size_t out_elems;   // floats in the output
    // workspace-free variant only: `win` is then the NCHW input itself
    int implicit;       // 1: workspace-free variant
    int Hi, Wi, p;
    uint32_t in_plane;  // Hi*Wi
    int cb;          // channels per K block
    int S;           // LDS floats reserved per channel strip
    int SP;          // the same rounded up to a multiple of 64 (pipelined generic kernel)
    int rmax;        // output rows a tile may touch
    int fullseg;     // ((Wo-1)*s + Wf)*Hf : strip floats of a fully covered output row
    int tiles_m;
    uint32_t nblocks;   // tiles of the whole layer (the pipelined kernel may run fewer workgroups)
    uint32_t nmain;     // pipelined kernel: tiles below this one are computed whole,
    uint32_t nhalf;     // the next nhalf tiles as two halves each, the rest in sixteenths
    uint32_t tail_at;   // grid position (block index) of the first sixteenth
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

// The same epilogue through a buffer descriptor, for the pipelined kernel: the base (image of
// the tile's first pixel, first channel of the wave) is wave-uniform and sits in scalar
// registers, the lane adds one 32-bit byte offset (its pixel, its first channel) and each store
// a scalar channel offset, so the sixteen stores cost no vector-ALU address arithmetic (plain
// pointer stores cost eight vector instructions each, which comes out of the MFMA rate).  The
// host has checked that a tile's outputs lie within 4 GiB of that base.  wm, wn: wave-uniform.
__device__ __forceinline__ void store_tile_desc(const MfmaParams &P, const floatx16 &acc, uint32_t P0,
                                                uint32_t Pend, int m0, int wm, int wn, int h, int l32)
{
    const int jw = m0 + wm * 32;                  // first channel of the wave
    if (jw >= P.Co) return;
    const uint32_t img0 = fdiv(P0, P.d_howo);     // image of the tile's first pixel
    const size_t obase = ((size_t)img0 * P.Co + (size_t)jw) * P.howo;
    const size_t left = (P.out_elems - obase) * 4u;
    const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc(
        P.out + obase, 0, left < 0xffffffffull ? left : 0xffffffffull, 0x00020000);
    const uint32_t Pm = P0 + (uint32_t)(wn * 32 + l32);
    if (Pm <= Pend) {
        const uint32_t img = fdiv(Pm, P.d_howo);
        const uint32_t pin = Pm - img * P.howo;
        const uint32_t voff = ((img - img0) * (uint32_t)P.Co * P.howo + pin + (uint32_t)(4 * h) * P.howo) * 4u;
        const uint32_t howo4 = P.howo * 4u;
        const bool full = jw + 32 <= P.Co;        // wave-uniform: every channel of the wave exists
        const int room = P.Co - jw - 4 * h;       // channels this lane may store, counted from its first
        if (full) {   // scalar branch: sixteen unconditional stores
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float val = acc[v];   // (a scalar copy: bit-casting the vector element directly stores element 0)
                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, val), ro, voff,
                                                      (uint32_t)(8 * (v >> 2) + (v & 3)) * howo4, 0);
            }
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int dj = 8 * (v >> 2) + (v & 3);
                const float val = acc[v];
                if (dj < room)
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, val), ro, voff, (uint32_t)dj * howo4, 0);
            }
        }
    }
}

hipError_t launch_conv_mfma_fast(MfmaParams P, const Shape &sh, uint32_t blocks, hipStream_t st,
                                 bool implicit = false, int filter_fetch_floats = 4, LaunchPlan *plan = nullptr);
hipError_t launch_conv_mfma_shallow(const float *win, const float *flt, float *out, const Shape &sh,
                                    hipStream_t st, bool implicit = false, LaunchPlan *plan = nullptr);
hipError_t launch_conv_mfma_1x1(const float *src, const float *flt, float *out, const Shape &sh,
                                hipStream_t st, bool implicit = false, LaunchPlan *plan = nullptr);

}  // namespace im2win
