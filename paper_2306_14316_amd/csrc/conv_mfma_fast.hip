// Software-pipelined variant of the MFMA im2win convolution for layers with
// many input channels and a small, compile-time filter (the 3x3 layers that
// make up most of the paper's Table 2).  Same tile, same strip geometry and
// same pair-step K order as conv_mfma.hip; what differs:
//   - the filter shape and the channels per K block are template constants,
//     so every LDS operand address is base + immediate and all staging
//     coordinates are computed once per thread, before the K loop;
//   - the next K block's global loads (filter rows as float4, strip words)
//     are issued into registers before the current block's MFMAs and written
//     to LDS after them (the prefetch/double-buffer idea of Section 3.3, done
//     in registers), so global latency overlaps the matrix work;
//   - the filter tile stays row-major [m][k] in LDS with an odd pitch, which
//     makes both the staging writes and the A-operand reads conflict-free; the
//     (u,v) -> window-order permutation is a compile-time offset on the read.
#include "conv_mfma_tile.h"

namespace im2win {

template <int HF, int WF, int CB, int JX>
__global__ __launch_bounds__(256) void conv_mfma_fast_kernel(MfmaParams P)
{
    constexpr int KHW = HF * WF;
    constexpr int KB = CB * KHW;            // K elements per block
    constexpr int CPR = KB / 4;             // float4 chunks per filter row per block
    constexpr int NF4 = MB * CPR;
    constexpr int JF = (NF4 + 255) / 256;   // float4 chunks per thread
    constexpr int PF = KB | 1;              // odd LDS pitch of a filter row
    static_assert(KB % 4 == 0, "K block must be a multiple of 4 floats");
    static_assert(CB % 2 == 0, "pair steps need an even channel count");

    extern __shared__ __align__(16) unsigned char smem[];
    float *sF = reinterpret_cast<float *>(smem);     // [MB][PF]
    float *sI = sF + round4(MB * PF);                // [CB][S]
    const int S = P.S;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int h = lane >> 5, l32 = lane & 31;

    const uint32_t lb = xcd_swizzle(blockIdx.x, gridDim.x);
    const uint32_t tile_n = fdiv(lb, P.d_tm);
    const uint32_t tile_m = lb - tile_n * (uint32_t)P.tiles_m;
    const int m0 = (int)tile_m * MB;
    const uint32_t P0 = tile_n * NB;
    const uint32_t Pend = min(P0 + NB - 1, P.npix - 1);

    // ---- strip geometry (rows q0..q1 of output pixels, q = i*Ho + m) ----
    const uint32_t q0 = fdiv(P0, P.d_wo), q1 = fdiv(Pend, P.d_wo);
    const int nlo0 = (int)(P0 - q0 * (uint32_t)P.Wo);
    const int sHf = P.s * HF;
    const int len0 = (((q1 == q0) ? (int)(Pend - P0) : (P.Wo - 1 - nlo0)) * P.s + WF) * HF;

    // source offset (relative to a channel plane) of strip word tid + 256*j, or -1
    int soff[JX];
#pragma unroll
    for (int j = 0; j < JX; ++j) soff[j] = -1;
    for (uint32_t q = q0; q <= q1; ++q) {
        const int rho = (int)(q - q0);
        const int nlo = rho == 0 ? nlo0 : 0;
        const int nhi = (q == q1) ? (int)(Pend - q * (uint32_t)P.Wo) : P.Wo - 1;
        const int seglen = ((nhi - nlo) * P.s + WF) * HF;
        const int segoff = rho == 0 ? 0 : len0 + (rho - 1) * P.fullseg;
        const uint32_t img = fdiv(q, P.d_ho);
        const int mq = (int)(q - img * (uint32_t)P.Ho);
        const int srcbase = (int)((img * (uint32_t)P.Ci * (uint32_t)P.Ho + (uint32_t)mq) * (uint32_t)P.rowlen) + nlo * sHf;
#pragma unroll
        for (int j = 0; j < JX; ++j) {
            const int x = tid + 256 * j - segoff;
            if (x >= 0 && x < seglen) soff[j] = srcbase + x;
        }
    }

    // ---- filter staging coordinates of this thread's float4 chunks ----
    int goff[JF], loff[JF];
#pragma unroll
    for (int j = 0; j < JF; ++j) {
        const int f = tid + 256 * j;
        const int row = f / CPR;
        const int e = (f - row * CPR) * 4;
        const bool live = (f < NF4) && (m0 + row < P.Co);
        goff[j] = live ? row * P.K + e : -1;
        loff[j] = (f < NF4) ? row * PF + e : -1;
    }

    // ---- per-lane operand bases ----
    int b_base;
    {
        const uint32_t Pl = min(P0 + (uint32_t)(wn * 32 + l32), Pend);
        const uint32_t ql = fdiv(Pl, P.d_wo);
        const int nl = (int)(Pl - ql * (uint32_t)P.Wo);
        const int rho = (int)(ql - q0);
        b_base = rho == 0 ? (nl - nlo0) * sHf : len0 + (rho - 1) * P.fullseg + nl * sHf;
    }
    const float *ap = sF + (wm * 32 + l32) * PF + h * KHW;
    const float *bp = sI + b_base + h * S;

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    float4 fr[JF];
    float ir[CB * JX];
    const float *gf = P.flt + (size_t)m0 * P.K;
    const float *gw = P.win;

    // Loads are unconditional (dead lanes read word 0 of a valid plane/row and
    // the value is replaced by zero), so that all of them are in flight at once.
    auto gload = [&](int c0) {
        const float *gfb = gf + (size_t)c0 * KHW;
#pragma unroll
        for (int j = 0; j < JF; ++j) {
            const float4 w = *reinterpret_cast<const float4 *>(gfb + (goff[j] >= 0 ? goff[j] : 0));
            fr[j] = goff[j] >= 0 ? w : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            const float *g = gw + (size_t)(c0 + c) * P.chan_stride;
#pragma unroll
            for (int j = 0; j < JX; ++j) {
                const float w = g[soff[j] >= 0 ? soff[j] : 0];
                ir[c * JX + j] = soff[j] >= 0 ? w : 0.0f;
            }
        }
    };

    gload(0);
    for (int c0 = 0; c0 < P.Ci; c0 += CB) {
        __syncthreads();   // every wave has finished reading the previous block from LDS
#pragma unroll
        for (int j = 0; j < JF; ++j) {
            if ((j + 1) * 256 <= NF4 || loff[j] >= 0) {
                float *d = sF + loff[j];
                d[0] = fr[j].x; d[1] = fr[j].y; d[2] = fr[j].z; d[3] = fr[j].w;
            }
        }
#pragma unroll
        for (int j = 0; j < JX; ++j) {
            const int x = tid + 256 * j;
            if (x < S) {
#pragma unroll
                for (int c = 0; c < CB; ++c) sI[c * S + x] = ir[c * JX + j];
            }
        }
        __syncthreads();
        if (c0 + CB < P.Ci) gload(c0 + CB);   // in flight while the matrix cores work

#pragma unroll
        for (int pr = 0; pr < CB / 2; ++pr) {
            const float *a2 = ap + 2 * pr * KHW;
            const float *b2 = bp + 2 * pr * S;
#pragma unroll
            for (int v = 0; v < WF; ++v)
#pragma unroll
                for (int u = 0; u < HF; ++u)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a2[u * WF + v], b2[v * HF + u], acc, 0, 0, 0);
        }
    }

    store_tile(P, acc, P0, Pend, m0, wm, wn, h, l32);
}

template <int HF, int WF, int CB, int JX>
static hipError_t launch_fast_t(const MfmaParams &P, uint32_t blocks, hipStream_t st)
{
    constexpr int KB = CB * HF * WF;
    constexpr int PF = KB | 1;
    const size_t lds = 4u * ((size_t)round4(MB * PF) + (size_t)CB * P.S);
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_mfma_fast_kernel<HF, WF, CB, JX>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((conv_mfma_fast_kernel<HF, WF, CB, JX>), dim3(blocks), dim3(256), lds, st, P);
    return hipGetLastError();
}

// Returns hipErrorNotSupported when the layer does not meet the fast path's conditions.
hipError_t launch_conv_mfma_fast(MfmaParams P, const Shape &sh, uint32_t blocks, hipStream_t st)
{
    const bool aligned = (reinterpret_cast<uintptr_t>(P.flt) & 15u) == 0 && (sh.K % 4 == 0);
    if (!aligned) return hipErrorNotSupported;
    if (sh.Hf == 3 && sh.Wf == 3 && sh.Ci % 8 == 0) {
        if (P.S <= 256) return launch_fast_t<3, 3, 8, 1>(P, blocks, st);
        if (P.S <= 512) return launch_fast_t<3, 3, 8, 2>(P, blocks, st);
    }
    return hipErrorNotSupported;
}

}  // namespace im2win
