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

typedef __attribute__((address_space(3))) float lds_float;   // a float in LDS

template <int HF, int WF, int CB, int JX>
__global__ __launch_bounds__(256) void conv_mfma_fast_kernel(MfmaParams P)
{
    constexpr int KHW = HF * WF;
    constexpr int KB = CB * KHW;            // K elements per block
    constexpr int CPR = KB / 4;             // float4 chunks per filter row per block
    constexpr int NF4 = MB * CPR;
    constexpr int JF = (NF4 + 255) / 256;   // float4 chunks per thread
    constexpr int PF = KB | 1;              // odd LDS pitch of a filter row
    constexpr int SS = 256 * JX;            // LDS floats per channel strip (compile-time stride)
    constexpr int SF_FLOATS = (MB * PF + 3) & ~3;
    constexpr int STAGE = SF_FLOATS + CB * SS;   // floats per LDS stage
    static_assert(KB % 4 == 0, "K block must be a multiple of 4 floats");
    static_assert(CB % 2 == 0, "pair steps need an even channel count");

    // two LDS stages, each [filter tile MB x PF][CB strips of SS floats]
    extern __shared__ __align__(16) unsigned char smem[];
    float *lds = reinterpret_cast<float *>(smem);

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

    // Byte offset (from the channel plane) of strip word tid + 256*j.  Words past
    // the tile's segments are never used as operands; they reload word 0.
    uint32_t soffb[JX];
#pragma unroll
    for (int j = 0; j < JX; ++j) soffb[j] = 0;
    for (uint32_t q = q0; q <= q1; ++q) {
        const int rho = (int)(q - q0);
        const int nlo = rho == 0 ? nlo0 : 0;
        const int nhi = (q == q1) ? (int)(Pend - q * (uint32_t)P.Wo) : P.Wo - 1;
        const int seglen = ((nhi - nlo) * P.s + WF) * HF;
        const int segoff = rho == 0 ? 0 : len0 + (rho - 1) * P.fullseg;
        const uint32_t img = fdiv(q, P.d_ho);
        const int mq = (int)(q - img * (uint32_t)P.Ho);
        const uint32_t srcbase = (img * (uint32_t)P.Ci * (uint32_t)P.Ho + (uint32_t)mq) * (uint32_t)P.rowlen + (uint32_t)(nlo * sHf);
#pragma unroll
        for (int j = 0; j < JX; ++j) {
            const int x = tid + 256 * j - segoff;
            if (x >= 0 && x < seglen) soffb[j] = (srcbase + (uint32_t)x) * 4u;
        }
    }

    // ---- filter staging coordinates of this thread's float4 chunks ----
    // Rows past Co feed accumulators that are never stored; they reload row 0.
    uint32_t goffb[JF];
    int loff[JF];
#pragma unroll
    for (int j = 0; j < JF; ++j) {
        const int f = tid + 256 * j;
        const int row = f / CPR;
        const int e = (f - row * CPR) * 4;
        const bool live = (f < NF4) && (m0 + row < P.Co);
        goffb[j] = live ? (uint32_t)(row * P.K + e) * 4u : 0u;
        loff[j] = (f < NF4) ? row * PF + e : -1;
    }

    // ---- per-lane operand bases (stage 0) ----
    int b_base;
    {
        const uint32_t Pl = min(P0 + (uint32_t)(wn * 32 + l32), Pend);
        const uint32_t ql = fdiv(Pl, P.d_wo);
        const int nl = (int)(Pl - ql * (uint32_t)P.Wo);
        const int rho = (int)(ql - q0);
        b_base = rho == 0 ? (nl - nlo0) * sHf : len0 + (rho - 1) * P.fullseg + nl * sHf;
    }
    const lds_float *ap0 = (const lds_float *)lds + (wm * 32 + l32) * PF + h * KHW;
    const lds_float *bp0 = (const lds_float *)lds + SF_FLOATS + b_base + h * SS;
    float *wI0 = lds + SF_FLOATS + tid;

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    float4 fr[JF];
    float ir[CB * JX];
    // Wave-uniform bases (kept in scalar registers) plus per-thread 32-bit byte
    // offsets that never change: the K loop spends no vector ALU work on addresses.
    const char *gf = reinterpret_cast<const char *>(P.flt + (size_t)m0 * P.K);
    const char *gw = reinterpret_cast<const char *>(P.win);
    const size_t plane_bytes = (size_t)P.chan_stride * 4u;

    // All loads of a block are issued back to back with no use of their values,
    // so they stay in flight until the block is written to LDS one iteration later.
    auto gload = [&](int kb) {
        const char *gfb = gf + (size_t)kb * (KB * 4);
#pragma unroll
        for (int j = 0; j < JF; ++j) fr[j] = *reinterpret_cast<const float4 *>(gfb + goffb[j]);
        const char *gwb = gw + (size_t)kb * CB * plane_bytes;
#pragma unroll
        for (int c = 0; c < CB; ++c) {
#pragma unroll
            for (int j = 0; j < JX; ++j)
                ir[c * JX + j] = *reinterpret_cast<const float *>(gwb + c * plane_bytes + soffb[j]);
        }
    };

    // registers -> LDS stage st (st is a compile-time constant at every call site)
    auto lds_store = [&](int st) {
        float *sF = lds + st * STAGE;
        float *sI = wI0 + st * STAGE;
#pragma unroll
        for (int j = 0; j < JF; ++j) {
            if ((j + 1) * 256 <= NF4 || loff[j] >= 0) {
                float *d = sF + loff[j];
                d[0] = fr[j].x; d[1] = fr[j].y; d[2] = fr[j].z; d[3] = fr[j].w;
            }
        }
#pragma unroll
        for (int c = 0; c < CB; ++c)
#pragma unroll
            for (int j = 0; j < JX; ++j) sI[c * SS + 256 * j] = ir[c * JX + j];
    };

    float a[2][KHW], b[2][KHW];
    auto lds_ops = [&](int st, int pr, int slot) {
        const lds_float *a2 = ap0 + st * STAGE + 2 * pr * KHW;
        const lds_float *b2 = bp0 + st * STAGE + 2 * pr * SS;
#pragma unroll
        for (int v = 0; v < WF; ++v)
#pragma unroll
            for (int u = 0; u < HF; ++u) {
                // volatile: keeps these as single-dword LDS reads with 16-bit immediate
                // offsets; merged two-address reads would need a VALU add each for
                // their 8-bit offsets, and VALU work comes out of the MFMA rate.
                a[slot][v * HF + u] = *(const volatile lds_float *)(a2 + u * WF + v);   // filter (u,v) -> window order
                b[slot][v * HF + u] = *(const volatile lds_float *)(b2 + v * HF + u);
            }
    };

    // One K block: the matrix cores work out of LDS stage st while block kb+1
    // moves from registers into the other stage and block kb+2 is requested from
    // global memory.  One barrier per block.
    const int nkb = P.Ci / CB;
    auto block = [&](int kb, int st) {
        lds_ops(st, 0, 0);
#pragma unroll
        for (int pr = 0; pr < CB / 2; ++pr) {
            if (pr + 1 < CB / 2) lds_ops(st, pr + 1, (pr + 1) & 1);
            if (pr == 0) {
                if (kb + 1 < nkb) lds_store(st ^ 1);
                if (kb + 2 < nkb) gload(kb + 2);
            }
#pragma unroll
            for (int t = 0; t < KHW; ++t)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[pr & 1][t], b[pr & 1][t], acc, 0, 0, 0);
        }
        __syncthreads();
    };

    gload(0);
    lds_store(0);
    if (nkb > 1) gload(1);
    __syncthreads();
    int kb = 0;
    for (; kb + 1 < nkb; kb += 2) {   // unrolled by two so that the stage is a constant
        block(kb, 0);
        block(kb + 1, 1);
    }
    if (kb < nkb) block(kb, 0);

    store_tile(P, acc, P0, Pend, m0, wm, wn, h, l32);
}

template <int HF, int WF, int CB, int JX>
static hipError_t launch_fast_t(const MfmaParams &P, uint32_t blocks, hipStream_t st)
{
    constexpr int KB = CB * HF * WF;
    constexpr int PF = KB | 1;
    constexpr size_t lds = 2u * 4u * (size_t)(((MB * PF + 3) & ~3) + CB * 256 * JX);
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
