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

#include <type_traits>

namespace im2win {

typedef __attribute__((address_space(3))) float lds_float;   // a float in LDS

template <int HF, int WF, int CB, int JX>
__global__ __launch_bounds__(256, 3) void conv_mfma_fast_kernel(MfmaParams P)
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
    // The tile is MB rows x CPR chunks of 4 floats.  Chunk columns are dealt out
    // so that each dword LDS write of a half-wave is conflict-free with the odd
    // row pitch: columns in groups of 8 (a half-wave = 4 consecutive rows x 8
    // chunks: 128 contiguous bytes per row in global memory), the CPR % 8
    // leftover columns one column x 32 rows per half-wave.
    // Rows past Co feed accumulators that are never stored; they reload row 0.
    constexpr int CG = CPR / 8;              // full groups of 8 chunk columns
    constexpr int NMAIN = MB * CG * 8;       // chunks in full groups
    uint32_t goffb[JF];
    int loff[JF];
#pragma unroll
    for (int j = 0; j < JF; ++j) {
        const int f = tid + 256 * j;
        int row, c4;
        if (f < NMAIN) {
            const int g = f >> 5, w = f & 31;
            row = 4 * (g / CG) + (w >> 3);
            c4 = 8 * (g % CG) + (w & 7);
        } else {
            const int r = f - NMAIN;
            row = r % MB;
            c4 = CG * 8 + r / MB;
        }
        const int e = c4 * 4;
        const bool live = (f < NF4) && (m0 + row < P.Co);
        goffb[j] = live ? (uint32_t)(row * P.K + e) * 4u : 0u;
        loff[j] = row * PF + e;
    }
    // A thread with no chunk in the last round repeats its first chunk (same data to
    // the same place), which keeps the staging code free of branches.
    if (tid + 256 * (JF - 1) >= NF4) { goffb[JF - 1] = goffb[0]; loff[JF - 1] = loff[0]; }

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

    // Prefetch registers: one set for the filter chunks (they come from L2), two
    // alternating sets for the strip words (they come from HBM and are given about
    // one and a half K blocks to arrive).
    float4 fr[JF];
    float ir[2][CB * JX];
    // Wave-uniform bases (kept in scalar registers) plus per-thread 32-bit byte
    // offsets that never change: the K loop spends no vector ALU work on addresses.
    const char *gf = reinterpret_cast<const char *>(P.flt + (size_t)m0 * P.K);
    const char *gw = reinterpret_cast<const char *>(P.win);
    const size_t plane_bytes = (size_t)P.chan_stride * 4u;

    auto load_f = [&](int kb, int j) {
        fr[j] = *reinterpret_cast<const float4 *>(gf + (size_t)kb * (KB * 4) + goffb[j]);
    };
    auto load_i = [&](int kb, int set, int c, int j) {
        ir[set][c * JX + j] = *reinterpret_cast<const float *>(gw + ((size_t)kb * CB + c) * plane_bytes + soffb[j]);
    };
    auto store_f = [&](int st, int j, int half) {   // half 0: words 0,1 of the chunk; half 1: words 2,3
        lds_float *d = (lds_float *)lds + st * STAGE + loff[j] + 2 * half;
        d[0] = half ? fr[j].z : fr[j].x;
        d[1] = half ? fr[j].w : fr[j].y;
    };
    auto store_i = [&](int st, int set, int c, int j) {
        ((lds_float *)wI0)[st * STAGE + c * SS + 256 * j] = ir[set][c * JX + j];
    };

    float a[2][KHW], b[2][KHW];
    // operand pair t of channel pair pr, from LDS stage st, into register slot `slot`
    auto lds_op = [&](int st, int pr, int slot, int t) {
        const int u = t % HF, v = t / HF;   // window order: v outer, u inner; the filter is stored (u,v)
        // volatile: keeps these as single-dword LDS reads with 16-bit immediate
        // offsets; merged two-address reads would need a VALU add each for
        // their 8-bit offsets, and VALU work comes out of the MFMA rate.
        a[slot][t] = *(const volatile lds_float *)(ap0 + st * STAGE + 2 * pr * KHW + u * WF + v);
        b[slot][t] = *(const volatile lds_float *)(bp0 + st * STAGE + 2 * pr * SS + t);
    };

    // ---- one K block --------------------------------------------------------------
    // The wave issues its MFMAs as one dependent chain, so everything else is
    // placed, in program order, in the shadow of an MFMA: after MFMA i come the two
    // operand reads for the same step of the next channel pair and one or two
    // staging instructions.  Block kb computes out of LDS stage ST, writes block
    // kb+1 (held in registers) to the other stage and requests block kb+2 from
    // global memory.  The barrier sits before the last channel pair: its operands
    // are already in registers, so after the barrier the other stage can be read
    // (first operands of block kb+1) and, in the next block, this stage can be
    // overwritten.  Scheduling barriers pin this order.
    constexpr int NG = CB / 2;            // channel pairs per block
    constexpr int NM = NG * KHW;          // MFMAs per block
    constexpr int NSLOT = (NG - 1) * KHW; // MFMAs before the barrier
    constexpr int NFW = 2 * JF;           // filter half-chunk stores
    constexpr int NIW = CB * JX;          // strip stores / loads
    static_assert(NG % 2 == 0, "operand slots alternate per channel pair");
    constexpr int NIWS = (NIW + 1) / 2;                       // slots that store strip words (two each)
    constexpr int LPS = (NIW + (NSLOT - NFW - NIWS) - 1) / (NSLOT - NFW - NIWS);   // strip loads per slot
    constexpr int NILS = (NIW + LPS - 1) / LPS;               // slots that load strip words
    static_assert(NSLOT - NFW - NIWS > 0 && NFW + NIWS + NILS <= NSLOT, "staging work must fit before the barrier");
    const int nkb = P.Ci / CB;
    auto block = [&](int kb, auto stc, auto has1c, auto has2c) {
        constexpr int ST = decltype(stc)::value;
        constexpr bool HAS1 = decltype(has1c)::value, HAS2 = decltype(has2c)::value;
#pragma unroll
        for (int i = 0; i < NM; ++i) {
            const int g = i / KHW, t = i % KHW;
            if (HAS1 && i == NSLOT) __syncthreads();
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g & 1][t], b[g & 1][t], acc, 0, 0, 0);
            if (g + 1 < NG) lds_op(ST, g + 1, (g + 1) & 1, t);
            else if (HAS1) lds_op(ST ^ 1, 0, 0, t);
            if (i < NFW) {                       // filter chunk i/2: store a half, then reload it
                if (HAS1) store_f(ST ^ 1, i / 2, i & 1);
                if (HAS2 && (i & 1)) load_f(kb + 2, i / 2);
            } else if (i < NFW + NIWS) {   // strip words of block kb+1: two stores per slot
                if (HAS1) {
                    const int w = 2 * (i - NFW);
                    store_i(ST ^ 1, ST ^ 1, w / JX, w % JX);
                    if (w + 1 < NIW) store_i(ST ^ 1, ST ^ 1, (w + 1) / JX, (w + 1) % JX);
                }
            } else if (i < NFW + NIWS + NILS) {   // strip words of block kb+2: LPS loads per slot
                if (HAS2) {
#pragma unroll
                    for (int q = 0; q < LPS; ++q) {
                        const int w = (i - NFW - NIWS) * LPS + q;
                        if (w < NIW) load_i(kb + 2, ST, w / JX, w % JX);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using T = std::true_type;
    using F = std::false_type;

    // ---- prologue: block 0 into stage 0, block 1 into the registers ----
#pragma unroll
    for (int j = 0; j < JF; ++j) load_f(0, j);
#pragma unroll
    for (int w = 0; w < NIW; ++w) load_i(0, 0, w / JX, w % JX);
#pragma unroll
    for (int j = 0; j < JF; ++j) { store_f(0, j, 0); store_f(0, j, 1); }
#pragma unroll
    for (int w = 0; w < NIW; ++w) store_i(0, 0, w / JX, w % JX);
    if (nkb > 1) {
#pragma unroll
        for (int j = 0; j < JF; ++j) load_f(1, j);
#pragma unroll
        for (int w = 0; w < NIW; ++w) load_i(1, 1, w / JX, w % JX);
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < KHW; ++t) lds_op(0, 0, 0, t);

    int kb = 0;
    for (; kb + 3 < nkb; kb += 2) {   // unrolled by two so that the stage is a constant
        block(kb, I0{}, T{}, T{});
        block(kb + 1, I1{}, T{}, T{});
    }
    const int rem = nkb - kb;   // 1, 2 or 3 blocks left
    if (rem == 3) {
        block(kb, I0{}, T{}, T{});
        block(kb + 1, I1{}, T{}, F{});
        block(kb + 2, I0{}, F{}, F{});
    } else if (rem == 2) {
        block(kb, I0{}, T{}, F{});
        block(kb + 1, I1{}, F{}, F{});
    } else {
        block(kb, I0{}, F{}, F{});
    }

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
    // strip words are addressed with 32-bit byte offsets from the start of the im2win tensor
    if ((unsigned long long)sh.N * sh.Ci * sh.Ho * (unsigned long long)sh.rowlen * 4ull >= (1ull << 32)) return hipErrorNotSupported;
    if (sh.Hf == 3 && sh.Wf == 3 && sh.Ci % 8 == 0) {
        if (P.S <= 256) return launch_fast_t<3, 3, 8, 1>(P, blocks, st);
        if (P.S <= 512) return launch_fast_t<3, 3, 8, 2>(P, blocks, st);
    }
    return hipErrorNotSupported;
}

}  // namespace im2win
