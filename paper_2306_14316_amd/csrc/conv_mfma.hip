// Forward convolution over the im2win tensor on the gfx950 fp32 matrix cores
// (the role of Algorithm 3, Section 3.2-3.3; the design is CDNA4's, not the
// paper's CUDA tiling).
//
// GEMM view (Algorithm 1): M = Co, N = Ni*Ho*Wo (output pixels, flattened in
// NCHW order), K = Ci*Hf*Wf.  A workgroup of 4 waves owns a 64 (M) x 64 (N)
// output tile; each wave owns a 32x32 sub-tile held in 16 accumulator
// registers and advances it with v_mfma_f32_32x32x2_f32.
//
// What the im2win layout buys (Section 3.1; Section 3.3 loads runs of windows that
// belong to one output row): the window of pixel (i,m,n) for channel r is the
// contiguous run What[i][r][m][n*s*Hf .. +Hf*Wf), and neighbouring pixels'
// windows overlap.  So for one channel the tile's 64 pixels need only a few
// contiguous strips of What (about (64*s + rows*(Wf-s))*Hf floats, against
// 64*Hf*Wf for an im2col tile), copied to LDS as they lie in memory.  A lane that
// feeds pixel n to the matrix core keeps ONE LDS base address; window element
// t = v*Hf + u is at base + t, a constant offset per K step -- none of the
// per-step divide/modulo index decoding of Algorithms 1-2.
//
// The two K slices that one MFMA consumes (lanes 0-31 / 32-63) are taken from
// two different channels at the same window element ("pair" steps), so odd
// window sizes (9, 49, 121) cost no padding.  An odd channel left over is
// split in two halves of its window ("split" steps, at most one zero K slice).
// The filter tile is staged to LDS in window order (v outer, u inner) and
// transposed to [k][m], so the A operand is also base + constant per step.
#include "conv_mfma_tile.h"
#include "runtime_cache.h"

#include <limits.h>

namespace im2win {

constexpr int PITCH = 65;    // LDS floats per filter-tile row [k][0..63], +1 against bank conflicts

// VALU_MK: the ablation variant "no matrix cores" (Section 4.4 takes out one optimisation at a
// time).  Tiling, staging and LDS layouts are the same; only the arithmetic differs: in place of
// the wave-level MFMA every thread keeps an M_T x N_T = 4 x 4 register tile of outputs and
// advances it with scalar v_fma_f32 outer products, the micro-kernel of Section 3.3 on the
// vector ALUs.
template <int KHW_T, bool VALU_MK = false>
__global__ __launch_bounds__(256) void conv_mfma_kernel(MfmaParams P)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int khw = KHW_T ? KHW_T : P.khw;
    const int S = P.S;
    int *tbl = reinterpret_cast<int *>(smem);                 // [S]   strip position -> source offset
    int *ftbl = tbl + round4(S);                              // [cb*khw] filter element -> LDS row offset
    float *sI = reinterpret_cast<float *>(ftbl + round4(P.cb * khw));   // [cb][S]
    float *sZero = sI + round4(P.cb * S);                     // [4]  zeros
    float *sF = sZero + 4;                                    // [cb*khw + 1][PITCH]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int h = lane >> 5, l32 = lane & 31;

    const uint32_t lb = xcd_swizzle(blockIdx.x, gridDim.x);
    const uint32_t tile_n = fdiv(lb, P.d_tm);
    const uint32_t tile_m = lb - tile_n * (uint32_t)P.tiles_m;
    const int m0 = (int)tile_m * MB;
    const uint32_t P0 = tile_n * NB;
    const uint32_t Pend = min(P0 + NB - 1, P.npix - 1);

    // ---- geometry of the tile's strips: output rows q0..q1 (q = i*Ho + m) ----
    const uint32_t q0 = fdiv(P0, P.d_wo), q1 = fdiv(Pend, P.d_wo);
    const int nlo0 = (int)(P0 - q0 * (uint32_t)P.Wo);
    const int sHf = P.s * P.Hf;
    const int len0 = (((q1 == q0) ? (int)(Pend - P0) : (P.Wo - 1 - nlo0)) * P.s + P.Wf) * P.Hf;

    int filled = 0;
    for (uint32_t q = q0; q <= q1; ++q) {
        const int rho = (int)(q - q0);
        const int nlo = rho == 0 ? nlo0 : 0;
        const int nhi = (q == q1) ? (int)(Pend - q * (uint32_t)P.Wo) : P.Wo - 1;
        const int seglen = ((nhi - nlo) * P.s + P.Wf) * P.Hf;
        const int segoff = rho == 0 ? 0 : len0 + (rho - 1) * P.fullseg;
        const uint32_t img = fdiv(q, P.d_ho);
        const int mq = (int)(q - img * (uint32_t)P.Ho);
        if (!P.implicit) {
            const int srcbase = (int)((img * (uint32_t)P.Ci * (uint32_t)P.Ho + (uint32_t)mq) * (uint32_t)P.rowlen) + nlo * sHf;
            for (int x = tid; x < seglen; x += 256) tbl[segoff + x] = srcbase + x;
        } else {
            // Workspace-free variant: P.win is the NCHW input.  Strip word kk*Hf + u of this
            // row is input row mq*s + u - p, column nlo*s + kk - p (Eq. 2), or zero padding.
            const int ncol = (nhi - nlo) * P.s + P.Wf;
            const int imgbase = (int)(img * (uint32_t)P.Ci * P.in_plane);
            for (int x = tid; x < seglen; x += 256) {
                const int u = x / ncol, kk = x - u * ncol;
                const int hh = mq * P.s + u - P.p, ww = nlo * P.s + kk - P.p;
                const bool inside = (hh >= 0) & (hh < P.Hi) & (ww >= 0) & (ww < P.Wi);
                tbl[segoff + kk * P.Hf + u] = inside ? imgbase + hh * P.Wi + ww : -1;
            }
        }
        filled = segoff + seglen;
    }
    for (int x = filled + tid; x < S; x += 256) tbl[x] = -1;
    for (int e = tid; e < P.cb * khw; e += 256) {
        const int c = (int)fdiv((uint32_t)e, P.d_khw);
        const int ko = e - c * khw;                 // u*Wf + v  (filter's own order)
        const int u = (int)fdiv((uint32_t)ko, P.d_wf);
        const int v = ko - u * P.Wf;
        ftbl[e] = (c * khw + v * P.Hf + u) * PITCH; // window order: v outer, u inner
    }
    if (tid < 4) sZero[tid] = 0.0f;

    // ---- per-lane operand bases ----
    int b_base;
    {
        const uint32_t Pl = min(P0 + (uint32_t)(wn * 32 + l32), Pend);
        const uint32_t ql = fdiv(Pl, P.d_wo);
        const int nl = (int)(Pl - ql * (uint32_t)P.Wo);
        const int rho = (int)(ql - q0);
        b_base = rho == 0 ? (nl - nlo0) * sHf : len0 + (rho - 1) * P.fullseg + nl * sHf;
    }
    const float *aF = sF + wm * 32 + l32;
    const float *bI = sI + b_base;

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    // register-tile variant: thread (tid / 16, tid % 16) owns output channels 4*(tid/16) .. +3 and
    // pixels 4*(tid%16) .. +3 of the tile; bb[j]: LDS strip position of pixel j's window
    constexpr int MT = 4, NT = 4;
    const int mt0 = (tid >> 4) * MT, nt0 = (tid & 15) * NT;
    int bb[NT];
    float racc[MT][NT];
    if (VALU_MK) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const uint32_t Pl = min(P0 + (uint32_t)(nt0 + j), Pend);
            const uint32_t ql = fdiv(Pl, P.d_wo);
            const int nl = (int)(Pl - ql * (uint32_t)P.Wo);
            const int rho = (int)(ql - q0);
            bb[j] = rho == 0 ? (nl - nlo0) * sHf : len0 + (rho - 1) * P.fullseg + nl * sHf;
#pragma unroll
            for (int i = 0; i < MT; ++i) racc[i][j] = 0.0f;
        }
    }

    for (int c0 = 0; c0 < P.Ci; c0 += P.cb) {
        const int nch = min(P.cb, P.Ci - c0);
        __syncthreads();   // tables ready (first pass) / previous block's reads done

        // ---- stage the im2win strips of nch channels ----
        for (int c = wave; c < nch; c += 4) {
            const float *g = P.win + (size_t)(c0 + c) * (P.implicit ? P.in_plane : P.chan_stride);
            float *d = sI + c * S;
            for (int x = lane; x < S; x += 64) {
                const int off = tbl[x];
                d[x] = off >= 0 ? g[off] : 0.0f;
            }
        }
        // ---- stage the filter tile, transposed to [k in window order][m] ----
        const int ne = nch * khw;
        if (P.vec4) {
            const int cpr = ne >> 2;
            const float *gf = P.flt + (size_t)m0 * P.K + (size_t)c0 * khw;
            for (int f = tid; f < MB * cpr; f += 256) {
                const int row = (int)fdiv((uint32_t)f, P.d_cpr);
                const int e = (f - row * cpr) * 4;
                float4 w = make_float4(0.f, 0.f, 0.f, 0.f);
                if (m0 + row < P.Co) w = *reinterpret_cast<const float4 *>(gf + (size_t)row * P.K + e);
                const int4 r = *reinterpret_cast<const int4 *>(ftbl + e);
                sF[r.x + row] = w.x;
                sF[r.y + row] = w.y;
                sF[r.z + row] = w.z;
                sF[r.w + row] = w.w;
            }
        } else {
            const float *gf = P.flt + (size_t)m0 * P.K + (size_t)c0 * khw;
            for (int row = wave; row < MB; row += 4) {
                const bool live = m0 + row < P.Co;
                for (int e = lane; e < ne; e += 64)
                    sF[ftbl[e] + row] = live ? gf[(size_t)row * P.K + e] : 0.0f;
            }
        }
        if ((nch & 1) && (khw & 1) && tid < MB) sF[ne * PITCH + tid] = 0.0f;   // zero K slice of a split step
        __syncthreads();

        if (VALU_MK) {
            // ---- register-tile micro-kernel: one 4 x 4 outer product per K element ----
            for (int c = 0; c < nch; ++c) {
                const float *ar = sF + (size_t)(c * khw) * PITCH + mt0;
                const float *br = sI + c * S;
#pragma unroll 3
                for (int t = 0; t < khw; ++t) {
                    float a[MT], b[NT];
#pragma unroll
                    for (int i = 0; i < MT; ++i) a[i] = ar[t * PITCH + i];
#pragma unroll
                    for (int j = 0; j < NT; ++j) b[j] = br[bb[j] + t];
#pragma unroll
                    for (int i = 0; i < MT; ++i)
#pragma unroll
                        for (int j = 0; j < NT; ++j) racc[i][j] = fmaf(a[i], b[j], racc[i][j]);
                }
            }
            continue;
        }

        // ---- pair steps: lanes 0-31 take channel 2j, lanes 32-63 channel 2j+1 ----
        const int npairs = nch >> 1;
        for (int pr = 0; pr < npairs; ++pr) {
            const float *bp = bI + (2 * pr + h) * S;
            const float *ap = aF + (2 * pr + h) * khw * PITCH;
            if (KHW_T) {
#pragma unroll
                for (int t = 0; t < KHW_T; ++t)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[t * PITCH], bp[t], acc, 0, 0, 0);
            } else {
#pragma unroll 4
                for (int t = 0; t < khw; ++t)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[t * PITCH], bp[t], acc, 0, 0, 0);
            }
        }
        // ---- split step: the odd channel's window halves go to the two lane halves ----
        if (nch & 1) {
            const int c = nch - 1;
            const int kh2 = (khw + 1) >> 1;
            const float *bp = bI + c * S + h * kh2;
            const float *ap = aF + (c * khw + h * kh2) * PITCH;
#pragma unroll 4
            for (int t = 0; t < kh2 - 1; ++t)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[t * PITCH], bp[t], acc, 0, 0, 0);
            const float *bl = (h && (khw & 1)) ? sZero : bp + (kh2 - 1);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[(kh2 - 1) * PITCH], *bl, acc, 0, 0, 0);
        }
    }

    if (VALU_MK) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const uint32_t Pm = P0 + (uint32_t)(nt0 + j);
            if (Pm > Pend) continue;
            const uint32_t img = fdiv(Pm, P.d_howo);
            float *o = P.out + (size_t)img * P.Co * P.howo + (Pm - img * P.howo);
#pragma unroll
            for (int i = 0; i < MT; ++i)
                if (m0 + mt0 + i < P.Co) o[(size_t)(m0 + mt0 + i) * P.howo] = racc[i][j];
        }
        return;
    }
    store_tile(P, acc, P0, Pend, m0, wm, wn, h, l32);
}

// ---------------------------------------------------------------------------
// Pipelined form of the generic kernel (the double buffer and prefetch of Section 3.3 for the layers
// none of the specialised kernels takes: padded 1x1, filter shapes without an instance of the
// software-pipelined kernel, few channels).  Same tile,
// strip geometry and K order as conv_mfma_kernel, but two LDS stages, and both operands of K block
// kb+1 travel from global memory straight into the other stage (buffer loads with the LDS
// destination in M0: no staging registers, no LDS store instructions) while the matrix cores work
// on block kb.  One barrier per block: it tells that every wave's loads of block kb have landed and
// that every wave has finished reading the stage block kb+1 is about to overwrite.
//   strips: wave w copies channels w, w+4, ... of the block, 64 consecutive LDS words per load, each
//           lane fetching the word its table entry names (the table holds byte offsets from the
//           tile's first strip word; the channel is the scalar offset);
//   filter: the tile stays row-major [m][k] in the filter's own (c, u, v) order with an odd pitch
//           (conflict-free A reads): wave w copies rows w, w+4, ..., 64 consecutive K elements per
//           load -- contiguous in memory and in LDS.  (A [k][m] tile, one lane per filter row, made
//           every load touch 64 cache lines.)  The window-order permutation (u,v) -> (v,u) is an
//           offset on the A read: compile-time for HF_T x WF_T instances, a scalar otherwise.
//           Columns past the block's K elements receive whatever follows in memory and are never
//           read; the column after them is kept at zero for the one zero K slice of a split step.
template <int HF_T, int WF_T>
__global__ __launch_bounds__(256) void conv_mfma_pipe_kernel(MfmaParams P)
{
    extern __shared__ __align__(16) unsigned char smem[];
    typedef __attribute__((address_space(3))) void lds_void;
    const int Hf = HF_T ? HF_T : P.Hf, Wf = WF_T ? WF_T : P.Wf;
    const int khw = Hf * Wf;
    const int SP = P.SP, cb = P.cb;
    const int nkc = (cb * khw + 63) >> 6;                     // 64-element pieces per filter row and block
    const int FP = nkc * 64 + 1;                              // LDS pitch of a filter row (odd); column FP-1 is the zero column
    uint32_t *tbl = reinterpret_cast<uint32_t *>(smem);       // [SP] strip position -> byte offset of its source word
    float *stage0 = reinterpret_cast<float *>(tbl + SP);      // two stages, each: strips [cb][SP], filter tile [MB][FP]
    const int stage_floats = cb * SP + MB * FP;
    float *sZero = stage0 + 2 * stage_floats;                 // [4] zeros

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int h = lane >> 5, l32 = lane & 31;

    const uint32_t lb = xcd_swizzle(blockIdx.x, gridDim.x);
    const uint32_t tile_n = fdiv(lb, P.d_tm);
    const uint32_t tile_m = lb - tile_n * (uint32_t)P.tiles_m;
    const int m0 = (int)tile_m * MB;
    const uint32_t P0 = tile_n * NB;
    const uint32_t Pend = min(P0 + NB - 1, P.npix - 1);

    // ---- geometry of the tile's strips: output rows q0..q1 (q = i*Ho + m) ----
    const uint32_t q0 = fdiv(P0, P.d_wo), q1 = fdiv(Pend, P.d_wo);
    const int nlo0 = (int)(P0 - q0 * (uint32_t)P.Wo);
    const int sHf = P.s * Hf;
    const int len0 = (((q1 == q0) ? (int)(Pend - P0) : (P.Wo - 1 - nlo0)) * P.s + Wf) * Hf;
    const uint32_t img0 = fdiv(q0, P.d_ho);
    const size_t tile_base = ((size_t)img0 * P.Ci * P.Ho + (q0 - img0 * (uint32_t)P.Ho)) * (size_t)P.rowlen + (size_t)(nlo0 * sHf);

    int filled = 0;
    for (uint32_t q = q0; q <= q1; ++q) {
        const int rho = (int)(q - q0);
        const int nlo = rho == 0 ? nlo0 : 0;
        const int nhi = (q == q1) ? (int)(Pend - q * (uint32_t)P.Wo) : P.Wo - 1;
        const int seglen = ((nhi - nlo) * P.s + Wf) * Hf;
        const int segoff = rho == 0 ? 0 : len0 + (rho - 1) * P.fullseg;
        const uint32_t img = fdiv(q, P.d_ho);
        const int mq = (int)(q - img * (uint32_t)P.Ho);
        const size_t src = ((size_t)img * P.Ci * P.Ho + (size_t)mq) * (size_t)P.rowlen + (size_t)(nlo * sHf);
        const uint32_t rel = (uint32_t)(src - tile_base);   // the host checked that a tile's rows span < 4 GiB
        for (int x = tid; x < seglen; x += 256) tbl[segoff + x] = (rel + (uint32_t)x) * 4u;
        filled = segoff + seglen;
    }
    for (int x = filled + tid; x < SP; x += 256) tbl[x] = 0u;   // words no operand uses: any valid source
    if (tid < 4) sZero[tid] = 0.0f;
    if (tid < 2 * MB) stage0[(tid >> 6) * stage_floats + cb * SP + (tid & 63) * FP + FP - 1] = 0.0f;   // zero columns

    // buffer descriptors: the tile's first strip word; the tile's first filter row
    auto desc = [](const float *base, size_t elems) __attribute__((always_inline)) {
        const size_t left = elems * 4u;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(base), 0,
                                                 left < 0xffffffffull ? left : 0xffffffffull, 0x00020000);
    };
    const __amdgpu_buffer_rsrc_t rw = desc(P.win + tile_base, P.win_elems - tile_base);
    const __amdgpu_buffer_rsrc_t rf = desc(P.flt + (size_t)m0 * P.K, ((size_t)P.Co - (size_t)m0) * (size_t)P.K);
    const uint32_t chan_bytes = P.chan_stride * 4u;
    const uint32_t lane4 = (uint32_t)lane * 4u;

    // ---- per-lane operand bases, relative to a stage ----
    int b_base;
    {
        const uint32_t Pl = min(P0 + (uint32_t)(wn * 32 + l32), Pend);
        const uint32_t ql = fdiv(Pl, P.d_wo);
        const int nl = (int)(Pl - ql * (uint32_t)P.Wo);
        const int rho = (int)(ql - q0);
        b_base = rho == 0 ? (nl - nlo0) * sHf : len0 + (rho - 1) * P.fullseg + nl * sHf;
    }
    const int a_base = cb * SP + (wm * 32 + l32) * FP;

    // K block (channels c0 .. c0+nch-1) on its way into stage st
    auto issue = [&](int c0, int nch, int st) __attribute__((always_inline)) {
        float *sI = stage0 + st * stage_floats, *sF = sI + cb * SP;
        for (int c = wave; c < nch; c += 4) {
            const uint32_t soff = (uint32_t)(c0 + c) * chan_bytes;
            for (int x0 = 0; x0 < SP; x0 += 64)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_void *)(sI + c * SP + x0), 4, tbl[x0 + lane], soff, 0, 0);
        }
        const int npc = (nch * khw + 63) >> 6;
        for (int m = wave; m < MB; m += 4) {
            // rows past Co feed accumulators that are never stored: they fetch the last real row
            const uint32_t soff = (uint32_t)(min(m, P.Co - 1 - m0) * P.K + c0 * khw) * 4u;
            for (int kc = 0; kc < npc; ++kc)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rf, (lds_void *)(sF + m * FP + kc * 64), 4, lane4, soff + (uint32_t)kc * 256u, 0, 0);
        }
    };

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    __syncthreads();   // table ready
    issue(0, min(cb, P.Ci), 0);
    int st = 0;
    for (int c0 = 0; c0 < P.Ci; c0 += cb, st ^= 1) {
        const int nch = min(cb, P.Ci - c0);
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's loads of the block have landed
        __syncthreads();
        if (c0 + cb < P.Ci) issue(c0 + cb, min(cb, P.Ci - c0 - cb), st ^ 1);

        const float *sS = stage0 + st * stage_floats;
        const float *aF = sS + a_base;
        const float *bI = sS + b_base;
        // ---- pair steps: lanes 0-31 take channel 2j, lanes 32-63 channel 2j+1 ----
        const int npairs = nch >> 1;
        if constexpr (HF_T == 1 && WF_T == 1) {
            // 1x1, stride 1, a full block of 64 channels: the strip length is 64 and the filter pitch 65, so
            // every operand address is lane base + immediate and the 32 steps unroll into one chain whose
            // LDS reads run ahead of the MFMAs (the loop below waits for two fresh reads before every MFMA).
            if (SP == 64 && cb == 64 && nch == 64) {
                const float *bp = bI + h * 64;
                const float *ap = aF + h;
#pragma unroll
                for (int pr = 0; pr < 32; ++pr)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[2 * pr], bp[2 * pr * 64], acc, 0, 0, 0);
                continue;
            }
        }
        for (int pr = 0; pr < npairs; ++pr) {
            const float *bp = bI + (2 * pr + h) * SP;
            const float *ap = aF + (2 * pr + h) * khw;
            if (HF_T) {
#pragma unroll
                for (int t = 0; t < HF_T * WF_T; ++t)   // window position t = v*Hf + u  <-  filter position u*Wf + v
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[(t % HF_T) * WF_T + t / HF_T], bp[t], acc, 0, 0, 0);
            } else {
                int t = 0;
                for (int v = 0; v < Wf; ++v)
                    for (int u = 0; u < Hf; ++u, ++t)
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[u * Wf + v], bp[t], acc, 0, 0, 0);
            }
        }
        // ---- split step: the odd channel's window halves go to the two lane halves ----
        if (nch & 1) {
            const int c = nch - 1;
            const int kh2 = (khw + 1) >> 1;
            const float *bp = bI + c * SP + h * kh2;
            const float *ap = aF + c * khw;
            int t = h * kh2;                                  // this lane half's window position
            int u = t % Hf, v = t / Hf;                       // (per lane half: vector arithmetic)
            for (int i = 0; i < kh2; ++i, ++t) {
                const bool past = t >= khw;                   // the zero K slice of an odd window (second half's last step)
                const float a = past ? aF[FP - 1] : ap[u * Wf + v];   // (the row's zero column)
                const float b = past ? sZero[0] : bp[i];
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
                if (++u == Hf) { u = 0; ++v; }
            }
        }
    }

    store_tile(P, acc, P0, Pend, m0, wm, wn, h, l32);
}

static size_t lds_bytes_pipe(int cb, int SP, int khw)
{
    const size_t FP = (size_t)((cb * khw + 63) / 64) * 64 + 1;
    return 4u * ((size_t)SP + 2u * ((size_t)cb * SP + (size_t)MB * FP) + 4u);
}

static size_t lds_bytes(int cb, int S, int khw)
{
    return 4u * ((size_t)round4(S) + round4(cb * khw) + round4(cb * S) + 4 + (size_t)(cb * khw + 1) * PITCH);
}

template <int KHW_T, bool VALU_MK = false>
static hipError_t launch_t(const MfmaParams &P, size_t lds, uint32_t blocks, hipStream_t st, LaunchPlan *plan)
{
    if (plan) {
        if (VALU_MK) plan_record(plan, dim3(blocks), 256, lds, "conv_mfma_kernel<%d, true>", KHW_T);
        else plan_record(plan, dim3(blocks), 256, lds, "conv_mfma_kernel<%d, false>", KHW_T);
        return hipSuccess;
    }
    if (lds > 48 * 1024) {
        static KernelCache kc;
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = allow_dynamic_lds(kc, reinterpret_cast<const void *>(&conv_mfma_kernel<KHW_T, VALU_MK>), lds, dev);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((conv_mfma_kernel<KHW_T, VALU_MK>), dim3(blocks), dim3(256), lds, st, P);
    return hipGetLastError();
}

// Tile-independent kernel parameters of a layer (everything but the generic kernel's K block).
// Returns false when the layer is outside what the tiled kernels index with 32-bit integers or
// stage in LDS (a tile's strips of one channel would not fit): the caller then takes the
// one-thread-per-output kernel, which handles any legal shape.
static bool fill_params(MfmaParams &P, const float *win, const float *flt, float *out, const Shape &sh)
{
    P.win = win; P.flt = flt; P.out = out;
    P.Ci = sh.Ci; P.Ho = sh.Ho; P.Wo = sh.Wo; P.Co = sh.Co; P.Hf = sh.Hf; P.Wf = sh.Wf; P.s = sh.s;
    P.rowlen = sh.rowlen; P.khw = sh.khw; P.K = sh.K;
    P.npix = (uint32_t)sh.npix;
    P.howo = (uint32_t)(sh.Ho * sh.Wo);
    P.chan_stride = (uint32_t)((size_t)sh.Ho * sh.rowlen);
    P.win_elems = (size_t)sh.N * sh.Ci * sh.Ho * (size_t)sh.rowlen;
    P.out_elems = (size_t)sh.npix * sh.Co;
    P.implicit = 0;
    P.Hi = sh.Hi; P.Wi = sh.Wi; P.p = sh.p;
    P.in_plane = (uint32_t)(sh.Hi * sh.Wi);
    P.tiles_m = (sh.Co + MB - 1) / MB;

    // Strip floats per channel: NB pixels over R output rows take ((NB - R)*s + R*Wf)*Hf floats.
    // With overlapping windows (s < Wf) that grows with R, at most rmax rows; otherwise it is
    // largest for the fewest rows NB pixels can lie in.  In 64 bits: the stride has no upper bound.
    int rmax = (NB + sh.Wo - 2) / sh.Wo + 1;
    if (rmax > NB) rmax = NB;
    const int rmin = (NB + sh.Wo - 1) / sh.Wo;
    const long long R = sh.s < sh.Wf ? rmax : rmin;
    const long long S = ((NB - R) * (long long)sh.s + R * sh.Wf) * sh.Hf + 1;
    const long long fullseg = ((long long)(sh.Wo - 1) * sh.s + sh.Wf) * sh.Hf;
    const long long step = (long long)sh.s * sh.Hf;   // floats between neighbouring windows
    if (S > 160 * 1024 / 4 || fullseg > INT_MAX || step * sh.Wo > INT_MAX) return false;
    P.fullseg = (int)fullseg;
    P.S = (int)S;
    P.rmax = rmax;
    P.SP = (int)((S - 1 + 63) & ~63LL);   // (the strips themselves take at most S - 1 floats)
    if (P.SP < 64) P.SP = 64;
    P.cb = 0;
    P.vec4 = 0;
    P.nblocks = 0; P.nmain = 0; P.nhalf = 0; P.tail_at = 0;
    P.d_wo = make_fastdiv((uint32_t)sh.Wo);
    P.d_ho = make_fastdiv((uint32_t)sh.Ho);
    P.d_howo = make_fastdiv(P.howo);
    P.d_khw = make_fastdiv((uint32_t)sh.khw);
    P.d_wf = make_fastdiv((uint32_t)sh.Wf);
    P.d_cpr = make_fastdiv(1);
    P.d_tm = make_fastdiv((uint32_t)P.tiles_m);
    return true;
}

// The generic kernel: picks the channels per K block that fit in LDS and launches.
static hipError_t launch_generic(MfmaParams &P, const Shape &sh, uint32_t blocks, hipStream_t st, LaunchPlan *plan,
                                 bool valu_microkernel = false)
{
    const size_t lds_max = 160 * 1024;
    int cb = sh.Ci < 8 ? sh.Ci : 8;
    while (cb > 1 && lds_bytes(cb, P.S, sh.khw) > lds_max) cb = (cb > 2) ? (((cb / 2) & ~1) < 2 ? 2 : ((cb / 2) & ~1)) : 1;
    if (lds_bytes(cb, P.S, sh.khw) > lds_max) return hipErrorInvalidConfiguration;
    P.cb = cb;
    const size_t lds = lds_bytes(cb, P.S, sh.khw);
    P.vec4 = (sh.Ci % cb == 0) && ((cb * sh.khw) % 4 == 0) && (sh.K % 4 == 0) &&
             ((reinterpret_cast<uintptr_t>(P.flt) & 15u) == 0);
    P.d_cpr = make_fastdiv((uint32_t)((cb * sh.khw) / 4 > 0 ? (cb * sh.khw) / 4 : 1));
    if (valu_microkernel) return sh.khw == 9 ? launch_t<9, true>(P, lds, blocks, st, plan) : launch_t<0, true>(P, lds, blocks, st, plan);
    switch (sh.khw) {
        case 9:   return launch_t<9>(P, lds, blocks, st, plan);
        case 49:  return launch_t<49>(P, lds, blocks, st, plan);
        case 121: return launch_t<121>(P, lds, blocks, st, plan);
        default:  return launch_t<0>(P, lds, blocks, st, plan);
    }
}

template <int HF_T, int WF_T>
static hipError_t launch_pipe_t(const MfmaParams &P, size_t lds, uint32_t blocks, hipStream_t st, LaunchPlan *plan)
{
    if (plan) { plan_record(plan, dim3(blocks), 256, lds, "conv_mfma_pipe_kernel<%d, %d>", HF_T, WF_T); return hipSuccess; }
    static KernelCache kc;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = allow_dynamic_lds(kc, reinterpret_cast<const void *>(&conv_mfma_pipe_kernel<HF_T, WF_T>), lds, dev);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((conv_mfma_pipe_kernel<HF_T, WF_T>), dim3(blocks), dim3(256), lds, st, P);
    return hipGetLastError();
}

// The pipelined generic kernel.  hipErrorNotSupported when a tile's strips or filter rows are out
// of reach of 32-bit byte offsets or two stages do not fit in LDS: the single-stage kernel then.
static hipError_t launch_generic_pipe(MfmaParams &P, const Shape &sh, uint32_t blocks, hipStream_t st, LaunchPlan *plan)
{
    const unsigned long long img_bytes = (unsigned long long)sh.Ci * sh.Ho * (unsigned long long)sh.rowlen * 4ull;
    if (img_bytes * (unsigned long long)(P.rmax + 1) >= (1ull << 32)) return hipErrorNotSupported;
    if ((unsigned long long)sh.K * 4ull * MB >= (1ull << 32)) return hipErrorNotSupported;
    // channels per K block: as many as give at most 64 K elements (one 64-element piece per filter
    // row and block), an even count where the layer has two or more; large windows take two channels,
    // or one where two stages would not fit otherwise
    int cb = 64 / sh.khw;
    cb &= ~1;
    if (cb < 2) cb = 2;
    if (cb > sh.Ci) cb = sh.Ci;
    if (cb == 2 && lds_bytes_pipe(2, P.SP, sh.khw) > 100 * 1024) cb = 1;
    const size_t lds = lds_bytes_pipe(cb, P.SP, sh.khw);
    if (lds > 160 * 1024) return hipErrorNotSupported;
    // Two stages cost LDS, hence resident workgroups, and with few K blocks there is little to overlap:
    // measured against the single-stage kernel the pipeline pays from about four blocks on (1x1 with
    // 256 and 512 channels +19-21 %, 4x4 stride 2 +52 %, 7x1 +21 %; a 64-channel 1x1 layer, one block,
    // -9 %; 3x3 with four channels -24 %).
    if ((sh.Ci + cb - 1) / cb < 4) return hipErrorNotSupported;
    P.cb = cb;
    if (sh.Hf == 1 && sh.Wf == 1) return launch_pipe_t<1, 1>(P, lds, blocks, st, plan);
    if (sh.Hf == 3 && sh.Wf == 3) return launch_pipe_t<3, 3>(P, lds, blocks, st, plan);
    return launch_pipe_t<0, 0>(P, lds, blocks, st, plan);
}

// Workspace-free convolution straight from the NCHW input: the pipelined kernel where the
// layer fits it, the generic kernel otherwise; a layer neither can tile (see fill_params; a
// window too large for the LDS filter tile) is computed by the direct one-thread-per-output kernel.
hipError_t launch_conv_implicit(const float *in, const float *flt, float *out, const Shape &sh,
                                hipStream_t st, LaunchPlan *plan)
{
    MfmaParams P;
    if (!fill_params(P, in, flt, out, sh)) return launch_conv_direct(in, flt, out, sh, st, plan);
    P.implicit = 1;
    P.win_elems = (size_t)sh.N * sh.Ci * sh.Hi * (size_t)sh.Wi;   // the tensor P.win points at is the input
    const uint32_t blocks = ((P.npix + NB - 1) / NB) * (uint32_t)P.tiles_m;
    hipError_t fe = launch_conv_mfma_shallow(in, flt, out, sh, st, true, plan);
    if (fe != hipErrorNotSupported) return fe;
    fe = launch_conv_mfma_fast(P, sh, blocks, st, true, 4, plan);
    if (fe != hipErrorNotSupported) return fe;
    fe = launch_conv_mfma_1x1(in, flt, out, sh, st, true, plan);
    if (fe != hipErrorNotSupported) return fe;
    fe = launch_generic(P, sh, blocks, st, plan);
    if (fe == hipErrorInvalidConfiguration) return launch_conv_direct(in, flt, out, sh, st, plan);
    return fe;
}

hipError_t launch_conv_mfma(const float *win, const float *flt, float *out, const Shape &sh,
                            hipStream_t st, int variant, LaunchPlan *plan)
{
    if (variant == kVariantNoMfma) return launch_conv_basic(win, flt, out, sh, st, plan);
    MfmaParams P;
    if (!fill_params(P, win, flt, out, sh)) return launch_conv_basic(win, flt, out, sh, st, plan);

    const uint32_t tiles_n = (P.npix + NB - 1) / NB;
    const uint32_t blocks = tiles_n * (uint32_t)P.tiles_m;
    if (variant == kVariantDefault || variant == kVariantNarrowLoads || variant == kVariantScalarLoads) {
        hipError_t fe = launch_conv_mfma_shallow(win, flt, out, sh, st, false, plan);
        if (fe != hipErrorNotSupported) return fe;
        fe = launch_conv_mfma_fast(P, sh, blocks, st, false,
                                   variant == kVariantNarrowLoads ? 2 : (variant == kVariantScalarLoads ? 1 : 4), plan);
        if (fe != hipErrorNotSupported) return fe;
    }
    if (variant == kVariantDefault) {
        const hipError_t oe = launch_conv_mfma_1x1(win, flt, out, sh, st, false, plan);
        if (oe != hipErrorNotSupported) return oe;
        const hipError_t pe = launch_generic_pipe(P, sh, blocks, st, plan);
        if (pe != hipErrorNotSupported) return pe;
    }
    // (a window too large for the generic kernel's LDS filter tile: the basic kernel computes it)
    const hipError_t ge = launch_generic(P, sh, blocks, st, plan, variant == kVariantValuMicrokernel);
    if (ge == hipErrorInvalidConfiguration) return launch_conv_basic(win, flt, out, sh, st, plan);
    return ge;
}

}  // namespace im2win
