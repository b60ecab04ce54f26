// Software-pipelined MFMA im2win convolution for layers with many input
// channels and a compile-time filter (3x3, 5x5, 7x7: all multi-channel layers of
// the paper's Table 2; also 1x7, 7x1, 1x3, 3x1, 2x2 and 4x4).  Same 64x64 tile, strip geometry and pair-step K order
// as conv_mfma.hip; what differs:
//   - the filter shape and the channels per K block are template constants,
//     so every LDS operand address is base + immediate and all staging
//     coordinates are computed once per thread, before the K loop;
//   - the next K blocks' global loads (filter rows as 16- or 8-byte chunks,
//     strip words) are issued into registers during the current block's MFMAs
//     and written to the other LDS stage one block later (the prefetch /
//     double-buffer idea of Section 3.3, done in registers), so global latency
//     overlaps the matrix work;
//   - the filter tile stays row-major [m][k] in LDS with an odd pitch, which
//     makes both the staging writes and the A-operand reads conflict-free; the
//     (u,v) -> window-order permutation is a compile-time offset on the read;
//   - every non-MFMA instruction of the K loop is placed, in program order,
//     between two MFMAs of the wave's dependent chain, where it issues for free.
#include "conv_mfma_tile.h"
#include "runtime_cache.h"

#include <type_traits>

namespace im2win {

typedef __attribute__((address_space(3))) float lds_float;   // a float in LDS
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float2v __attribute__((ext_vector_type(2)));

// MFMA operands are read from LDS R steps ahead, through a ring of R register
// pairs; R divides the MFMAs per K block so that ring positions line up from one
// block to the next.
constexpr int pick_ring(int nm)
{
    const int cand[] = {9, 10, 8, 7, 11, 12, 6, 5};
    for (int r : cand)
        if (nm % r == 0) return r;
    return 0;
}
// ... and, where half tiles run half of a block's MFMAs per wave, half of that count too.
constexpr int pick_ring_half(int nm)
{
    const int cand[] = {9, 10, 8, 7, 11, 12, 6, 5};
    for (int r : cand)
        if (nm % 2 == 0 && nm % r == 0 && (nm / 2) % r == 0) return r;
    return 0;
}

// ---- leftover tiles: sixteen 16x16 pieces per tile ------------------------------------------
// A workgroup alone on a compute unit already keeps all four matrix pipes busy, so when fewer
// tiles than compute units are left after the last full round of the grid they take a whole
// tile time while most of the chip idles.  Each of those tiles is cut into sixteen 16x16
// output pieces, one workgroup each (v_mfma_f32_16x16x4_f32), and inside the workgroup the four
// waves split the channels: wave w multiplies channels [w*Ci/4, (w+1)*Ci/4) and the four partial
// sums are added in a fixed order through LDS.  The waves share no operand, so nothing is
// staged in LDS and the K loop has no barrier: a lane's filter taps of one channel and its
// pixel's window of one channel are both contiguous runs in memory (the window order of
// Section 3.1), read straight into registers D channel groups ahead.  A piece lasts one cold
// load latency plus its MFMA chain: sixteenths keep the chain short and, for 64 channels, have
// every load in flight at once (32x32 quadrants with the same wave split exposed a second load
// latency and gained nothing).
typedef float floatx4 __attribute__((ext_vector_type(4)));

template <int HF, int WF, bool IMP>
__device__ __forceinline__ void tail_piece(const MfmaParams &P, uint32_t lt, int piece, float *lds,
                                           int lane, int wave)
{
    constexpr int KHW = HF * WF;
    constexpr int D = 7;   // channel groups (four channels each) in flight per wave
    const int kq = lane >> 4, l16 = lane & 15;   // the lane's channel within a group, its row / pixel
    const int sm = piece & 3, sn = piece >> 2;
    const uint32_t tile_n = fdiv(lt, P.d_tm);
    const uint32_t tile_m = lt - tile_n * (uint32_t)P.tiles_m;
    const uint32_t P0 = tile_n * NB;
    const uint32_t Pend = min(P0 + NB - 1, P.npix - 1);
    const int mq = (int)tile_m * MB + sm * 16;      // first output channel of the piece
    const uint32_t Pq = P0 + (uint32_t)(sn * 16);   // its first pixel
    if (mq >= P.Co || Pq > Pend) return;            // nothing of this piece exists (whole workgroup)

    auto desc = [](const float *base, size_t elems) __attribute__((always_inline)) {
        const size_t left = elems * 4u;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(base), 0,
                                                 left < 0xffffffffull ? left : 0xffffffffull, 0x00020000);
    };
    // filter: descriptor on the piece's rows; the lane reads row l16 (rows past Co repeat the
    // last one, their sums are never stored), channel kq of each group
    const __amdgpu_buffer_rsrc_t rf = desc(P.flt + (size_t)mq * P.K, ((size_t)P.Co - (size_t)mq) * (size_t)P.K);
    const uint32_t voffA = (uint32_t)(min(l16, P.Co - 1 - mq) * P.K + kq * KHW) * 4u;

    // pixels: descriptor on the first pixel's window (its image in the workspace-free variant);
    // the lane's pixel (pixels past the tile's last one repeat it, never stored)
    const uint32_t q0 = fdiv(Pq, P.d_wo), img0 = fdiv(q0, P.d_ho);
    const uint32_t Pl = min(Pq + (uint32_t)l16, Pend);
    const uint32_t ql = fdiv(Pl, P.d_wo), imgl = fdiv(ql, P.d_ho);
    const int nl = (int)(Pl - ql * (uint32_t)P.Wo), ml = (int)(ql - imgl * (uint32_t)P.Ho);
    const uint32_t plane_bytes = (IMP ? P.in_plane : P.chan_stride) * 4u;
    size_t base_off;
    uint32_t voffB[IMP ? KHW : 1];
    uint32_t inside = 0;   // workspace-free variant: bit t set when window element t lies in the image
    if (!IMP) {
        const int n0 = (int)(Pq - q0 * (uint32_t)P.Wo), mm0 = (int)(q0 - img0 * (uint32_t)P.Ho);
        base_off = ((size_t)img0 * P.Ci * P.Ho + (size_t)mm0) * (size_t)P.rowlen + (size_t)(n0 * P.s * HF);
        const size_t offl = ((size_t)imgl * P.Ci * P.Ho + (size_t)ml) * (size_t)P.rowlen + (size_t)(nl * P.s * HF);
        voffB[0] = (uint32_t)(offl - base_off) * 4u + (uint32_t)kq * plane_bytes;   // host: a tile's rows span < 4 GiB
    } else {
        base_off = (size_t)img0 * P.Ci * P.in_plane;
        const uint32_t rel = (imgl - img0) * (uint32_t)P.Ci * P.in_plane;           // host: a tile's images span < 4 GiB
#pragma unroll
        for (int t = 0; t < KHW; ++t) {
            const int u = t % HF, v = t / HF;
            const int hh = ml * P.s + u - P.p, ww = nl * P.s + v - P.p;
            const bool in = (hh >= 0) & (hh < P.Hi) & (ww >= 0) & (ww < P.Wi);
            inside |= in ? (1u << t) : 0u;
            voffB[t] = in ? (rel + (uint32_t)(hh * P.Wi + ww)) * 4u + (uint32_t)kq * plane_bytes : 0u;
        }
    }
    const __amdgpu_buffer_rsrc_t rw = desc(P.win + base_off, P.win_elems - base_off);

    const int ngroups = P.Ci >> 4;        // channel groups per wave (the host checked Ci % 16 == 0)
    const int c0 = wave * (P.Ci >> 2);    // the wave's first channel

    float fa[D][KHW], fb[D][KHW];
    auto run = [](float (&dst)[KHW], const __amdgpu_buffer_rsrc_t &r, uint32_t voff, uint32_t soff)
                   __attribute__((always_inline)) {   // KHW consecutive floats (4-byte aligned)
#pragma unroll
        for (int i = 0; i + 4 <= KHW; i += 4) {
            const float4v w = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(r, voff + 4u * i, soff, 0));
            dst[i] = w.x; dst[i + 1] = w.y; dst[i + 2] = w.z; dst[i + 3] = w.w;
        }
#pragma unroll
        for (int i = KHW & ~3; i < KHW; ++i)
            dst[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff + 4u * i, soff, 0));
    };
    auto fetch = [&](float (&da)[KHW], float (&db)[KHW], int g) __attribute__((always_inline)) {
        const uint32_t c = (uint32_t)(c0 + 4 * g);
        run(da, rf, voffA, c * (uint32_t)(KHW * 4));
        if (!IMP) {
            run(db, rw, voffB[0], c * plane_bytes);
        } else {
#pragma unroll
            for (int t = 0; t < KHW; ++t)
                db[t] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rw, voffB[IMP ? t : 0], c * plane_bytes, 0));
        }
    };

    floatx4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d < ngroups) fetch(fa[d], fb[d], d);
    for (int g0 = 0; g0 < ngroups; g0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (g0 + d < ngroups) {
#pragma unroll
                for (int t = 0; t < KHW; ++t) {
                    const int u = t % HF, v = t / HF;   // window order: v outer, u inner; the filter is stored (u,v)
                    const float b = IMP ? (((inside >> t) & 1u) ? fb[d][t] : 0.0f) : fb[d][t];
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[d][u * WF + v], b, acc, 0, 0, 0);
                }
                if (g0 + d + D < ngroups) fetch(fa[d], fb[d], g0 + d + D);
            }
        }
    }

    // ((wave 0 + wave 1) + wave 2) + wave 3, then wave 0 stores the piece: accumulator register
    // v of lane (kq, l16) holds output channel 4*kq + v and pixel l16 of the piece
    if (wave > 0) {
#pragma unroll
        for (int v = 0; v < 4; ++v) lds[((wave - 1) * 4 + v) * 64 + lane] = acc[v];
    }
    __syncthreads();
    if (wave == 0) {
        const uint32_t Pm = Pq + (uint32_t)l16;
        if (Pm <= Pend) {
            const uint32_t img = fdiv(Pm, P.d_howo);
            const uint32_t pin = Pm - img * P.howo;
            float *o = P.out + (size_t)img * P.Co * P.howo + pin;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int j = mq + 4 * kq + v;
                const float r = ((acc[v] + lds[v * 64 + lane]) + lds[(4 + v) * 64 + lane]) + lds[(8 + v) * 64 + lane];
                if (j < P.Co) o[(size_t)j * P.howo] = r;
            }
        }
    }
}

// CW: floats per filter staging chunk (4: 16-byte loads; 2 and 1: the 8- and 4-byte loads of the
// load-width ablation).
// OCC: workgroups per CU the register allocation should leave room for.
// IMP: workspace-free variant.  P.win is the NCHW input; the tile's im2win strips
// (Section 3.1) are built directly in LDS -- same LDS layout, same MFMA loop -- by
// gathering input rows: strip word k*HF + u of output row m comes from input row
// m*s + u - p, column k - p (zero outside the image).
// PER: the grid may hold fewer workgroups than tiles; a workgroup then takes tiles blockIdx.x,
// + gridDim.x, ... and keeps the pipeline running across tile boundaries.
// Leftover tiles.  Workgroups 0 .. P.nmain-1 compute the tiles 0 .. P.nmain-1 whole; then come
// two workgroups for each of the next P.nhalf tiles (HALF), then sixteen for each of the rest (TAIL).
// HALF: a workgroup takes one half (32 pixels) of its tile, two waves per 32x32 block of
// outputs, each multiplying half of the channels of every K block (the two partial sums meet in
// LDS before the store).  For leftovers too many for the sixteenths: a half tile is staged
// through LDS like a whole one, at 3/4 of its traffic.
// TAIL: a workgroup takes one sixteenth of its tile (tail_piece above).
// RAG: Ci is not a multiple of CB.  The last K block then holds Ci % CB real channels; the words
// of the missing ones -- strip words and filter columns, whatever the loads brought in from the
// neighbouring channel planes and filter rows -- are replaced by +0.0 when that block is written
// to LDS, so the MFMA loop itself is unchanged.  (Whole tiles only: not combined with PER, TAIL, HALF.)
template <int HF, int WF, int CB, int JX, int CW, int OCC, bool IMP, bool PER, bool TAIL, bool HALF = false, bool RAG = false>
__global__ __launch_bounds__(256, OCC) void conv_mfma_fast_kernel(MfmaParams P)
{
    constexpr int KHW = HF * WF;
    constexpr int KB = CB * KHW;            // K elements per block
    constexpr int CPR = KB / CW;            // chunks per filter row per block
    constexpr int NFC = MB * CPR;           // chunks per filter tile
    constexpr int JF = (NFC + 255) / 256;   // chunks per thread
    constexpr int PF = KB | 1;              // odd LDS pitch of a filter row
    constexpr int SS = 256 * JX;            // LDS floats per channel strip (compile-time stride)
    constexpr int SF_FLOATS = (MB * PF + 3) & ~3;
    constexpr int STAGE = SF_FLOATS + CB * SS;   // floats per LDS stage
    constexpr int R = HALF ? pick_ring_half((CB / 2) * KHW) : pick_ring((CB / 2) * KHW);
    static_assert(R > 0, "no ring length divides the MFMAs per block");
    static_assert(CW == 4 || CW == 2 || CW == 1, "chunks are 16, 8 or 4 bytes");
    static_assert(KB % CW == 0, "K block must be a whole number of chunks");
    static_assert(CB % 2 == 0, "pair steps need an even channel count");
    static_assert(!RAG || (!PER && !TAIL && !HALF), "a ragged last K block comes with whole tiles only");

    // two LDS stages, each [filter tile MB x PF][CB strips of SS floats]
    extern __shared__ __align__(16) unsigned char smem[];
    float *lds = reinterpret_cast<float *>(smem);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int h = lane >> 5, l32 = lane & 31;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);   // the same, known to be wave-uniform
    const int wm_u = wave_u & 1, wn_u = wave_u >> 1;
    static_assert(!HALF || (!PER && (CB / 2) % 2 == 0),
                  "half tiles: the channel pairs of a K block split evenly between two waves");
    // half-tile workgroups: which tile, which half; waves 0/1 take the first half of the channel
    // pairs of every K block, waves 2/3 the second (hk = 1)
    // bid: the workgroup's place in the order "whole tiles, halves, sixteenths".  In the grid itself
    // the sixteenths sit at blocks P.tail_at ... (a multiple of 8, so XCDs are unchanged): dispatched
    // in the middle of the layer, their cold loads are covered by the whole tiles running beside them.
    uint32_t bid = blockIdx.x;
    if constexpr (TAIL) {
        const uint32_t end_main = P.nmain + 2u * P.nhalf, npb = gridDim.x - end_main;
        if (bid >= P.tail_at && bid < P.tail_at + npb) bid = end_main + (bid - P.tail_at);
        else if (bid >= P.tail_at + npb) bid -= npb;
    }
    const bool hmode = HALF && bid >= P.nmain && bid < P.nmain + 2u * P.nhalf;   // workgroup-uniform
    const uint32_t vb_first = hmode ? P.nmain + ((bid - P.nmain) >> 1) : bid;
    const int hpix = hmode ? (int)((bid - P.nmain) & 1u) * 32 : 0;   // first pixel of the half, within the tile
    const int wn_g = hmode ? 0 : wn;             // pixel block of the wave within the (half) tile
    const int hk = hmode ? (wave >> 1) : 0, hk_u = hmode ? (wave_u >> 1) : 0;

    if constexpr (TAIL) if (bid >= P.nmain + 2u * P.nhalf) {
        // Piece q of leftover tile t.  Workgroup b runs on XCD b % 8 and the pieces start at a
        // multiple of 8: the sixteen pieces of a tile are dealt to the same XCD, whose L2 then
        // serves their shared filter rows and windows (the last L % 8 tiles aside).
        const uint32_t first = P.nmain + P.nhalf;   // first tile computed in pieces
        const uint32_t sub = bid - (P.nmain + 2u * P.nhalf), L = P.nblocks - first, full = L & ~7u;
        uint32_t t, q;
        if (sub < 16u * full) {
            t = (sub & 7u) + ((sub >> 7) << 3);
            q = (sub >> 3) & 15u;
        } else {
            const uint32_t s2 = sub - 16u * full, Lr = L - full;
            q = s2 / Lr;
            t = full + (s2 - q * Lr);
        }
        tail_piece<HF, WF, IMP>(P, first + t, (int)q, lds, lane, wave_u);
        return;
    }

    const int sHf = P.s * HF;
    const uint32_t ntiles = P.nblocks;   // all tiles of the layer; this workgroup takes blockIdx.x, + gridDim.x, ...

    // ---- per-tile state: the tile being computed ("c") and the one after it ("n") ----
    // P0/Pend: first and last pixel; m0: first output channel; bp: per-lane LDS base of the B
    // operand (stage 0); soffb: byte offset (from the tile's descriptor base, same channel) of
    // strip word tid + 256*j -- words past the tile's segments are never used as operands and
    // reload word 0.  Workspace-free variant: thread word tid + 256*j of a segment is taken
    // row by row of the input (u outer, column inner: neighbouring lanes read neighbouring
    // input words) and lands at LDS strip position loffI; words that fall in the zero padding
    // (and unused ones) load word 0 and store +0.0 (bit j of zero).
    // rf / rw: buffer descriptors on the tile's filter rows / its first strip word (its first
    // image in the workspace-free variant); the host has checked that a tile's strips lie
    // within 4 GiB of that word.
    uint32_t P0_c = 0, Pend_c = 0, P0_n = 0, Pend_n = 0;
    int m0_c = 0, m0_n = 0;
    const lds_float *bp_c = nullptr, *bp_n = nullptr;
    uint32_t soffb_c[JX], soffb_n[JX];
    int loffI_c[JX], loffI_n[JX];
    uint32_t zero_c = 0, zero_n = 0;
    auto desc = [](const float *base, size_t elems) __attribute__((always_inline)) {
        const size_t left = elems * 4u;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(base), 0,
                                                 left < 0xffffffffull ? left : 0xffffffffull, 0x00020000);
    };
    __amdgpu_buffer_rsrc_t rf_c = desc(P.flt, 0), rf_n = desc(P.flt, 0), rw_c = desc(P.win, 0), rw_n = desc(P.win, 0);

    auto tile_geometry = [&](uint32_t vb, uint32_t &P0, uint32_t &Pend, int &m0, const lds_float *&bp,
                             uint32_t (&soffb)[JX], int (&loffI)[JX], uint32_t &zero,
                             __amdgpu_buffer_rsrc_t &rf, __amdgpu_buffer_rsrc_t &rw) __attribute__((always_inline)) {
        const uint32_t lb = (TAIL || HALF) ? (vb < P.nmain ? xcd_swizzle(vb, P.nmain) : vb) : xcd_swizzle(vb, ntiles);
        const uint32_t tile_n = fdiv(lb, P.d_tm);
        const uint32_t tile_m = lb - tile_n * (uint32_t)P.tiles_m;
        m0 = (int)tile_m * MB;
        P0 = tile_n * NB;
        Pend = min(P0 + NB - 1, P.npix - 1);
        if (HALF && hmode) {   // the half's own 32 pixels (the caller has checked that it has any)
            P0 += (uint32_t)hpix;
            Pend = min(P0 + 31u, Pend);
        }

        // strip geometry (rows q0..q1 of output pixels, q = i*Ho + m)
        const uint32_t q0 = fdiv(P0, P.d_wo), q1 = fdiv(Pend, P.d_wo);
        const int nlo0 = (int)(P0 - q0 * (uint32_t)P.Wo);
        const int len0 = (((q1 == q0) ? (int)(Pend - P0) : (P.Wo - 1 - nlo0)) * P.s + WF) * HF;
        // float offset, in channel plane 0, of the first strip word of the tile
        // (workspace-free variant: of the tile's first image in the input)
        const uint32_t img0 = fdiv(q0, P.d_ho);
        const size_t tile_base =
            IMP ? (size_t)img0 * P.Ci * P.in_plane
                : ((size_t)img0 * P.Ci * P.Ho + (q0 - img0 * (uint32_t)P.Ho)) * (size_t)P.rowlen + (size_t)(nlo0 * sHf);
        rf = desc(P.flt + (size_t)m0 * P.K, ((size_t)P.Co - (size_t)m0) * (size_t)P.K);
        rw = desc(P.win + tile_base, P.win_elems - tile_base);   // (P.win_elems: floats in the tensor P.win points at)

        zero = 0;
#pragma unroll
        for (int j = 0; j < JX; ++j) { soffb[j] = 0; loffI[j] = tid + 256 * j; if (IMP) zero |= 1u << j; }
        for (uint32_t q = q0; q <= q1; ++q) {
            const int rho = (int)(q - q0);
            const int nlo = rho == 0 ? nlo0 : 0;
            const int nhi = (q == q1) ? (int)(Pend - q * (uint32_t)P.Wo) : P.Wo - 1;
            const int seglen = ((nhi - nlo) * P.s + WF) * HF;
            const int segoff = rho == 0 ? 0 : len0 + (rho - 1) * P.fullseg;
            const uint32_t img = fdiv(q, P.d_ho);
            const int mq = (int)(q - img * (uint32_t)P.Ho);
            if (!IMP) {
                const size_t src = ((size_t)img * P.Ci * P.Ho + (size_t)mq) * (size_t)P.rowlen + (size_t)(nlo * sHf);
                const uint32_t rel = (uint32_t)(src - tile_base);   // the host checked that a tile's rows span < 4 GiB
#pragma unroll
                for (int j = 0; j < JX; ++j) {
                    const int x = tid + 256 * j - segoff;
                    if (x >= 0 && x < seglen) soffb[j] = (rel + (uint32_t)x) * 4u;
                }
            } else {
                const int ncol = (nhi - nlo) * P.s + WF;
                const uint32_t rel = (img - img0) * (uint32_t)P.Ci * P.in_plane;   // host: a tile's images span < 4 GiB
#pragma unroll
                for (int j = 0; j < JX; ++j) {
                    const int x = tid + 256 * j - segoff;
                    if (x >= 0 && x < seglen) {
                        int u = 0;
#pragma unroll
                        for (int t = 1; t < HF; ++t) u += (x >= t * ncol) ? 1 : 0;
                        const int kk = x - u * ncol;
                        const int hh = mq * P.s + u - P.p, ww = nlo * P.s + kk - P.p;
                        const bool inside = (hh >= 0) & (hh < P.Hi) & (ww >= 0) & (ww < P.Wi);
                        loffI[j] = segoff + kk * HF + u;
                        zero = inside ? (zero & ~(1u << j)) : (zero | (1u << j));
                        soffb[j] = inside ? (rel + (uint32_t)(hh * P.Wi + ww)) * 4u : 0u;
                    }
                }
            }
        }
        // per-lane B operand base: the lane's window start in the LDS strip
        const uint32_t Pl = min(P0 + (uint32_t)(wn_g * 32 + l32), Pend);
        const uint32_t ql = fdiv(Pl, P.d_wo);
        const int nl = (int)(Pl - ql * (uint32_t)P.Wo);
        const int rhol = (int)(ql - q0);
        const int b_base = rhol == 0 ? (nl - nlo0) * sHf : len0 + (rhol - 1) * P.fullseg + nl * sHf;
        bp = (const lds_float *)lds + SF_FLOATS + b_base + h * SS + hk * ((CB / 2) * SS);
    };
    if (HALF && hmode) {   // a ragged last tile may have no pixel in its second half (whole workgroup)
        const uint32_t tn = fdiv(vb_first, P.d_tm);
        if (tn * NB + (uint32_t)hpix >= P.npix) return;
    }
    tile_geometry(vb_first, P0_c, Pend_c, m0_c, bp_c, soffb_c, loffI_c, zero_c, rf_c, rw_c);
    const int m0 = m0_c;   // (filter staging below: with several tiles per workgroup every row of every tile is live)

    // Prefetch registers for the strip words: two alternating sets (the words come from HBM
    // and are given about one and a half K blocks to arrive).  Global loads go through the
    // tiles' buffer descriptors: a wave-uniform base held in scalar registers, the thread's
    // constant 32-bit byte offset, and a scalar offset that selects the K block and channel.
    // The K loop spends no vector ALU work on addresses.
    float ir[2][CB * JX];
    const uint32_t plane_bytes = (IMP ? P.in_plane : P.chan_stride) * 4u;
    auto load_i = [&](int kb, int set, int c, int j, const __amdgpu_buffer_rsrc_t &rw, const uint32_t (&soffb)[JX]) __attribute__((always_inline)) {
        ir[set][c * JX + j] = __builtin_bit_cast(
            float, __builtin_amdgcn_raw_buffer_load_b32(rw, soffb[j], (uint32_t)(kb * CB + c) * plane_bytes, 0));
    };
    // The strip words of the first tile's first two K blocks are requested here, before the
    // filter staging coordinates are worked out: they have the longest way to come.
    const int nkb = RAG ? (P.Ci + CB - 1) / CB : P.Ci / CB;
    const int last_ch = P.Ci - (nkb - 1) * CB;   // channels of the last K block (CB unless RAG)
#pragma unroll
    for (int w = 0; w < CB * JX; ++w) load_i(0, 0, w / JX, w % JX, rw_c, soffb_c);
    if (nkb > 1) {
#pragma unroll
        for (int w = 0; w < CB * JX; ++w) load_i(1, 1, w / JX, w % JX, rw_c, soffb_c);
    }

    // ---- filter staging coordinates of this thread's chunks ----
    // The tile is MB rows x CPR chunks of CW floats.  Chunk columns are dealt out
    // so that each dword LDS write of a half-wave is conflict-free with the odd
    // row pitch: a half-wave covers CW consecutive rows x 32/CW chunk columns
    // (128 contiguous bytes per row in global memory); the CPR % (32/CW) leftover
    // columns go one column x 32 rows per half-wave.
    // Rows past Co feed accumulators that are never stored; they reload row 0.
    constexpr int COLS = 32 / CW;              // chunk columns per half-wave
    constexpr int CG = CPR / COLS;             // full column groups
    constexpr int NMAIN = MB * CG * COLS;      // chunks in full groups
    uint32_t goffb[JF];
    int loff[JF];
#pragma unroll
    for (int j = 0; j < JF; ++j) {
        const int f = tid + 256 * j;
        int row, cc;
        if (CG > 0 && f < NMAIN) {
            const int g = f >> 5, w = f & 31;
            row = CW * (g / (CG > 0 ? CG : 1)) + (w / COLS);
            cc = COLS * (g % (CG > 0 ? CG : 1)) + (w % COLS);
        } else {
            const int r = f - NMAIN;
            row = r % MB;
            cc = CG * COLS + r / MB;
        }
        const int e = cc * CW;
        const bool live = (f < NFC) && (m0 + row < P.Co);
        goffb[j] = live ? (uint32_t)(row * P.K + e) * 4u : 0u;
        loff[j] = row * PF + e;
    }
    // A thread with no chunk in the last round repeats its first chunk (same data to
    // the same place), which keeps the staging code free of branches.
    if (tid + 256 * (JF - 1) >= NFC) { goffb[JF - 1] = goffb[0]; loff[JF - 1] = loff[0]; }
    // RAG: bit j*CW + w set when word w of chunk j lies in a channel the last K block does not have
    uint32_t fzero = 0;
    if (RAG) {
        static_assert(!RAG || JF * CW <= 32, "one mask bit per staged filter word");
#pragma unroll
        for (int j = 0; j < JF; ++j) {
            const int e = (loff[j] % PF);   // first K element of the chunk within the block
#pragma unroll
            for (int w = 0; w < CW; ++w) fzero |= (e + w >= last_ch * KHW) ? (1u << (j * CW + w)) : 0u;
        }
    }

    const lds_float *ap0 = (const lds_float *)lds + (wm * 32 + l32) * PF + h * KHW + hk * ((CB / 2) * KHW);
    float *wI0 = lds + SF_FLOATS + tid;

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    // Prefetch registers of the filter chunks: one set (they come from L2).
    float fr[JF][CW];

    auto load_f = [&](int kb, int j, const __amdgpu_buffer_rsrc_t &rf) __attribute__((always_inline)) {
        if constexpr (CW == 4) {
            const float4v w = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rf, goffb[j], kb * (KB * 4), 0));
            fr[j][0] = w.x; fr[j][1] = w.y; fr[j][CW - 2] = w.z; fr[j][CW - 1] = w.w;
        } else if constexpr (CW == 2) {
            const float2v w = __builtin_bit_cast(float2v, __builtin_amdgcn_raw_buffer_load_b64(rf, goffb[j], kb * (KB * 4), 0));
            fr[j][0] = w.x; fr[j][1] = w.y;
        } else {
            fr[j][0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rf, goffb[j], kb * (KB * 4), 0));
        }
    };
    constexpr int WPS = CW >= 2 ? 2 : 1;   // words per filter store slot
    // last: the K block being written is the ragged last one (RAG instances only)
    auto store_f = [&](int st, int j, int half, bool last = false) __attribute__((always_inline)) {   // words WPS*half .. of chunk j
        lds_float *d = (lds_float *)lds + st * STAGE + loff[j] + WPS * half;
        const int b = j * CW + WPS * half;
        d[0] = (RAG && last && ((fzero >> b) & 1u)) ? 0.0f : fr[j][WPS * half];
        if constexpr (WPS == 2) d[1] = (RAG && last && ((fzero >> (b + 1)) & 1u)) ? 0.0f : fr[j][WPS * half + 1];
    };
    auto store_i = [&](int st, int set, int c, int j, const int (&loffI)[JX], uint32_t zero, bool last = false) __attribute__((always_inline)) {
        const bool gone = RAG && last && c >= last_ch;   // wave-uniform
        if (IMP)
            ((lds_float *)lds)[SF_FLOATS + loffI[j] + st * STAGE + c * SS] = (((zero >> j) & 1u) || gone) ? 0.0f : ir[set][c * JX + j];
        else
            ((lds_float *)wI0)[st * STAGE + c * SS + 256 * j] = gone ? 0.0f : ir[set][c * JX + j];
    };

    // ---- one K block --------------------------------------------------------------
    // The wave issues its MFMAs as one dependent chain, so everything else is
    // placed, in program order, in the shadow of an MFMA: after MFMA i come the two
    // operand reads for step i+R (a ring of R register pairs) and one or two
    // staging instructions.  Block kb computes out of LDS stage ST, writes block
    // kb+1 (held in registers) to the other stage and requests block kb+2 from
    // global memory.  The barrier sits R steps before the end of the block: the
    // operands of those last steps are already in registers, so after the barrier
    // the other stage can be read (first operands of block kb+1) and, in the next
    // block, this stage can be overwritten.  Scheduling barriers pin this order.
    constexpr int NG = CB / 2;            // channel pairs per block
    constexpr int NM = NG * KHW;          // MFMAs per block
    constexpr int NSLOT = NM - R;         // MFMAs before the barrier
    constexpr int HPC = CW >= 2 ? CW / 2 : 1;   // store slots per filter chunk (two words each; one for 4-byte chunks)
    constexpr int NFW = HPC * JF;         // filter store slots
    constexpr int NIW = CB * JX;          // strip stores / loads
    constexpr int NIWS = (NIW + 1) / 2;   // slots that store strip words (two each)
    static_assert(NM > R && NSLOT - NFW - NIWS > 0, "K block too short for the pipeline");
    constexpr int LPS = (NIW + (NSLOT - NFW - NIWS) - 1) / (NSLOT - NFW - NIWS);   // strip loads per slot
    constexpr int NILS = (NIW + LPS - 1) / LPS;                                      // slots that load strip words
    static_assert(NFW + NIWS + NILS <= NSLOT, "staging work must fit before the barrier");

    // BW: a filter height of four (two) makes every window start a multiple of four (two) floats into its
    // strip (and all strip and stage sizes are), so the B operands of BW consecutive steps -- one window
    // column -- are one aligned 16-byte (8-byte) LDS read.  With single-word reads such a layer is bound by
    // LDS: its windows start s*Hf floats apart, at 4x4 stride 2 a wave's 32 reads fall into four banks
    // (bank-conflict cycles were 71 % of the LDS-active cycles, LDS active 94 % of the time; 64 -> 128
    // channels at 64x64: 117 -> 136 TFLOP/s with the wide reads).  The ring then holds R/BW vectors of B.
    constexpr int BW = (HALF || R % 4 != 0) ? 1 : (HF == 4 ? 4 : (HF == 2 ? 2 : 1));
    typedef float bvec_t __attribute__((ext_vector_type(BW == 1 ? 2 : BW)));   // (no one-element vector type: unused then)
    float a[R], b[BW == 1 ? R : 1];
    bvec_t bq[BW == 1 ? 1 : R / BW];
    // operands of step i (0 <= i < NM) of a block, from LDS stage st, into ring slot i % R;
    // bp: the B base of the tile the block belongs to
    auto lds_op = [&](int st, int i, const lds_float *bp) __attribute__((always_inline)) {
        const int g = i / KHW, t = i % KHW;
        const int u = t % HF, v = t / HF;   // window order: v outer, u inner; the filter is stored (u,v)
        // volatile: keeps these as single-dword LDS reads with 16-bit immediate
        // offsets (merged two-address reads have 8-bit offsets and would need a VALU
        // add each -- and VALU work comes out of the MFMA rate).
        a[i % R] = *(const volatile lds_float *)(ap0 + st * STAGE + 2 * g * KHW + u * WF + v);
        if constexpr (BW > 1) {
            // the vector of steps i-BW+1 .. i goes out with its last step: its ring slot was read by the
            // MFMAs R steps earlier, the last of which has just been issued
            if (i % BW == BW - 1) {
                typedef __attribute__((address_space(3))) bvec_t lds_bvec;
                bq[(i / BW) % (R / BW)] = *(const volatile lds_bvec *)(bp + st * STAGE + 2 * g * SS + (t - (BW - 1)));
            }
        } else {
            b[i % R] = *(const volatile lds_float *)(bp + st * STAGE + 2 * g * SS + t);
        }
    };
    auto b_of = [&](int i) __attribute__((always_inline)) -> float {
        if constexpr (BW > 1) return bq[(i / BW) % (R / BW)][i % BW];
        else return b[i % R];
    };

    // NX1 / NX2: the block after this one / the one after that belongs to the next tile (a
    // workgroup with several tiles keeps the pipeline running across the tile boundary);
    // kb2: index, within its own tile, of the block whose global loads are issued here.
    auto block = [&](int kb2, auto stc, auto has1c, auto has2c, auto nx1c, auto nx2c) __attribute__((always_inline)) {
        constexpr int ST = decltype(stc)::value;
        constexpr bool HAS1 = decltype(has1c)::value, HAS2 = decltype(has2c)::value;
        constexpr bool NX1 = decltype(nx1c)::value, NX2 = decltype(nx2c)::value;
        constexpr bool LAST = RAG && HAS1 && !HAS2;   // this block writes the tile's last K block to LDS
#pragma unroll
        for (int i = 0; i < NM; ++i) {
            if (HAS1 && i == NSLOT) __syncthreads();
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i % R], b_of(i), acc, 0, 0, 0);
            // ring slot i % R is free again: fetch the operands of step i + R (of this
            // block, or of the next one out of the other stage)
            if (i + R < NM) lds_op(ST, i + R, bp_c);
            else if (HAS1) { if (NX1) lds_op(ST ^ 1, i + R - NM, bp_n); else lds_op(ST ^ 1, i + R - NM, bp_c); }
            if (i < NFW) {                       // filter chunk i/HPC: store a half, then reload it
                if (HAS1) store_f(ST ^ 1, i / HPC, i % HPC, LAST);
                if (HAS2 && (i % HPC == HPC - 1)) { if (NX2) load_f(kb2, i / HPC, rf_n); else load_f(kb2, i / HPC, rf_c); }
            } else if (i < NFW + NIWS) {   // strip words of the next block: two stores per slot
                if (HAS1) {
                    const int w = 2 * (i - NFW);
                    if (NX1) {
                        store_i(ST ^ 1, ST ^ 1, w / JX, w % JX, loffI_n, zero_n);
                        if (w + 1 < NIW) store_i(ST ^ 1, ST ^ 1, (w + 1) / JX, (w + 1) % JX, loffI_n, zero_n);
                    } else {
                        store_i(ST ^ 1, ST ^ 1, w / JX, w % JX, loffI_c, zero_c, LAST);
                        if (w + 1 < NIW) store_i(ST ^ 1, ST ^ 1, (w + 1) / JX, (w + 1) % JX, loffI_c, zero_c, LAST);
                    }
                }
            } else if (i < NFW + NIWS + NILS) {   // strip words of the block after that: LPS loads per slot
                if (HAS2) {
#pragma unroll
                    for (int q = 0; q < LPS; ++q) {
                        const int w = (i - NFW - NIWS) * LPS + q;
                        if (w < NIW) {
                            if (NX2) load_i(kb2, ST, w / JX, w % JX, rw_n, soffb_n);
                            else load_i(kb2, ST, w / JX, w % JX, rw_c, soffb_c);
                        }
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

    // ---- prologue: block 0 of the first tile into stage 0, its block 1 into the registers ----
#pragma unroll
    for (int j = 0; j < JF; ++j) load_f(0, j, rf_c);
#pragma unroll
    for (int j = 0; j < JF; ++j)
#pragma unroll
        for (int hh = 0; hh < HPC; ++hh) store_f(0, j, hh);
#pragma unroll
    for (int w = 0; w < NIW; ++w) store_i(0, 0, w / JX, w % JX, loffI_c, zero_c);
    if (nkb > 1) {
#pragma unroll
        for (int j = 0; j < JF; ++j) load_f(1, j, rf_c);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < R; ++i) lds_op(0, i, bp_c);

    // ---- half tile: the same pipeline with half of the MFMA steps per K block ----
    if constexpr (HALF) if (hmode) {
        constexpr int NMH = NM / 2;          // this wave's MFMAs per block: its half of the channel pairs
        constexpr int NSLOTH = NMH - R;      // MFMAs before the barrier
        constexpr int NITEM = NFW + NIWS + NIW;              // staging items: filter half-stores, strip stores (two each), strip loads
        constexpr int IPS = (NITEM + NSLOTH - 1) / NSLOTH;   // items per slot
        static_assert(NSLOTH > 0, "K block too short for the pipeline");
        auto block_half = [&](int kb2, auto stc, auto has1c, auto has2c) __attribute__((always_inline)) {
            constexpr int ST = decltype(stc)::value;
            constexpr bool HAS1 = decltype(has1c)::value, HAS2 = decltype(has2c)::value;
#pragma unroll
            for (int i = 0; i < NMH; ++i) {
                if (HAS1 && i == NSLOTH) __syncthreads();
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i % R], b[i % R], acc, 0, 0, 0);
                if (i + R < NMH) lds_op(ST, i + R, bp_c);
                else if (HAS1) lds_op(ST ^ 1, i + R - NMH, bp_c);
                if (i < NSLOTH) {
#pragma unroll
                    for (int it = i * IPS; it < (i + 1) * IPS && it < NITEM; ++it) {
                        if (it < NFW) {                       // filter chunk it/HPC: store a half, then reload it
                            if (HAS1) store_f(ST ^ 1, it / HPC, it % HPC);
                            if (HAS2 && (it % HPC == HPC - 1)) load_f(kb2, it / HPC, rf_c);
                        } else if (it < NFW + NIWS) {         // strip words of the next block: two stores
                            if (HAS1) {
                                const int w = 2 * (it - NFW);
                                store_i(ST ^ 1, ST ^ 1, w / JX, w % JX, loffI_c, zero_c);
                                if (w + 1 < NIW) store_i(ST ^ 1, ST ^ 1, (w + 1) / JX, (w + 1) % JX, loffI_c, zero_c);
                            }
                        } else {                              // strip words of the block after that
                            const int w = it - NFW - NIWS;
                            if (HAS2) load_i(kb2, ST, w / JX, w % JX, rw_c, soffb_c);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        int kb = 0;
        for (; kb + 3 < nkb; kb += 2) {
            block_half(kb + 2, I0{}, T{}, T{});
            block_half(kb + 3, I1{}, T{}, T{});
        }
        const int rem = nkb - kb;   // 1, 2 or 3 blocks left
        if (rem == 3) {
            block_half(kb + 2, I0{}, T{}, T{});
            block_half(0, I1{}, T{}, F{});
            block_half(0, I0{}, F{}, F{});
        } else if (rem == 2) {
            block_half(0, I0{}, T{}, F{});
            block_half(0, I1{}, F{}, F{});
        } else {
            block_half(0, I0{}, F{}, F{});
        }
        // the two partial sums of a block of outputs: waves 2/3 hand theirs to waves 0/1 through
        // LDS (every wave has taken its last operands before the stages are overwritten)
        __syncthreads();
        if (hk_u) {
#pragma unroll
            for (int v = 0; v < 16; ++v) lds[((wm_u * 16 + v) * 64) + lane] = acc[v];
        }
        __syncthreads();
        if (!hk_u) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] += lds[((wm_u * 16 + v) * 64) + lane];
            store_tile_desc(P, acc, P0_c, Pend_c, m0_c, wm_u, 0, h, l32);
        }
        return;
    }

    // ---- tiles of this workgroup ----
    // The host gives a workgroup more than one tile only when nkb is even (every tile then
    // starts in LDS stage 0) and Co is a multiple of the tile height.
    for (uint32_t vb = bid;;) {
        const bool has_next = PER && vb + gridDim.x < ntiles;   // wave-uniform
        if (has_next) tile_geometry(vb + gridDim.x, P0_n, Pend_n, m0_n, bp_n, soffb_n, loffI_n, zero_n, rf_n, rw_n);

        int kb = 0;
        for (; kb + 3 < nkb; kb += 2) {   // unrolled by two so that the stage is a constant
            block(kb + 2, I0{}, T{}, T{}, F{}, F{});
            block(kb + 3, I1{}, T{}, T{}, F{}, F{});
        }
        const int rem = nkb - kb;   // 1, 2 or 3 blocks left
        if (has_next) {             // rem == 2: the next tile's blocks 0 and 1 are fetched meanwhile
            block(0, I0{}, T{}, T{}, F{}, T{});
            block(1, I1{}, T{}, T{}, T{}, T{});
        } else if (rem == 3) {
            block(kb + 2, I0{}, T{}, T{}, F{}, F{});
            block(0, I1{}, T{}, F{}, F{}, F{});
            block(0, I0{}, F{}, F{}, F{}, F{});
        } else if (rem == 2) {
            block(0, I0{}, T{}, F{}, F{}, F{});
            block(0, I1{}, F{}, F{}, F{}, F{});
        } else {
            block(0, I0{}, F{}, F{}, F{}, F{});
        }

        store_tile_desc(P, acc, P0_c, Pend_c, m0_c, wm_u, wn_u, h, l32);
        if (!has_next) break;

        // the next tile becomes the current one
        vb += gridDim.x;
        P0_c = P0_n; Pend_c = Pend_n; m0_c = m0_n; bp_c = bp_n; zero_c = zero_n; rf_c = rf_n; rw_c = rw_n;
#pragma unroll
        for (int j = 0; j < JX; ++j) { soffb_c[j] = soffb_n[j]; loffI_c[j] = loffI_n[j]; }
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    }
}

template <int HF, int WF, int CB, int JX, int CW, int OCC>
static hipError_t launch_fast_i(const MfmaParams &P, uint32_t blocks, hipStream_t st, bool implicit, LaunchPlan *plan);

template <int HF, int WF, int CB, int JX, int CW, int OCC, bool IMP = false>
static hipError_t launch_fast_t(const MfmaParams &P, uint32_t blocks, hipStream_t st, LaunchPlan *plan)
{
    constexpr int KB = CB * HF * WF;
    constexpr int PF = KB | 1;
    constexpr size_t lds = 2u * 4u * (size_t)(((MB * PF + 3) & ~3) + CB * 256 * JX);
    if (P.Ci % CB != 0) {
        // ragged last K block: whole tiles, one per workgroup (only the 16-byte filter-fetch instances exist)
        if constexpr (CW == ((HF == 7 && WF == 7) ? 2 : 4)) {
            MfmaParams Q = P;
            Q.nblocks = blocks; Q.nmain = blocks; Q.nhalf = 0; Q.tail_at = blocks;
            void (*kern)(MfmaParams) = &conv_mfma_fast_kernel<HF, WF, CB, JX, CW, OCC, IMP, false, false, false, true>;
            if (plan) {
                plan_record(plan, dim3(blocks), 256, lds, "conv_mfma_fast_kernel<%d, %d, %d, %d, %d, %d, %s, false, false, false, true>",
                            HF, WF, CB, JX, CW, OCC, tf(IMP));
                return hipSuccess;
            }
            static KernelCache kcr;
            int dev = 0;
            hipError_t e = hipGetDevice(&dev);
            if (e != hipSuccess) return e;
            if ((e = allow_dynamic_lds(kcr, reinterpret_cast<const void *>(kern), lds, dev)) != hipSuccess) return e;
            hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), lds, st, Q);
            return hipGetLastError();
        } else {
            return hipErrorNotSupported;
        }
    }
    // Several tiles per workgroup (the pipeline then runs across tile boundaries) when every tile
    // starts in LDS stage 0 (an even number of K blocks), every filter row of every tile exists,
    // and there are at least three tiles per resident workgroup.  It pays for short K loops --
    // with 8 blocks per tile the per-tile start-up is an eighth of the work (+8 % measured) --
    // and costs 1-3 % with 16 or more, where it is not used.  The count is a multiple of 8 so
    // that a workgroup's tiles stay on its XCD under the block-id remapping.
    MfmaParams Q = P;
    Q.nblocks = blocks;
    Q.nmain = blocks;
    uint32_t grid = blocks;
    int dev = 0, ncu = 0;
    hipError_t e = device_cus(&dev, &ncu);
    if (e != hipSuccess && plan) { e = hipSuccess; ncu = 256; }   // planning without a device: an MI355X's 256 compute units
    if (e != hipSuccess) return e;
    if ((Q.Ci / CB) % 2 == 0 && Q.Ci / CB <= 12 && Q.Co % MB == 0) {
        const uint32_t resident = ((uint32_t)ncu * OCC) & ~7u;
        if (resident >= 8 && blocks >= 3 * resident) grid = resident;
    }
    // Leftover tiles: the workgroups go out in rounds that end together, and a compute unit is
    // as fast with one workgroup as with OCC of them, so a layer takes as long as its busiest
    // compute unit: ceil(tiles / ncu) tile times.  Workgroups dispatched late are spread evenly
    // over the compute units, so the last blocks % ncu tiles are cut up to give every unit a
    // share (3x3 instances; the 5x5 instance knows the halves only):
    //   - up to ncu/2 of them into two halves of 32 pixels each, staged through LDS like a
    //     whole tile -- a compute unit then ends with one whole tile and one half instead of
    //     two whole tiles;
    //   - up to ncu/8 of them (the rest, when it is that small and Ci is a multiple of 16)
    //     into sixteenths, which read their operands without sharing them through LDS: four
    //     times the traffic of a whole tile, but one cold load latency long (measured against
    //     the halves on 64- and 256-channel layers, they win up to 32-44 leftover tiles of 256).
    constexpr bool PIECEABLE = HF == 3 && WF == 3 && CB == 8;
    constexpr bool HALFABLE = PIECEABLE || (HF == 5 && WF == 5 && CB == 4);   // (the 5x5 instance: halves only)
    uint32_t nhalf = 0, npiece = 0;
    if (HALFABLE && grid == blocks && ncu >= 8 && ncu % 8 == 0) {   // (a layer with fewer tiles than compute units is all leftover)
        const uint32_t left = blocks % (uint32_t)ncu, eighth = (uint32_t)ncu / 8, halfcu = (uint32_t)ncu / 2;
        const bool pieces_ok = PIECEABLE && Q.Ci % 16 == 0;
        if (pieces_ok && left <= eighth) npiece = left;
        else if (left <= halfcu) nhalf = left;
        else if (pieces_ok && left - halfcu <= eighth) { nhalf = halfcu; npiece = left - halfcu; }
        Q.nmain = blocks - nhalf - npiece;
        grid = Q.nmain + 2 * nhalf + 16 * npiece;
    }
    Q.nhalf = nhalf;
    Q.tail_at = Q.nmain + 2 * nhalf;
    void (*kern)(MfmaParams) = &conv_mfma_fast_kernel<HF, WF, CB, JX, CW, OCC, IMP, false, false>;
    int which = 0;   // which of this launcher's five kernel instances
    if (grid < blocks) { kern = &conv_mfma_fast_kernel<HF, WF, CB, JX, CW, OCC, IMP, true, false>; which = 1; }
    if (npiece && !nhalf) { kern = &conv_mfma_fast_kernel<HF, WF, CB, JX, CW, OCC, IMP, false, PIECEABLE>; which = 2; }
    if (nhalf && !npiece) { kern = &conv_mfma_fast_kernel<HF, WF, CB, JX, CW, OCC, IMP, false, false, HALFABLE>; which = 3; }
    if (nhalf && npiece) { kern = &conv_mfma_fast_kernel<HF, WF, CB, JX, CW, OCC, IMP, false, PIECEABLE, HALFABLE>; which = 4; }
    if (plan) {
        const bool per = which == 1, tail = (which == 2 || which == 4) && PIECEABLE, half = (which == 3 || which == 4) && HALFABLE;
        plan_record(plan, dim3(grid), 256, lds, "conv_mfma_fast_kernel<%d, %d, %d, %d, %d, %d, %s, %s, %s, %s, false>",
                    HF, WF, CB, JX, CW, OCC, tf(IMP), tf(per), tf(tail), tf(half));
        return hipSuccess;
    }
    static KernelCache kc[5];
    if ((e = allow_dynamic_lds(kc[which], reinterpret_cast<const void *>(kern), lds, dev)) != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, Q);
    return hipGetLastError();
}

template <int HF, int WF, int CB, int JX, int CW, int OCC>
static hipError_t launch_fast_i(const MfmaParams &P, uint32_t blocks, hipStream_t st, bool implicit, LaunchPlan *plan)
{
    return implicit ? launch_fast_t<HF, WF, CB, JX, CW, OCC, true>(P, blocks, st, plan)
                    : launch_fast_t<HF, WF, CB, JX, CW, OCC, false>(P, blocks, st, plan);
}

// Returns hipErrorNotSupported when the layer does not meet the fast path's conditions.
// implicit: P.win is the NCHW input (P.Hi, P.Wi, P.p, P.in_plane set; P.win_elems = its size).
// filter_fetch_floats: 4, or 2 / 1 for the load-width ablation instances (8- and 4-byte filter
// fetches), which exist for 3x3 layers only; other layers then run their default instance.
hipError_t launch_conv_mfma_fast(MfmaParams P, const Shape &sh, uint32_t blocks, hipStream_t st, bool implicit,
                                 int filter_fetch_floats, LaunchPlan *plan)
{
    // Filter rows are fetched in 16-byte (7x7: 8-byte) pieces from a 16-byte (8-byte) aligned filter.
    // With K = Ci*Hf*Wf not a multiple of four the rows themselves start at odd multiples of four
    // bytes: the buffer loads take that (the ablation instances ask for aligned rows).
    const uintptr_t fa = reinterpret_cast<uintptr_t>(P.flt);
    const bool al16 = (fa & 15u) == 0, al8 = (fa & 7u) == 0;
    const bool rows16 = al16 && (sh.K % 4 == 0);
    // Strip words are addressed with 32-bit byte offsets from the tile's first strip word (from
    // its first image in the workspace-free variant): the rows of a tile (at most P.rmax of
    // them, in at most that many images) must span < 4 GiB.
    const unsigned long long img_bytes =
        implicit ? (unsigned long long)sh.Ci * sh.Hi * (unsigned long long)sh.Wi * 4ull
                 : (unsigned long long)sh.Ci * sh.Ho * (unsigned long long)sh.rowlen * 4ull;
    if (img_bytes * (unsigned long long)(P.rmax + 1) >= (1ull << 32)) return hipErrorNotSupported;
    // filter words likewise: 32-bit byte offsets from the tile's first filter row
    if ((unsigned long long)sh.K * 4ull * MB >= (1ull << 32)) return hipErrorNotSupported;
    // output words: 32-bit byte offsets from (image of the tile's first pixel, first channel of the wave)
    if (((unsigned long long)sh.Co * (unsigned long long)P.rmax + 64ull) * (unsigned long long)sh.Ho * sh.Wo * 4ull >= (1ull << 32))
        return hipErrorNotSupported;
    if (filter_fetch_floats == 2 && !implicit && sh.Hf == 3 && sh.Wf == 3 && sh.Ci % 8 == 0 && rows16) {   // ablation: 8-byte filter chunks
        if (P.S <= 256) return launch_fast_t<3, 3, 8, 1, 2, 3, false>(P, blocks, st, plan);
        if (P.S <= 512) return launch_fast_t<3, 3, 8, 2, 2, 3, false>(P, blocks, st, plan);
    }
    if (filter_fetch_floats == 1 && !implicit && sh.Hf == 3 && sh.Wf == 3 && sh.Ci % 8 == 0 && rows16) {   // ablation: 4-byte filter chunks
        if (P.S <= 256) return launch_fast_t<3, 3, 8, 1, 1, 3, false>(P, blocks, st, plan);
        if (P.S <= 512) return launch_fast_t<3, 3, 8, 2, 1, 3, false>(P, blocks, st, plan);
    }
    // (Ci need not be a multiple of the K block: the last block is then zero-filled)
    if (sh.Hf == 3 && sh.Wf == 3 && sh.Ci >= 8 && al16) {
        if (P.S <= 256) return launch_fast_i<3, 3, 8, 1, 4, 3>(P, blocks, st, implicit, plan);
        if (P.S <= 512) return launch_fast_i<3, 3, 8, 2, 4, 3>(P, blocks, st, implicit, plan);
    }
    if (sh.Hf == 5 && sh.Wf == 5 && sh.Ci >= 4 && al16) {
        if (P.S <= 256) return launch_fast_i<5, 5, 4, 1, 4, 2>(P, blocks, st, implicit, plan);
        if (P.S <= 512) return launch_fast_i<5, 5, 4, 2, 4, 2>(P, blocks, st, implicit, plan);
        if (P.S <= 768) return launch_fast_i<5, 5, 4, 3, 4, 2>(P, blocks, st, implicit, plan);   // (stride 2)
    }
    if (sh.Hf == 7 && sh.Wf == 7 && sh.Ci >= 2 && al8) {
        if (P.S <= 512) return launch_fast_i<7, 7, 2, 2, 2, 2>(P, blocks, st, implicit, plan);
        if (P.S <= 1024) return launch_fast_i<7, 7, 2, 4, 2, 2>(P, blocks, st, implicit, plan);
    }
    // Asymmetric filters (1x7 / 7x1 and 1x3 / 3x1 pairs that factor a square filter): the same pipeline
    // with eight (sixteen) channels per K block; a column filter's strips are Hf times longer.
    if (sh.Hf == 1 && sh.Wf == 7 && sh.Ci >= 8 && al16) {
        if (P.S <= 256) return launch_fast_i<1, 7, 8, 1, 4, 3>(P, blocks, st, implicit, plan);
        if (P.S <= 512) return launch_fast_i<1, 7, 8, 2, 4, 2>(P, blocks, st, implicit, plan);
    }
    if (sh.Hf == 7 && sh.Wf == 1 && sh.Ci >= 8 && al16) {
        if (P.S <= 512) return launch_fast_i<7, 1, 8, 2, 4, 2>(P, blocks, st, implicit, plan);
    }
    if (sh.Hf == 1 && sh.Wf == 3 && sh.Ci >= 16 && al16) {
        if (P.S <= 256) return launch_fast_i<1, 3, 16, 1, 4, 2>(P, blocks, st, implicit, plan);
    }
    if (sh.Hf == 3 && sh.Wf == 1 && sh.Ci >= 16 && al16) {
        if (P.S <= 256) return launch_fast_i<3, 1, 16, 1, 4, 2>(P, blocks, st, implicit, plan);
    }
    // 4x4 (the stride-2 down- and up-sampling layers of generator / discriminator networks): four channels per block
    if (sh.Hf == 4 && sh.Wf == 4 && sh.Ci >= 4 && al16) {
        if (P.S <= 512) return launch_fast_i<4, 4, 4, 2, 4, 2>(P, blocks, st, implicit, plan);
        if (P.S <= 768) return launch_fast_i<4, 4, 4, 3, 4, 2>(P, blocks, st, implicit, plan);
    }
    // 2x2 (stride-2 down-sampling): sixteen channels per block.  (P.S counts one float more than the
    // strips hold; at stride 2 a tile's 64 windows are exactly 256 floats.)
    if (sh.Hf == 2 && sh.Wf == 2 && sh.Ci >= 16 && al16) {
        if (P.S - 1 <= 256) return launch_fast_i<2, 2, 16, 1, 4, 2>(P, blocks, st, implicit, plan);
    }
    return hipErrorNotSupported;
}

}  // namespace im2win
