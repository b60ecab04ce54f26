// Filter-stationary MFMA im2win convolution for layers with few input channels
// and a large window (the 7x7/stride-2 and 11x11/stride-4 stem layers, Table 2's
// Conv1-Conv3/Conv7): K = Ci*Hf*Wf is small (27..363) while N = Ni*Ho*Wo is huge.
//
// Design (CDNA4's, not the paper's CUDA tiling):
//   - persistent workgroups: the grid takes the 64-pixel tiles round by round, the
//     workgroups of one XCD on neighbouring tiles (what an XCD writes at any time is
//     one contiguous stretch of every output plane);
//   - every wave keeps the A operand (its 32 filter rows, its share of K) in
//     registers for the whole kernel -- the filter is read from memory once per
//     wave, never staged per tile -- so each MFMA needs one LDS read only;
//   - the B operand is the tile's contiguous im2win strips (Section 3.1) in LDS,
//     double-buffered: the next tile's strips are copied into the other LDS stage by
//     direct global-to-LDS loads while the matrix cores work;
//   - K order: channel pairs ride the two lane halves of v_mfma_f32_32x32x2_f32
//     ("pair" steps); an odd last channel is split in two halves of its window
//     ("split" steps); every operand address is lane base + immediate;
//   - when K is too large for one wave's registers (11x11x3 = 363) two waves
//     share a 32x32 output block, each taking half of the K steps, and exchange
//     half of their accumulators through LDS before the store (KS = 2);
//   - every output store is issued by every wave (masked lanes pass an offset the
//     buffer unit rejects), so the wait for the strips can count past the stores.
#include "conv_mfma_tile.h"
#include "runtime_cache.h"

#include <algorithm>
#include <type_traits>
#include <utility>

namespace im2win {

typedef __attribute__((address_space(3))) float lds_f32;

template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), in order
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

constexpr int SH_RMAX = 3;   // a 64-pixel tile may touch at most this many output rows
constexpr int SH_G_MAX = 8;  // B operands are fetched from LDS up to this many steps ahead
// A byte offset that no output descriptor of this kernel covers (their sizes are capped at it, and
// the launcher keeps real offsets below it): the buffer unit drops a store at or beyond the size.
constexpr uint32_t OOB = 0xFFFFFF00u;

struct ShallowParams {
    const float *win;
    const float *flt;
    float *out;
    int Ho, Wo, Co, s;
    int rowlen, K;
    uint32_t npix, howo, chan_stride, ntiles;
    int fullseg;      // ((Wo-1)*s + Wf)*Hf
    int img_stride;   // Ci*Ho*rowlen : floats between the same row of consecutive images
    size_t win_elems, out_elems;   // floats in the tensor `win` points at / in the output
    // workspace-free variant only: `win` is then the NCHW input itself
    int Hi, Wi, p;
    int in_plane, in_img;   // Hi*Wi, Ci*Hi*Wi
    FastDiv d_wo, d_ho, d_howo;
};

// Compile-time description of MFMA step i of the K loop.
template <int HF, int WF, int CI>
struct Steps {
    static constexpr int KHW = HF * WF, KH2 = (KHW + 1) / 2, NPAIR = CI / 2, ODD = CI & 1;
    static constexpr int T = NPAIR * KHW + ODD * KH2;
    // The odd channel's window is split between the lane halves: lanes 0-31 take positions [0, SPL), lanes
    // 32-63 [SPL, KHW), KH2 steps with one zero slice where a half has one position fewer.  11x11: SPL is a
    // multiple of four floats (60, the zero slice then being the first half's last step), which keeps the second
    // half's operands 16-byte aligned; the other windows split at KH2 (zero slice: the second half's last step).
    static constexpr int SPL = HF == 11 ? ((KHW / 2) & ~3) : KH2;
    static_assert(SPL <= KH2 && KHW - SPL <= KH2, "both halves fit the split steps");
    // window position of split step t for lane half hh, or -1: zero slice
    __host__ __device__ static constexpr int split_pos(int t, int hh) { return hh ? (SPL + t < KHW ? SPL + t : -1) : (t < SPL ? t : -1); }
    __host__ __device__ static constexpr bool is_pair(int i) { return i < NPAIR * KHW; }
    // window position (v*HF + u) -> filter position (u*WF + v)
    __host__ __device__ static constexpr int filt_pos(int t) { return (t % HF) * WF + (t / HF); }
};

// The B operand reads of one wave's TW steps (steps ksi*TW ...), grouped into units: four consecutive steps whose
// operands are four consecutive LDS words starting at a multiple of four -- one 16-byte read -- or a single step.
// Offsets are relative to the lane's pair base (window start in the strip of its channel of the pair) or split
// base (window start + its half's first position in the odd channel's strip); SS: floats per channel strip.
template <int TW>
struct ReadUnits {
    int n;
    int first[TW], len[TW], split[TW], off[TW];   // per unit: first step, steps, which base, offset in floats
    int unit_of[TW];                              // per step: its unit
};
template <class St, int TW, int SS>
constexpr ReadUnits<TW> make_read_units(int ksi)
{
    ReadUnits<TW> u{};
    auto is_split = [](int i) { return !St::is_pair(i); };
    auto offs = [](int i) { return St::is_pair(i) ? 2 * (i / St::KHW) * SS + i % St::KHW : i - St::NPAIR * St::KHW; };
    int k = 0;
    for (int s = 0; s < TW;) {
        const int i = ksi * TW + s;
        bool quad = s + 3 < TW && offs(i) % 4 == 0;
        for (int e = 1; e < 4 && quad; ++e)
            quad = is_split(i + e) == is_split(i) && offs(i + e) == offs(i) + e;
        const int len = quad ? 4 : 1;
        u.first[k] = s; u.len[k] = len; u.split[k] = is_split(i) ? 1 : 0; u.off[k] = offs(i);
        for (int e = 0; e < len; ++e) u.unit_of[s + e] = k;
        s += len;
        ++k;
    }
    u.n = k;
    return u;
}

// IMP: workspace-free variant.  P.win is the NCHW input and each tile's im2win strips
// (Eq. 2) are gathered from it: strip word kk*HF + u of a row segment is input row
// m*s + u - p, column (first column of the segment) + kk - p, or zero padding.  The
// LDS layout, the MFMA chain and the results are the same.
// G: a tile is G groups of 64 pixels.  Each wave then advances G independent 32x32 blocks with
// the same filter registers (step by step, G MFMAs per step), and the per-tile work (geometry,
// barrier, state hand-over) is paid once per 64*G pixels -- what layers with a very short K
// (3x3x3 = 14 MFMA steps) need.
// WIDE (with G == 4, output planes of a multiple of four pixels, a 16-byte aligned output): lane
// l32 of a wave takes pixels 4*l32 .. 4*l32+3 of the wave's 128, one per group, so the four
// accumulators of a channel that a lane holds are neighbours in memory and leave in one 16-byte
// store: a wave's store instruction then writes 512 contiguous bytes per channel instead of 128.
// Such layers are bound by their output stream, and 128-byte runs that do not start on a line
// boundary (planes of 222x222) are written at well under half the rate of long runs.
// Waves per SIMD the register allocation of an instance is held to (its minimum occupancy).
// The 7x7 instances run three waves per SIMD; left alone the allocator takes a few registers
// too many for the third.  (The workspace-free ones would spill.)
template <int HF, bool IMP, int G>
constexpr int shallow_waves_per_simd() { return (HF == 7 && G == 1 && !IMP) ? 3 : 1; }

// BV (11x11 with a stride that is a multiple of four, two-call path): every window then starts a multiple
// of four floats into its row segment, the segments are placed at multiples of four floats in LDS, and the B
// operands of four consecutive K steps -- four consecutive window words -- are one aligned 16-byte LDS read.
// Windows 44 floats apart put a wave's 32 single-word reads into eight banks (4-way conflicts); the 16-byte
// reads of eight neighbouring lanes cover all 32.
template <int HF, int WF, int CI, int WM, int KS, int JX, bool IMP, int G, bool WIDE, bool BV = false>
__global__ __launch_bounds__(64 * WM * 2 * KS) __attribute__((amdgpu_waves_per_eu(shallow_waves_per_simd<HF, IMP, G>())))
void conv_mfma_shallow_kernel(ShallowParams P)
{
    using St = Steps<HF, WF, CI>;
    constexpr int KHW = St::KHW, KH2 = St::KH2, NPAIR = St::NPAIR, T = St::T;
    constexpr int TW = T / KS;                 // MFMA steps per wave
    constexpr int NT = 64 * WM * 2 * KS;       // threads per workgroup
    constexpr int SS = JX * NT;                // LDS floats per channel strip
    constexpr int STAGE = CI * SS + 4;         // one LDS stage: CI strips + a zero slot
    constexpr int SH_G = (KS == 2 || WIDE) ? 4 : SH_G_MAX;   // shorter rings where registers are scarce
    constexpr int NBT = NB * G;                // pixels per tile
    static_assert(T % KS == 0, "K steps must split evenly between the waves of a block");
    static_assert(G == 1 || KS == 1, "pixel groups are not combined with a split K");
    static_assert(!WIDE || G == 4, "16-byte stores take one pixel from each of four groups");
    static_assert(!BV || (G == 1 && !IMP && !WIDE && St::SPL % 4 == 0 && HF % 2 == 1), "16-byte operand reads: aligned windows and split");

    extern __shared__ __align__(16) unsigned char smem[];
    lds_f32 *lds = (lds_f32 *)reinterpret_cast<float *>(smem);   // [2][STAGE] then the exchange area

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: kept in a scalar register
    const int ks = wave % KS, wm = (wave / KS) % WM, wn = wave / (KS * WM);
    const int h = lane >> 5, l32 = lane & 31;
    const int mrow = (int)blockIdx.y * (WM * 32) + wm * 32 + l32;   // this lane's filter row

    // ---- A operand: this wave's K steps of filter row mrow, kept in registers ----
    // Step i of lane half hh reads filter element elem(i, hh) of the row (or is the
    // one zero slice of an odd window).  The element index is picked with scalar
    // selects on the wave's K share and one vector select on the lane half, so each
    // register costs one load.
    float a[TW];
    {
        const float *frow = P.flt + (size_t)min(mrow, P.Co - 1) * P.K;
        const bool live = mrow < P.Co;
        auto elem = [](int i, int hh) -> int {   // -1: zero slice
            if (St::is_pair(i)) return (2 * (i / KHW) + hh) * KHW + St::filt_pos(i % KHW);
            const int t = St::split_pos(i - NPAIR * KHW, hh);
            return t >= 0 ? (CI - 1) * KHW + St::filt_pos(t) : -1;
        };
#pragma unroll
        for (int ii = 0; ii < TW; ++ii) {
            int e0 = elem(ii, 0), e1 = elem(ii, 1);
            if (KS == 2 && ks) { e0 = elem(TW + ii, 0); e1 = elem(TW + ii, 1); }
            const int e = h ? e1 : e0;
            const float w = frow[e < 0 ? 0 : e];
            a[ii] = (live && e >= 0) ? w : 0.0f;
        }
    }

    // ---- tile pipeline ------------------------------------------------------------
    // A tile is 64 consecutive output pixels (flattened NCHW order); it touches rows
    // q0..q1 (q = image*Ho + output row), at most SH_RMAX of them.  Row r's strip is
    // a contiguous run of the im2win tensor; the strips lie back to back in LDS.
    //
    // A wave issues its MFMAs as one dependent chain and issues in order, so work
    // placed between two MFMAs of the chain is free while work placed outside the
    // chain leaves the matrix pipe idle.  Everything a tile needs besides its MFMAs
    // is therefore cut into small pieces that ride inside the chain of the tile
    // before or after it:
    //   chain of tile T carries   - geometry, offsets and loads of tile T+1 (straight into the
    //                               other LDS stage; the workspace-free variant loads into
    //                               registers and writes LDS late in the chain, so that the
    //                               loads have had most of it to arrive),
    //                             - window position / output pointer of tile T+1,
    //                             - the output stores of tile T-1 (with KS == 2 each one
    //                               first adds the partner wave's partial sum from LDS).
    // Accumulators alternate between two register sets with the tile parity.  (The instances with
    // 16-byte stores keep one set and store a tile right behind its own chain instead.)
    const int sHf = P.s * HF;
    constexpr int NIW = CI * JX;                 // strip words per thread and tile
    constexpr int NL = (NIW + 1) / 2;            // pieces that load (and, workspace-free, write to LDS) two words each
    constexpr int NE = (KS == 2) ? 8 : 16;       // output-store pieces
    constexpr int NOP = WIDE ? 1 : G;            // output positions a lane keeps per tile
    constexpr int NSTP = WIDE ? 0 : NE * G;      // store pieces that ride in the next tile's chain
    constexpr int P_GEO = 0, P_OFF = 4, P_LD = P_OFF + JX, P_WPOS = P_LD + NL, P_OPTR = P_WPOS + G,
                  P_ST = P_OPTR + NOP, P_LDS = P_ST + NSTP, NP = P_LDS + NL;
    // pixel of the tile that lane l32 of pixel half wn computes in group g
    auto tile_pixel = [&](int g) __attribute__((always_inline)) { return WIDE ? wn * (32 * G) + G * l32 + g : g * NB + wn * 32 + l32; };

    // state of the tile being fetched ("n": next) -- wave-uniform unless noted
    uint32_t nP0 = 0, nPend = 0, nq0 = 0, nq1 = 0, nimg0 = 0;
    int nnlo0 = 0, nlen0 = 0, nm0r = 0, nt1 = 0, nt2 = 0, nd1 = 0, nd2 = 0, nfilled = 1;
    size_t nbase = 0;
    uint32_t noff[JX];      // per thread: byte offset of its strip words from nbase
    int nlpos[JX];          // (IMP) per thread: LDS strip position of each of its words
    uint32_t nzero = 0;     // (IMP) per thread: bit j set when word j is zero padding (or unused)
    // (IMP) per row segment r of the tile, wave-uniform: columns, their reciprocal, float offset
    // of (row m*s - p, column nlo*s - p) from nbase, and those two coordinates
    int gncol0 = 1, gncol1 = 1, gncol2 = 1, ggb0 = 0, ggb1 = 0, ggb2 = 0;
    int ghb0 = 0, ghb1 = 0, ghb2 = 0, gwb0 = 0, gwb1 = 0, gwb2 = 0;
    float grcp0 = 1.f, grcp1 = 1.f, grcp2 = 1.f;
    float ir[NIW];          // per thread: the strip words in flight
    int nwpos[G];           // per lane and pixel group: LDS position of its window
    // Output stores go through a buffer descriptor whose base is wave-uniform (first
    // channel of the wave, image of the tile's first pixel); the lane adds a 32-bit
    // byte offset (its pixel, its first channel) and each store a scalar channel offset.
    size_t nobase = 0;      // uniform: float offset of that base in the output
    uint32_t nooff[G];      // per lane and group: byte offset from the base, or OOB when its pixel is past the layer
    // state of the tile being computed ("c") and of the one before it ("p")
    int cwpos[G];
    size_t cobase = 0, pobase = 0;
    uint32_t cooff[G], pooff[G];
#pragma unroll
    for (int g = 0; g < G; ++g) { nwpos[g] = 0; nooff[g] = OOB; cwpos[g] = 0; cooff[g] = OOB; pooff[g] = OOB; }
    floatx16 acc[2][G];
    float own[8];           // (KS == 2) this wave's partial sums of that half, kept from the previous tile
    // (KS == 2) this lane's slots in the exchange area: where it leaves the partner's half of a tile's
    // sums and where it finds its own half of the partner's.  One register each, computed once and made
    // opaque, so that every access is base + immediate (parity and register index are compile-time);
    // left to itself the compiler kept a separate address register per access and spilled them, and
    // every reload then waited for all memory traffic in flight.
    const lds_f32 *xmine = lds, *xtheirs = lds;
    if (KS == 2) {
        uint32_t om = (uint32_t)(2 * STAGE + ((wn * WM + wm) * 2 + ks) * 512 + lane) * 4u;
        uint32_t ot = (uint32_t)(2 * STAGE + ((wn * WM + wm) * 2 + (ks ^ 1)) * 512 + lane) * 4u;
        asm volatile("" : "+v"(om), "+v"(ot));
        xmine = (const lds_f32 *)((const __attribute__((address_space(3))) char *)lds + om);
        xtheirs = (const lds_f32 *)((const __attribute__((address_space(3))) char *)lds + ot);
    }

    // Tiles of this workgroup: tile0, tile0 + tstep, ... below tile_end.  The grid takes the tiles
    // round by round, and workgroups that share an XCD (every eighth one) take neighbouring tiles of
    // a round: what an XCD writes at any time is one contiguous stretch of every output plane, so
    // the cache lines that two tiles share are completed in its L2 while they are still there, and
    // memory sees long runs.  (Measured against one contiguous range of tiles per workgroup: Table 2's
    // Conv7 481 -> 359 us, Conv3 272 -> 261 us, never slower.)
    const uint32_t tstep = gridDim.x, tile_end = P.ntiles;
    const uint32_t xcd = blockIdx.x % 8u;
    const uint32_t tile0 = xcd * (tstep / 8u) + min(xcd, tstep % 8u) + blockIdx.x / 8u;
    if (tile0 >= tile_end) return;   // whole workgroup: no barrier is skipped by part of it
    const int jw = (int)blockIdx.y * (WM * 32) + wm * 32;   // first channel of this wave
    const int jl = jw + 4 * h;                               // first channel of this lane
    const uint32_t howo4 = P.howo * 4u;
    const int room = P.Co - jl;                              // channels this lane may store (<= 0: none)
    const bool chan_full = P.Co - jw >= 32;                  // wave-uniform: every lane of the wave stores all of its channels

    // A wave-uniform 32-bit value made opaque to the optimiser, in a scalar register.  (In the
    // multi-group instances the compiler does not always prove the value uniform, hence the
    // explicit first-lane read there.)
    auto pin = [](auto &x) __attribute__((always_inline)) {
        if constexpr (G == 1) {
            asm volatile("" : "+s"(x));
        } else {
            int v = __builtin_amdgcn_readfirstlane((int)x);
            asm volatile("" : "+s"(v));
            x = (std::remove_reference_t<decltype(x)>)v;
        }
    };
    // Buffer descriptor over `elems` floats from `base`, its size saturated to 4 GiB - 1 with
    // word-sized scalar operations (a 64-bit compare would go to the vector ALU).
    auto make_desc = [&](float *base, size_t elems) __attribute__((always_inline)) {
        const size_t left = elems * 4u;
        uint32_t lo = (uint32_t)left, hi = (uint32_t)(left >> 32);
        pin(hi);   // (left alone, the two words are recombined into that 64-bit compare)
        const uint32_t num = min(lo | (0u - (uint32_t)(hi != 0u)), OOB);
        return __builtin_amdgcn_make_buffer_rsrc(base, 0, num, 0x00020000);
    };
    // Descriptor over the output from float offset `obase` to its end.
    auto out_desc = [&](size_t obase) __attribute__((always_inline)) { return make_desc(P.out + obase, P.out_elems - obase); };
    __amdgpu_buffer_rsrc_t cdesc = out_desc(0), pdesc = out_desc(0);   // descriptors of the computed / previous tile
    // Every output store is issued by every wave on every tile, with no branch and no lane mask
    // around it: a lane that must not store (its pixel past the layer, its channel past Co) gives
    // the offset OOB, which no descriptor covers, and the buffer unit drops its write.  A fixed
    // number of stores per tile is what lets the wave count them at the end of the tile (see
    // strips_landed).  The channel test is skipped by a scalar branch in waves whose 32 channels all
    // exist.  dj: channel offset of accumulator register q from the lane's first channel.
    auto store_offset = [&](uint32_t ooff, int dj) __attribute__((always_inline)) -> uint32_t {
        uint32_t vo = ooff;
        if (__builtin_expect(!chan_full, 0)) {
            vo = dj < room ? vo : OOB;
            asm volatile("" : "+v"(vo));   // (keeps this a branch: as a select it is one more vector instruction per store)
        }
        return vo;
    };
    // One piece of the work for tile `t` (pieces are numbered in dependency order).
    auto piece = [&](auto pc, uint32_t t, int st_next, const floatx16 (&pacc)[G], int xpar) __attribute__((always_inline)) {
        constexpr int p = decltype(pc)::value;
        if constexpr (p == P_GEO) {
            nP0 = t * NBT;
            nPend = min(nP0 + NBT - 1, P.npix - 1);
            nq0 = fdiv(nP0, P.d_wo);
            nq1 = fdiv(nPend, P.d_wo);
            nnlo0 = (int)(nP0 - nq0 * (uint32_t)P.Wo);
            nlen0 = (((nq1 == nq0) ? (int)(nPend - nP0) : (P.Wo - 1 - nnlo0)) * P.s + WF) * HF;
            // The scalar results are made opaque here so that the optimiser leaves this
            // arithmetic in its own MFMA slot instead of sinking all of it to the first use.
            pin(nq0); pin(nq1); pin(nnlo0); pin(nlen0);
        } else if constexpr (p == P_GEO + 1) {
            nimg0 = fdiv(nq0, P.d_ho);
            nm0r = (int)(nq0 - nimg0 * (uint32_t)P.Ho);
            if (IMP) {
                nbase = (size_t)nimg0 * P.in_img;
                gncol0 = nlen0 / HF;
                grcp0 = __builtin_amdgcn_rcpf((float)gncol0);
                ghb0 = nm0r * P.s - P.p;
                gwb0 = nnlo0 * P.s - P.p;
                ggb0 = ghb0 * P.Wi + gwb0;
            } else {
                nbase = ((size_t)nimg0 * P.img_stride) + (size_t)nm0r * P.rowlen + (size_t)(nnlo0 * sHf);
            }
            nfilled = nlen0;
            pin(nimg0); pin(nm0r);
        } else if constexpr (p == P_GEO + 2 || p == P_GEO + 3) {
            // row r = 1 or 2 of the tile: LDS position where it starts, and
            // (source float offset relative to nbase) - (LDS position)
            constexpr int r = p - P_GEO - 1;
            const uint32_t q = nq0 + r;
            const bool has = q <= nq1;
            const uint32_t img = fdiv(q, P.d_ho);
            const int mq = (int)(q - img * (uint32_t)P.Ho);
            const int nhi = (q == nq1) ? (int)(nPend - q * (uint32_t)P.Wo) : P.Wo - 1;
            // LDS position of the segment: right behind the one before it (BV: at the next multiple of four floats)
            const int pos1 = BV ? (nlen0 + 3) & ~3 : nlen0;
            const int pos = r == 1 ? pos1 : (BV ? (pos1 + P.fullseg + 3) & ~3 : pos1 + P.fullseg);
            const int d = (int)(img - nimg0) * P.img_stride + (mq - nm0r) * P.rowlen - nnlo0 * sHf - pos;
            if (r == 1) { nt1 = has ? pos : 0x3fffffff; nd1 = has ? d : 0; }
            else        { nt2 = has ? pos : 0x3fffffff; nd2 = has ? d : 0; }
            if (IMP) {
                const int nc = nhi * P.s + WF, hb = mq * P.s - P.p;
                const float rc = __builtin_amdgcn_rcpf((float)nc);
                const int gb = (int)(img - nimg0) * P.in_img + hb * P.Wi - P.p;
                if (r == 1) { gncol1 = nc; grcp1 = rc; ghb1 = hb; gwb1 = -P.p; ggb1 = gb; }
                else        { gncol2 = nc; grcp2 = rc; ghb2 = hb; gwb2 = -P.p; ggb2 = gb; }
            }
            if (BV) nfilled = has ? pos + (nhi * P.s + WF) * HF : nfilled;
            else nfilled += has ? (nhi * P.s + WF) * HF : 0;
            if (r == 1) { pin(nt1); pin(nd1); } else { pin(nt2); pin(nd2); }
            pin(nfilled);
        } else if constexpr (p >= P_OFF && p < P_LD) {
            constexpr int j = p - P_OFF;
            if (IMP) {
                // word g of the tile's gather list: segment, then (u, kk) with u outer so that
                // neighbouring lanes read neighbouring input words
                const int g = tid + NT * j;
                const bool in1 = g >= nt1, in2 = g >= nt2;
                // (plain values first: selects are taken between values, not between references)
                const int t1 = nt1, t2 = nt2, c0 = gncol0, c1 = gncol1, c2 = gncol2;
                const float r0 = grcp0, r1 = grcp1, r2 = grcp2;
                const int b0 = ggb0, b1 = ggb1, b2 = ggb2, h0 = ghb0, h1 = ghb1, h2 = ghb2;
                const int w0 = gwb0, w1 = gwb1, w2 = gwb2;
                const int segoff = in2 ? t2 : (in1 ? t1 : 0);
                const int ncol = in2 ? c2 : (in1 ? c1 : c0);
                const float rcp = in2 ? r2 : (in1 ? r1 : r0);
                const int gb = in2 ? b2 : (in1 ? b1 : b0);
                const int hb = in2 ? h2 : (in1 ? h1 : h0);
                const int wb = in2 ? w2 : (in1 ? w1 : w0);
                const int x = g - segoff;
                // x / ncol: (x + 0.5) / ncol is at least 0.5/ncol away from an integer, far more
                // than the rounding error of the two float operations
                const int u = (int)(((float)x + 0.5f) * rcp);
                const int kk = x - u * ncol;
                const bool used = g < nfilled;
                const bool inside = used & ((uint32_t)(hb + u) < (uint32_t)P.Hi) & ((uint32_t)(wb + kk) < (uint32_t)P.Wi);
                noff[j] = inside ? (uint32_t)(gb + u * P.Wi + kk) * 4u : 0u;
                nlpos[j] = used ? segoff + kk * HF + u : g;
                nzero = inside ? (nzero & ~(1u << j)) : (nzero | (1u << j));
            } else {
                const int xc = min(tid + NT * j, nfilled - 1);   // words past the strips are never operands
                int d = xc < nt1 ? 0 : nd1;
                d = xc < nt2 ? d : nd2;
                noff[j] = (uint32_t)(xc + d) * 4u;
            }
        } else if constexpr (p >= P_LD && p < P_WPOS) {
            // descriptor on the tile's first strip word; the channel is a scalar offset.  The strips are
            // copied as they lie in memory, lane after lane, so the loads write LDS directly (no staging
            // registers, no LDS store instructions): the wave's 64 words land at the uniform address in M0.
            // The workspace-free variant permutes the words and takes them through registers.
            const __amdgpu_buffer_rsrc_t rw = make_desc(const_cast<float *>(P.win + nbase), P.win_elems - nbase);
#pragma unroll
            for (int w = 2 * (p - P_LD); w < 2 * (p - P_LD) + 2 && w < NIW; ++w) {
                const uint32_t soff = (uint32_t)(w / JX) * (IMP ? (uint32_t)P.in_plane : P.chan_stride) * 4u;
                if constexpr (IMP) {
                    ir[w] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rw, noff[w % JX], soff, 0));
                } else {
                    // (the wave's share of the destination is made opaque here: left to itself the compiler keeps
                    // all 2*NIW destinations of the two stages in scalar registers for the whole kernel, spills them
                    // to vector lanes and reads each back with a vector instruction per tile)
                    uint32_t wv = (uint32_t)wave * 64u;
                    if constexpr (!WIDE) asm volatile("" : "+s"(wv));   // (the one-workgroup-per-CU instances measured 1 % slower with it)
                    lds_f32 *dst = lds + st_next * STAGE + (w / JX) * SS + NT * (w % JX) + wv;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (__attribute__((address_space(3))) void *)dst, 4,
                                                             noff[w % JX], soff, 0, 0);
                }
            }
        } else if constexpr (p >= P_WPOS && p < P_OPTR) {
            constexpr int g = p - P_WPOS;
            if constexpr (WIDE) {
                // The lane's four neighbouring pixels: one division for the first, the others follow it in its
                // row or (rows are at least four pixels long here) start the next row's strip.  A lane whose
                // pixels are past the layer computes the layer's last four again (never stored).
                if constexpr (g == 0) {
                    const uint32_t Pl = min(nP0 + (uint32_t)tile_pixel(0), nPend - 3u);
                    const uint32_t ql = fdiv(Pl, P.d_wo);
                    const int nl = (int)(Pl - ql * (uint32_t)P.Wo);
                    const int rho = (int)(ql - nq0);
                    const int w0 = (rho == 0 ? -nnlo0 * sHf : nlen0 + (rho - 1) * P.fullseg) + nl * sHf;
                    const int wrapped = nlen0 + rho * P.fullseg + (nl - P.Wo) * sHf;   // counted from the next row's strip
#pragma unroll
                    for (int gg = 0; gg < G; ++gg) nwpos[gg] = (nl + gg >= P.Wo ? wrapped : w0) + gg * sHf;
                }
            } else {
                const uint32_t Pl = min(nP0 + (uint32_t)tile_pixel(g), nPend);
                const uint32_t ql = fdiv(Pl, P.d_wo);
                const int nl = (int)(Pl - ql * (uint32_t)P.Wo);
                const int rho = (int)(ql - nq0);
                if (BV) nwpos[g] = rho == 0 ? (nl - nnlo0) * sHf : (rho == 1 ? nt1 : nt2) + nl * sHf;   // (the segment's own position)
                else nwpos[g] = rho == 0 ? (nl - nnlo0) * sHf : nlen0 + (rho - 1) * P.fullseg + nl * sHf;
            }
        } else if constexpr (p >= P_OPTR && p < P_ST) {
            constexpr int g = p - P_OPTR;
            const uint32_t Pm = nP0 + (uint32_t)tile_pixel(g);   // (WIDE: the first of the lane's four pixels)
            const uint32_t Pc = min(Pm, nPend);
            const uint32_t img = fdiv(Pc, P.d_howo);
            const uint32_t pin = Pc - img * P.howo;
            const uint32_t img0 = fdiv(nP0, P.d_howo);   // uniform
            nobase = ((size_t)img0 * P.Co + jw) * P.howo;
            const uint32_t off = ((img - img0) * (uint32_t)P.Co * P.howo + pin) * 4u + (uint32_t)(4 * h) * howo4;
            nooff[g] = Pm <= nPend ? off : OOB;
        } else if constexpr (p >= P_ST && p < P_LDS) {
            // one output store of the previous tile (pixel group g, register q of its block)
            constexpr int g = (p - P_ST) / NE, q = (p - P_ST) % NE;
            if constexpr (KS == 2) {
                // add the partner's partial sum to this wave's (kept in own[]) first; these
                // instances are short of scalar registers and rebuild the descriptor here
                const float val = own[q] + *(const volatile lds_f32 *)(xtheirs + xpar * (WM * 2 * 2 * 512) + q * 64);
                const int dj = (ks ? 16 : 0) + 8 * (q >> 2) + (q & 3);
                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, val), out_desc(pobase), store_offset(pooff[0], dj), (uint32_t)dj * howo4, 0);
            } else {
                const int dj = 8 * (q >> 2) + (q & 3);
                const float val = pacc[g][q];
                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, val), pdesc, store_offset(pooff[g], dj), (uint32_t)dj * howo4, 0);
            }
        } else if constexpr (p >= P_LDS && p < NP) {
            if constexpr (IMP) {
#pragma unroll
                for (int w = 2 * (p - P_LDS); w < 2 * (p - P_LDS) + 2 && w < NIW; ++w)
                    lds[st_next * STAGE + (w / JX) * SS + nlpos[w % JX]] = ((nzero >> (w % JX)) & 1u) ? 0.0f : ir[w];
            }
        }
    };
    // The next tile's strips must be in LDS before the barrier that ends a tile.  The direct loads
    // are counted by the wave's vector-memory counter, which the output stores share, and the
    // counter retires in issue order.  A tile's loads are issued before the stores that ride in the
    // same chain, and every wave issues all of those stores, so the loads have landed as soon as no
    // more than that many operations are outstanding: the wave does not wait for its stores to be
    // acknowledged, which at one or two waves per SIMD would idle the matrix pipe once per tile.
    // (The other counters are left alone.)
    constexpr int NSTORES = NE * NOP < 63 ? NE * NOP : 63;   // store instructions per tile and wave behind its loads (the counter holds 63)
    auto strips_landed = [](bool stores_behind) __attribute__((always_inline)) {
        if (IMP) return;
        if (stores_behind) __builtin_amdgcn_s_waitcnt(0x0F70 | (NSTORES & 15) | ((NSTORES >> 4) << 14));
        else __builtin_amdgcn_s_waitcnt(0x0F70);
    };
    // Workgroup barrier between tiles.  Only LDS traffic has to be ordered across it (the strips, the
    // K-half exchange); a fence over all address spaces would also wait for every output store.
    auto tile_barrier = []() __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };
    // pieces lo..hi-1
    auto pieces = [&](auto loc, auto hic, uint32_t t, int st_next, const floatx16 (&pacc)[G], int xpar) __attribute__((always_inline)) {
        constexpr int lo = decltype(loc)::value, hi = decltype(hic)::value;
        static_for<hi - lo>([&](auto k) __attribute__((always_inline)) { piece(std::integral_constant<int, lo + decltype(k)::value>{}, t, st_next, pacc, xpar); });
    };

    if (tid < 8) { lds[CI * SS + (tid & 3) + (tid >> 2) * STAGE] = 0.0f; }   // zero slots of both stages

    // ---- prologue: tile0's strips into stage 0 (all "next tile" pieces but the stores) ----
    {
        floatx16 z;
#pragma unroll
        for (int v = 0; v < 16; ++v) z[v] = 0.0f;
#pragma unroll
        for (int g = 0; g < G; ++g) { acc[0][g] = z; acc[1][g] = z; }
        pieces(std::integral_constant<int, P_GEO>{}, std::integral_constant<int, P_ST>{}, tile0, 0, acc[0], 0);
        pieces(std::integral_constant<int, P_LDS>{}, std::integral_constant<int, NP>{}, tile0, 0, acc[0], 0);
    }
    strips_landed(false);
    __syncthreads();

    // ---- one tile: the MFMA chain with the pieces in its shadow -------------------
    auto tile_body = [&](auto parc, uint32_t tile) __attribute__((always_inline)) {
        constexpr int PAR = decltype(parc)::value;      // tile parity: LDS stage, accumulator set
        constexpr int AP = (KS == 2 || WIDE) ? 0 : PAR;   // with KS == 2 only 8 sums outlive the chain (own[]); WIDE: none
        // the fetched tile becomes the computed tile
        cobase = nobase;
        if (KS == 1) cdesc = out_desc(cobase);
#pragma unroll
        for (int g = 0; g < G; ++g) { cwpos[g] = nwpos[g]; cooff[g] = nooff[g]; }
        const uint32_t nxt = tile + tstep < tile_end ? tile + tstep : tile;   // the last tile refetches itself (unused)
        const lds_f32 *sbase = lds + PAR * STAGE;
        const lds_f32 *bpair[G], *bsplit[G], *bzero[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            bpair[g] = sbase + cwpos[g] + h * SS;
            bsplit[g] = sbase + cwpos[g] + (CI - 1) * SS + h * St::SPL;
            // the zero slice: a zero word where the half's last step would read past the window (the second half,
            // split at KH2); a first half that ends early re-reads the other half's first position, times a zero
            // filter register (a word of the lane's own window)
            bzero[g] = (h && St::SPL + KH2 > KHW) ? sbase + CI * SS : bsplit[g] + (KH2 - 1);
        }
        auto run = [&](auto ksc) __attribute__((always_inline)) {
            constexpr int KSI = decltype(ksc)::value;
            auto bread = [&](int ii, int g) __attribute__((always_inline)) -> float {
                const int i = KSI * TW + ii;   // global step index (compile-time after unrolling)
                if (St::is_pair(i)) {
                    const int pp = i / KHW, t = i % KHW;
                    return *(const volatile lds_f32 *)(bpair[g] + 2 * pp * SS + t);
                }
                const int t = i - NPAIR * KHW;
                if (t == KH2 - 1) return *(const volatile lds_f32 *)bzero[g];
                return *(const volatile lds_f32 *)(bsplit[g] + t);
            };
            if constexpr (BV) {
                // 16-byte operand reads: a ring of NU units (quads or single words), unit k + NU fetched right
                // behind the last MFMA of unit k
                constexpr ReadUnits<TW> U = make_read_units<St, TW, SS>(KSI);
                constexpr int NU = 3;
                typedef float f32x4 __attribute__((ext_vector_type(4)));
                typedef __attribute__((address_space(3))) f32x4 lds_f32x4;
                f32x4 bu[NU];
                auto fetch = [&](auto kc) __attribute__((always_inline)) {
                    constexpr int k = decltype(kc)::value;
                    const lds_f32 *ptr = (U.split[k] ? bsplit[0] : bpair[0]) + U.off[k];
                    if constexpr (U.len[k] == 4) bu[k % NU] = *(const volatile lds_f32x4 *)ptr;
                    else bu[k % NU].x = *(const volatile lds_f32 *)ptr;
                };
                static_for<(NU < U.n ? NU : U.n)>([&](auto kc) __attribute__((always_inline)) { fetch(kc); });
                __builtin_amdgcn_sched_barrier(0);
                static_for<TW>([&](auto ic) __attribute__((always_inline)) {
                    constexpr int ii = decltype(ic)::value;
                    constexpr int k = U.unit_of[ii], e = ii - U.first[k];
                    if constexpr (ii == 0) {
                        floatx16 z;
#pragma unroll
                        for (int v = 0; v < 16; ++v) z[v] = 0.0f;
                        acc[AP][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], bu[0][0], z, 0, 0, 0);
                    } else {
                        acc[AP][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ii], bu[k % NU][e], acc[AP][0], 0, 0, 0);
                    }
                    if constexpr (e == U.len[k] - 1 && k + NU < U.n) fetch(std::integral_constant<int, k + NU>{});
                    constexpr int m = ii, NM = TW;
                    constexpr int plo = (m * NP + NM - 1) / NM, phi = ((m + 1) * NP + NM - 1) / NM;
                    pieces(std::integral_constant<int, plo>{}, std::integral_constant<int, phi>{}, nxt, PAR ^ 1, acc[AP ^ 1], PAR ^ 1);
                    __builtin_amdgcn_sched_barrier(0);
                });
            } else {
                float b[G][SH_G];   // rings of B operands, SH_G steps ahead of the MFMAs
    #pragma unroll
                for (int e = 0; e < SH_G; ++e)
    #pragma unroll
                    for (int g = 0; g < G; ++g)
                        if (e < TW) b[g][e] = bread(e, g);
                __builtin_amdgcn_sched_barrier(0);
                static_for<TW>([&](auto ic) __attribute__((always_inline)) {
                    constexpr int ii = decltype(ic)::value;
                    static_for<G>([&](auto gc) __attribute__((always_inline)) {
                        constexpr int g = decltype(gc)::value;
                        if constexpr (ii == 0) {
                            floatx16 z;
    #pragma unroll
                            for (int v = 0; v < 16; ++v) z[v] = 0.0f;
                            acc[AP][g] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[g][0], z, 0, 0, 0);
                        } else {
                            acc[AP][g] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ii], b[g][ii % SH_G], acc[AP][g], 0, 0, 0);
                        }
                        if (ii + SH_G < TW) b[g][ii % SH_G] = bread(ii + SH_G, g);
                        // pieces whose slot is this MFMA: piece p rides behind MFMA p*(TW*G)/NP of the tile
                        constexpr int m = ii * G + g, NM = TW * G;
                        constexpr int plo = (m * NP + NM - 1) / NM, phi = ((m + 1) * NP + NM - 1) / NM;
                        pieces(std::integral_constant<int, plo>{}, std::integral_constant<int, phi>{}, nxt, PAR ^ 1, acc[AP ^ 1], PAR ^ 1);
                        __builtin_amdgcn_sched_barrier(0);
                    });
                });
            }
            if constexpr (WIDE) {
                // The tile's sums leave right behind its chain, from the one set of accumulators: register q
                // of the wave's four blocks is a lane's four neighbouring pixels of channel dj (all inside the
                // layer or all outside: the pixel count is a multiple of four here).  This wave's matrix pipe
                // idles meanwhile; the other workgroup of the CU fills it.
                typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                typedef float f32x4 __attribute__((ext_vector_type(4)));
                auto store_all = [&](auto fullc) __attribute__((always_inline)) {
                    static_for<16>([&](auto qc) __attribute__((always_inline)) {
                        constexpr int q = decltype(qc)::value;
                        constexpr int dj = 8 * (q >> 2) + (q & 3);
                        f32x4 v;   // (element by element: a bit cast applied to a vector element reads element 0)
                        v.x = acc[0][0][q]; v.y = acc[0][1][q]; v.z = acc[0][2][q]; v.w = acc[0][3][q];
                        uint32_t vo = cooff[0];
                        if constexpr (!decltype(fullc)::value) vo = dj < room ? vo : OOB;
                        // Nothing is scheduled between the store and four idle cycles behind it: an instance whose
                        // allocation rewrote a store's four data registers in the very next instructions wrote
                        // stale values in a few lanes now and then (the data of a 16-byte store leave the register
                        // file over several cycles).
                        __builtin_amdgcn_sched_barrier(0);
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), cdesc, vo, (uint32_t)dj * howo4, 0);
                        asm volatile("s_nop 3");
                        __builtin_amdgcn_sched_barrier(0);
                    });
                };
                if (chan_full) store_all(std::true_type{});   // (one branch per tile: all 32 channels of the wave exist)
                else store_all(std::false_type{});
            }
            if (KS == 2) {
                // hand the partner the half of this tile's accumulators that it owns, keep the other
                // (register indices are compile-time constants here: KSI is this wave's K share)
                lds_f32 *mine = const_cast<lds_f32 *>(xmine) + PAR * (WM * 2 * 2 * 512);   // (ks == KSI in this instance of run)
#pragma unroll
                for (int v = 0; v < 8; ++v) mine[v * 64] = acc[0][0][KSI ? v : 8 + v];
#pragma unroll
                for (int v = 0; v < 8; ++v) own[v] = acc[0][0][KSI ? 8 + v : v];
            }
        };
        if (KS == 1) {
            run(std::integral_constant<int, 0>{});
        } else {
            if (ks == 0) run(std::integral_constant<int, 0>{});
            else run(std::integral_constant<int, KS - 1>{});
        }
        // the computed tile becomes the previous tile
        pobase = cobase;
        if (KS == 1) pdesc = cdesc;
#pragma unroll
        for (int g = 0; g < G; ++g) { pooff[g] = cooff[g]; }
        strips_landed(true);
        tile_barrier();
    };

    uint32_t tile = tile0;
    for (; tile + tstep < tile_end; tile += 2 * tstep) {   // unrolled by two: stage and accumulator set are constants
        tile_body(std::integral_constant<int, 0>{}, tile);
        tile_body(std::integral_constant<int, 1>{}, tile + tstep);
    }
    int lastpar = 1;
    if (tile < tile_end) { tile_body(std::integral_constant<int, 0>{}, tile); lastpar = 0; }

    // ---- drain: exchange reads and stores of the last tile -------------------------
    if (lastpar == 0) pieces(std::integral_constant<int, P_ST>{}, std::integral_constant<int, P_LDS>{}, 0u, 0, acc[0], 0);
    else pieces(std::integral_constant<int, P_ST>{}, std::integral_constant<int, P_LDS>{}, 0u, 0, acc[1], 1);
}

template <int HF, int WF, int CI, int WM, int KS, int JX, bool IMP, int G, bool WIDE, bool BV = false>
static hipError_t launch_shallow_k(ShallowParams P, int mgroups, hipStream_t st, LaunchPlan *plan)
{
    P.ntiles = (P.npix + NB * G - 1) / (NB * G);
    constexpr int NT = 64 * WM * 2 * KS;
    constexpr int SS = JX * NT;
    constexpr int STAGE = CI * SS + 4;
    constexpr size_t lds = 4u * (size_t)(2 * STAGE + (KS == 2 ? 2 * WM * 2 * 2 * 8 * 64 : 0));
    auto kern = &conv_mfma_shallow_kernel<HF, WF, CI, WM, KS, JX, IMP, G, WIDE, BV>;
    static KernelCache kc;
    int dev = 0, ncu = 0;
    hipError_t e = device_cus(&dev, &ncu);
    const bool blind = e != hipSuccess && plan;   // planning without a device: an MI355X's 256 compute units
    if (blind) { e = hipSuccess; ncu = 256; }
    if (e != hipSuccess) return e;
    if (!plan && (e = allow_dynamic_lds(kc, reinterpret_cast<const void *>(kern), lds, dev)) != hipSuccess) return e;
    // Persistent grid: enough workgroups to give every CU its share of resident waves.
    int per_cu = 0;
    if (blind) per_cu = (int)std::min<size_t>(3, (160 * 1024) / lds);   // (LDS is what limits these kernels)
    else if ((e = resident_per_cu(kc, reinterpret_cast<const void *>(kern), NT, lds, dev, &per_cu)) != hipSuccess) return e;
    if (per_cu < 1) return hipErrorInvalidConfiguration;
    if (per_cu > 3) per_cu = 3;
    // The instances with 16-byte stores are bound by the output stream: with one workgroup per CU the
    // tiles in flight on an XCD write 2 MB per round, which its 4 MB L2 holds until the neighbouring
    // tiles have completed the shared lines; two or three per CU measured a third slower.
    if (WIDE) per_cu = 1;
    uint32_t gx = (uint32_t)(ncu * per_cu) / (uint32_t)mgroups;
    if (gx >= 8) gx &= ~7u;   // (whole rows of the grid per XCD, whatever blockIdx.y)
    if (gx < 1) gx = 1;
    if (gx > P.ntiles) gx = P.ntiles;
    if (plan) {
        plan_record(plan, dim3(gx, mgroups), NT, lds, "conv_mfma_shallow_kernel<%d, %d, %d, %d, %d, %d, %s, %d, %s, %s>",
                    HF, WF, CI, WM, KS, JX, tf(IMP), G, tf(WIDE), tf(BV));
        return hipSuccess;
    }
    hipLaunchKernelGGL(kern, dim3(gx, mgroups), dim3(NT), lds, st, P);
    return hipGetLastError();
}

template <int HF, int WF, int CI, int WM, int KS, int JX, int G = 1, bool WIDE = false>
static hipError_t launch_shallow_t(const ShallowParams &P, int mgroups, hipStream_t st, bool implicit, LaunchPlan *plan)
{
    return implicit ? launch_shallow_k<HF, WF, CI, WM, KS, JX, true, G, WIDE>(P, mgroups, st, plan)
                    : launch_shallow_k<HF, WF, CI, WM, KS, JX, false, G, WIDE>(P, mgroups, st, plan);
}

// Returns hipErrorNotSupported when the layer does not meet this kernel's conditions.
// implicit: `win` is the NCHW input (workspace-free variant).
hipError_t launch_conv_mfma_shallow(const float *win, const float *flt, float *out, const Shape &sh,
                                    hipStream_t st, bool implicit, LaunchPlan *plan)
{
    // rows a tile of 64*g pixels may touch, and its strip floats per channel (0: too many rows)
    auto rows_of = [&](int g) {
        int r = (NB * g + sh.Wo - 2) / sh.Wo + 1;
        return r > NB * g ? NB * g : r;
    };
    auto strip_of = [&](int g) -> long long {   // (64 bits: the stride has no upper bound)
        const int r = rows_of(g);
        if (r > SH_RMAX) return 0;
        const int over = sh.Wf > sh.s ? sh.Wf - sh.s : 0;
        return ((long long)NB * g * sh.s + (long long)r * over) * sh.Hf + 1;
    };
    const long long S = strip_of(1);
    if (S == 0 || S > 4096) return hipErrorNotSupported;   // (the largest instance below holds 3072 floats per strip)
    // 32-bit strip offsets: the rows of one tile must lie within 2 GiB of each other
    const long long span = (implicit ? (long long)sh.Ci * sh.Hi * sh.Wi : (long long)sh.Ci * sh.Ho * sh.rowlen) * 4LL * (SH_RMAX + 1);
    if (span >= (1LL << 31)) return hipErrorNotSupported;
    // 32-bit output offsets from (image of the tile's first pixel, wave's first channel): up to two images
    // ahead, and all of them below the offset that stands for "no store"
    if (((long long)sh.Co * (SH_RMAX + 1) + 64) * sh.Ho * sh.Wo * 4LL >= (long long)OOB) return hipErrorNotSupported;

    ShallowParams P;
    P.win = win; P.flt = flt; P.out = out;
    P.Ho = sh.Ho; P.Wo = sh.Wo; P.Co = sh.Co; P.s = sh.s;
    P.rowlen = sh.rowlen; P.K = sh.K;
    P.npix = (uint32_t)sh.npix;
    P.howo = (uint32_t)(sh.Ho * sh.Wo);
    P.chan_stride = (uint32_t)((size_t)sh.Ho * sh.rowlen);
    P.ntiles = (P.npix + NB - 1) / NB;
    P.fullseg = ((sh.Wo - 1) * sh.s + sh.Wf) * sh.Hf;
    P.img_stride = sh.Ci * sh.Ho * sh.rowlen;
    P.win_elems = implicit ? (size_t)sh.N * sh.Ci * sh.Hi * (size_t)sh.Wi : (size_t)sh.N * P.img_stride;
    P.Hi = sh.Hi; P.Wi = sh.Wi; P.p = sh.p;
    P.in_plane = sh.Hi * sh.Wi;
    P.in_img = sh.Ci * sh.Hi * sh.Wi;
    P.out_elems = (size_t)sh.npix * sh.Co;
    P.d_wo = make_fastdiv((uint32_t)sh.Wo);
    P.d_ho = make_fastdiv((uint32_t)sh.Ho);
    P.d_howo = make_fastdiv(P.howo);

    if (sh.Ci != 3) return hipErrorNotSupported;
    const int wm = sh.Co <= 32 ? 1 : (sh.Co <= 64 ? 2 : 3);
    const int mgroups = (sh.Co + wm * 32 - 1) / (wm * 32);
    if (sh.Hf == 7 && sh.Wf == 7) {
        if (wm == 1 && S <= 4 * 128) return launch_shallow_t<7, 7, 3, 1, 1, 4>(P, mgroups, st, implicit, plan);
        if (wm == 1 && S <= 8 * 128) return launch_shallow_t<7, 7, 3, 1, 1, 8>(P, mgroups, st, implicit, plan);
        if (wm == 2 && S <= 4 * 256) return launch_shallow_t<7, 7, 3, 2, 1, 4>(P, mgroups, st, implicit, plan);
        if (wm == 3 && S <= 3 * 384) return launch_shallow_t<7, 7, 3, 3, 1, 3>(P, mgroups, st, implicit, plan);
    } else if (sh.Hf == 11 && sh.Wf == 11) {
        // 16-byte operand reads where every window starts a multiple of four floats into its row segment (the
        // segments are then placed at multiples of four in LDS: up to three floats of padding before two of them)
        const bool bv = !implicit && sh.s % 4 == 0;
        if (bv && wm == 1 && S + 6 <= 12 * 256) return launch_shallow_k<11, 11, 3, 1, 2, 12, false, 1, false, true>(P, mgroups, st, plan);
        if (bv && wm == 2 && S + 6 <= 6 * 512) return launch_shallow_k<11, 11, 3, 2, 2, 6, false, 1, false, true>(P, mgroups, st, plan);
        if (bv && wm == 3 && S + 6 <= 4 * 768) return launch_shallow_k<11, 11, 3, 3, 2, 4, false, 1, false, true>(P, mgroups, st, plan);
        if (wm == 1 && S <= 12 * 256) return launch_shallow_t<11, 11, 3, 1, 2, 12>(P, mgroups, st, implicit, plan);
        if (wm == 2 && S <= 6 * 512) return launch_shallow_t<11, 11, 3, 2, 2, 6>(P, mgroups, st, implicit, plan);
        if (wm == 3 && S <= 4 * 768) return launch_shallow_t<11, 11, 3, 3, 2, 4>(P, mgroups, st, implicit, plan);
    } else if (sh.Hf == 3 && sh.Wf == 3) {
        // K = 27 is 14 MFMA steps: tiles of four pixel groups where the layer has enough of them
        const long long S4 = strip_of(4);
        const bool many = P.npix >= 4u * NB * 4u * 768u;
        // 16-byte stores: four neighbouring pixels never straddle two output planes, and they are aligned
        const bool wide = P.howo % 4u == 0 && sh.Wo >= 4 && reinterpret_cast<uintptr_t>(out) % 16u == 0;
        if (many && S4 > 0) {
            // one or two 32-channel blocks per workgroup; the accumulators of a third do not fit the
            // register file, so wider layers run as separate groups of 32 channels
            const int wm4 = wm == 2 ? 2 : 1;
            const int mg4 = (sh.Co + wm4 * 32 - 1) / (wm4 * 32);
            if (wm4 == 1 && S4 <= 7 * 128)
                return wide ? launch_shallow_t<3, 3, 3, 1, 1, 7, 4, true>(P, mg4, st, implicit, plan)
                            : launch_shallow_t<3, 3, 3, 1, 1, 7, 4>(P, mg4, st, implicit, plan);
            if (wm4 == 2 && S4 <= 4 * 256)
                return wide ? launch_shallow_t<3, 3, 3, 2, 1, 4, 4, true>(P, mg4, st, implicit, plan)
                            : launch_shallow_t<3, 3, 3, 2, 1, 4, 4>(P, mg4, st, implicit, plan);
        }
        if (wm == 1 && S <= 2 * 128) return launch_shallow_t<3, 3, 3, 1, 1, 2>(P, mgroups, st, implicit, plan);
        if (wm == 2 && S <= 1 * 256) return launch_shallow_t<3, 3, 3, 2, 1, 1>(P, mgroups, st, implicit, plan);
        if (wm == 3 && S <= 1 * 384) return launch_shallow_t<3, 3, 3, 3, 1, 1>(P, mgroups, st, implicit, plan);
    }
    return hipErrorNotSupported;
}

}  // namespace im2win
