// Filter-stationary MFMA im2win convolution for layers with few input channels
// and a large window (the 7x7/stride-2 and 11x11/stride-4 stem layers, Table 2's
// Conv1-Conv3/Conv7): K = Ci*Hf*Wf is small (27..363) while N = Ni*Ho*Wo is huge.
//
// Design (CDNA4's, not the paper's CUDA tiling):
//   - persistent workgroups: each one walks a strided list of 64-pixel tiles;
//   - every wave keeps the A operand (its 32 filter rows, its share of K) in
//     registers for the whole kernel -- the filter is read from memory once per
//     wave, never staged per tile -- so each MFMA needs one LDS read only;
//   - the B operand is the tile's contiguous im2win strips (Section 3.1) in LDS,
//     double-buffered: the next tile's strips are loaded into registers while the
//     matrix cores work and written to the other LDS stage at the end of the tile;
//   - K order: channel pairs ride the two lane halves of v_mfma_f32_32x32x2_f32
//     ("pair" steps); an odd last channel is split in two halves of its window
//     ("split" steps); every operand address is lane base + immediate;
//   - when K is too large for one wave's registers (11x11x3 = 363) two waves
//     share a 32x32 output block, each taking half of the K steps, and exchange
//     half of their accumulators through LDS before the store (KS = 2).
#include "conv_mfma_tile.h"

#include <type_traits>

namespace im2win {

typedef __attribute__((address_space(3))) float lds_f32;

constexpr int SH_RMAX = 3;   // a 64-pixel tile may touch at most this many output rows
constexpr int SH_G = 8;      // B operands are fetched from LDS this many steps ahead

struct ShallowParams {
    const float *win;
    const float *flt;
    float *out;
    int Ho, Wo, Co, s;
    int rowlen, K;
    uint32_t npix, howo, chan_stride, ntiles;
    int fullseg;      // ((Wo-1)*s + Wf)*Hf
    int img_stride;   // Ci*Ho*rowlen : floats between the same row of consecutive images
    FastDiv d_wo, d_ho, d_howo;
};

// Compile-time description of MFMA step i of the K loop.
template <int HF, int WF, int CI>
struct Steps {
    static constexpr int KHW = HF * WF, KH2 = (KHW + 1) / 2, NPAIR = CI / 2, ODD = CI & 1;
    static constexpr int T = NPAIR * KHW + ODD * KH2;
    __host__ __device__ static constexpr bool is_pair(int i) { return i < NPAIR * KHW; }
    // window position (v*HF + u) -> filter position (u*WF + v)
    __host__ __device__ static constexpr int filt_pos(int t) { return (t % HF) * WF + (t / HF); }
};

template <int HF, int WF, int CI, int WM, int KS, int JX>
__global__ __launch_bounds__(64 * WM * 2 * KS) void conv_mfma_shallow_kernel(ShallowParams P)
{
    using St = Steps<HF, WF, CI>;
    constexpr int KHW = St::KHW, KH2 = St::KH2, NPAIR = St::NPAIR, T = St::T;
    constexpr int TW = T / KS;                 // MFMA steps per wave
    constexpr int NT = 64 * WM * 2 * KS;       // threads per workgroup
    constexpr int SS = JX * NT;                // LDS floats per channel strip
    constexpr int STAGE = CI * SS + 4;         // one LDS stage: CI strips + a zero slot
    constexpr int NG = (TW + SH_G - 1) / SH_G;
    static_assert(T % KS == 0, "K steps must split evenly between the waves of a block");

    extern __shared__ __align__(16) unsigned char smem[];
    lds_f32 *lds = (lds_f32 *)reinterpret_cast<float *>(smem);   // [2][STAGE] then the exchange area

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
            const int t = i - NPAIR * KHW + hh * KH2;
            return t < KHW ? (CI - 1) * KHW + St::filt_pos(t) : -1;
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

    // ---- per-tile geometry ------------------------------------------------------
    // A tile is 64 consecutive output pixels (flattened NCHW order); it touches rows
    // q0..q1 (q = image*Ho + output row), at most SH_RMAX of them.  Row r's strip is
    // a contiguous run of the im2win tensor; the strips lie back to back in LDS.
    // Everything below that depends only on the tile index is wave-uniform and is
    // computed on the scalar unit.
    const int sHf = P.s * HF;

    float ir[CI * JX];
    // Request the strips of `tile` from global memory (values land in ir[]).
    auto gload = [&](uint32_t tile) {
        const uint32_t P0 = tile * NB;
        const uint32_t Pend = min(P0 + NB - 1, P.npix - 1);
        const uint32_t q0 = fdiv(P0, P.d_wo), q1 = fdiv(Pend, P.d_wo);
        const int nlo0 = (int)(P0 - q0 * (uint32_t)P.Wo);
        const int len0 = (((q1 == q0) ? (int)(Pend - P0) : (P.Wo - 1 - nlo0)) * P.s + WF) * HF;
        const uint32_t img0 = fdiv(q0, P.d_ho);
        const int m0r = (int)(q0 - img0 * (uint32_t)P.Ho);
        const size_t base = ((size_t)img0 * P.img_stride) + (size_t)m0r * P.rowlen + (size_t)(nlo0 * sHf);
        // rows 1 and 2: LDS position where they start (t1, t2), their length, and
        // (source float offset relative to base) - (LDS position) = d1, d2
        int t1 = 0x3fffffff, t2 = 0x3fffffff, d1 = 0, d2 = 0, filled = len0;
        if (q0 + 1 <= q1) {
            const uint32_t q = q0 + 1;
            const uint32_t img = fdiv(q, P.d_ho);
            const int mq = (int)(q - img * (uint32_t)P.Ho);
            const int nhi = (q == q1) ? (int)(Pend - q * (uint32_t)P.Wo) : P.Wo - 1;
            t1 = len0;
            d1 = (int)(img - img0) * P.img_stride + (mq - m0r) * P.rowlen - nlo0 * sHf - len0;
            filled += (nhi * P.s + WF) * HF;
        }
        if (q0 + 2 <= q1) {
            const uint32_t q = q0 + 2;
            const uint32_t img = fdiv(q, P.d_ho);
            const int mq = (int)(q - img * (uint32_t)P.Ho);
            const int nhi = (q == q1) ? (int)(Pend - q * (uint32_t)P.Wo) : P.Wo - 1;
            t2 = len0 + P.fullseg;
            d2 = (int)(img - img0) * P.img_stride + (mq - m0r) * P.rowlen - nlo0 * sHf - t2;
            filled += (nhi * P.s + WF) * HF;
        }
        const char *gb = reinterpret_cast<const char *>(P.win + base);
#pragma unroll
        for (int j = 0; j < JX; ++j) {
            const int xc = min(tid + NT * j, filled - 1);   // words past the strips are never operands
            int d = xc < t1 ? 0 : d1;
            d = xc < t2 ? d : d2;
            const uint32_t off = (uint32_t)(xc + d) * 4u;
#pragma unroll
            for (int c = 0; c < CI; ++c)
                ir[c * JX + j] = *reinterpret_cast<const float *>(gb + (size_t)c * P.chan_stride * 4u + off);
        }
    };
    auto lds_store = [&](int st) {
        lds_f32 *d = lds + st * STAGE + tid;
#pragma unroll
        for (int c = 0; c < CI; ++c)
#pragma unroll
            for (int j = 0; j < JX; ++j) d[c * SS + NT * j] = ir[c * JX + j];
    };

    if (tid < 8) { lds[CI * SS + (tid & 3) + (tid >> 2) * STAGE] = 0.0f; }   // zero slots of both stages

    // Each workgroup walks a contiguous range of tiles: neighbouring tiles share
    // strip words (L2 hits) and write to the same pages of the output.
    const uint32_t per = (P.ntiles + gridDim.x - 1) / gridDim.x;
    uint32_t tile = blockIdx.x * per;
    const uint32_t tile_end = min(tile + per, P.ntiles);
    if (tile >= tile_end) return;   // whole workgroup: no barrier is skipped by part of it
    gload(tile);
    lds_store(0);
    __syncthreads();

    for (int it = 0; tile < tile_end; ++it, ++tile) {
        const int st = it & 1;
        const uint32_t next = tile + 1;
        const bool has_next = next < tile_end;
        if (has_next) gload(next);   // in flight during this tile's matrix work

        // ---- this tile: where the lane's window starts in the LDS strips -----------
        const uint32_t P0 = tile * NB;
        const uint32_t Pend = min(P0 + NB - 1, P.npix - 1);
        int wpos;
        {
            const uint32_t q0 = fdiv(P0, P.d_wo), q1 = fdiv(Pend, P.d_wo);
            const int nlo0 = (int)(P0 - q0 * (uint32_t)P.Wo);
            const int len0 = (((q1 == q0) ? (int)(Pend - P0) : (P.Wo - 1 - nlo0)) * P.s + WF) * HF;
            const uint32_t Pl = min(P0 + (uint32_t)(wn * 32 + l32), Pend);
            const uint32_t ql = fdiv(Pl, P.d_wo);
            const int nl = (int)(Pl - ql * (uint32_t)P.Wo);
            const int rho = (int)(ql - q0);
            wpos = rho == 0 ? (nl - nlo0) * sHf : len0 + (rho - 1) * P.fullseg + nl * sHf;
        }

        // ---- K loop: TW MFMA steps, B operands fetched SH_G steps ahead -----------
        const lds_f32 *sbase = lds + st * STAGE;
        const lds_f32 *bpair = sbase + wpos + h * SS;
        const lds_f32 *bsplit = sbase + wpos + (CI - 1) * SS + h * KH2;
        const lds_f32 *bzero = (h && (KHW & 1)) ? sbase + CI * SS : bsplit + (KH2 - 1);
        floatx16 acc;
        auto run = [&](auto ksc) {
            constexpr int KSI = decltype(ksc)::value;
            auto bread = [&](int ii) -> float {
                const int i = KSI * TW + ii;   // global step index (compile-time after unrolling)
                if (St::is_pair(i)) {
                    const int p = i / KHW, t = i % KHW;
                    return *(const volatile lds_f32 *)(bpair + 2 * p * SS + t);
                }
                const int t = i - NPAIR * KHW;
                if (t == KH2 - 1) return *(const volatile lds_f32 *)bzero;
                return *(const volatile lds_f32 *)(bsplit + t);
            };
            // The scheduling barriers pin the order "reads of group g+1, then MFMAs of
            // group g": left alone the compiler sinks every LDS read to just before its
            // MFMA and the matrix pipe waits out one LDS latency per step.
            float b[2][SH_G];
#pragma unroll
            for (int e = 0; e < SH_G; ++e)
                if (e < TW) b[0][e] = bread(e);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = 0; g < NG; ++g) {
#pragma unroll
                for (int e = 0; e < SH_G; ++e)
                    if ((g + 1) * SH_G + e < TW) b[(g + 1) & 1][e] = bread((g + 1) * SH_G + e);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int e = 0; e < SH_G; ++e) {
                    const int ii = g * SH_G + e;
                    if (ii < TW) {
                        if (ii == 0) {
                            floatx16 z;
#pragma unroll
                            for (int v = 0; v < 16; ++v) z[v] = 0.0f;
                            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0][0], z, 0, 0, 0);
                        } else {
                            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ii], b[g & 1][e], acc, 0, 0, 0);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        if (KS == 1) {
            run(std::integral_constant<int, 0>{});
        } else {
            if (ks == 0) run(std::integral_constant<int, 0>{});
            else run(std::integral_constant<int, KS - 1>{});
        }

        // ---- combine the K halves (KS == 2): each wave of a pair ends up owning 8
        // of the 16 accumulator registers of the block ------------------------------
        if (KS == 2) {
            lds_f32 *xch = lds + 2 * STAGE + ((wn * WM + wm) * 2) * (8 * 64);   // [2 waves][8][64]
            lds_f32 *mine = xch + ks * (8 * 64) + lane;
            const lds_f32 *theirs = xch + (ks ^ 1) * (8 * 64) + lane;
#pragma unroll
            for (int v = 0; v < 8; ++v) mine[v * 64] = ks ? acc[v] : acc[8 + v];   // the half the partner will own
            __syncthreads();
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                const float o = theirs[v * 64];
                if (ks) acc[8 + v] += o; else acc[v] += o;
            }
        }

        // ---- epilogue ---------------------------------------------------------------
        // Lane (h, l32) holds pixel l32 of the wave's 32 and, in register v, output
        // channel jl + 8*(v/4) + v%4 with jl = block base + 4*h.  The per-lane part of
        // the address is formed once; the per-register part is wave-uniform.
        {
            const uint32_t Pm = P0 + (uint32_t)(wn * 32 + l32);
            if (Pm <= Pend) {
                const uint32_t img = fdiv(Pm, P.d_howo);
                const uint32_t pin = Pm - img * P.howo;
                const int jl = (int)blockIdx.y * (WM * 32) + wm * 32 + 4 * h;
                float *o = P.out + ((size_t)img * P.Co + jl) * P.howo + pin;
                const int room = P.Co - jl;   // channels jl .. Co-1 exist
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    if (KS == 2 && ((v >> 3) != ks)) continue;   // the partner stores that half
                    const int dj = 8 * (v >> 2) + (v & 3);
                    if (dj < room) o[(size_t)dj * P.howo] = acc[v];
                }
            }
        }

        if (has_next) lds_store(st ^ 1);
        __syncthreads();
    }
}

template <int HF, int WF, int CI, int WM, int KS, int JX>
static hipError_t launch_shallow_t(const ShallowParams &P, int mgroups, hipStream_t st)
{
    constexpr int NT = 64 * WM * 2 * KS;
    constexpr int SS = JX * NT;
    constexpr int STAGE = CI * SS + 4;
    constexpr size_t lds = 4u * (size_t)(2 * STAGE + (KS == 2 ? WM * 2 * 2 * 8 * 64 : 0));
    auto kern = &conv_mfma_shallow_kernel<HF, WF, CI, WM, KS, JX>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    // Persistent grid: enough workgroups to give every CU its share of resident waves.
    int per_cu = 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, NT, lds);
    if (e != hipSuccess) return e;
    if (per_cu < 1) return hipErrorInvalidConfiguration;
    if (per_cu > 3) per_cu = 3;
    int dev = 0, ncu = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
    uint32_t gx = (uint32_t)(ncu * per_cu) / (uint32_t)mgroups;
    if (gx < 1) gx = 1;
    if (gx > P.ntiles) gx = P.ntiles;
    hipLaunchKernelGGL(kern, dim3(gx, mgroups), dim3(NT), lds, st, P);
    return hipGetLastError();
}

// Returns hipErrorNotSupported when the layer does not meet this kernel's conditions.
hipError_t launch_conv_mfma_shallow(const float *win, const float *flt, float *out, const Shape &sh,
                                    hipStream_t st)
{
    // strip floats per channel for a 64-pixel tile, and the rows it may touch
    int rmax = (NB + sh.Wo - 2) / sh.Wo + 1;
    if (rmax > NB) rmax = NB;
    if (rmax > SH_RMAX) return hipErrorNotSupported;
    const int over = sh.Wf > sh.s ? sh.Wf - sh.s : 0;
    const int S = (NB * sh.s + rmax * over) * sh.Hf + 1;
    // 32-bit strip offsets: the rows of one tile must lie within 2 GiB of each other
    const long long span = (long long)sh.Ci * sh.Ho * sh.rowlen * 4LL * (rmax + 1);
    if (span >= (1LL << 31)) return hipErrorNotSupported;

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
    P.d_wo = make_fastdiv((uint32_t)sh.Wo);
    P.d_ho = make_fastdiv((uint32_t)sh.Ho);
    P.d_howo = make_fastdiv(P.howo);

    if (sh.Ci != 3) return hipErrorNotSupported;
    const int wm = sh.Co <= 32 ? 1 : (sh.Co <= 64 ? 2 : 3);
    const int mgroups = (sh.Co + wm * 32 - 1) / (wm * 32);
    if (sh.Hf == 7 && sh.Wf == 7) {
        if (wm == 1 && S <= 4 * 128) return launch_shallow_t<7, 7, 3, 1, 1, 4>(P, mgroups, st);
        if (wm == 1 && S <= 8 * 128) return launch_shallow_t<7, 7, 3, 1, 1, 8>(P, mgroups, st);
        if (wm == 2 && S <= 4 * 256) return launch_shallow_t<7, 7, 3, 2, 1, 4>(P, mgroups, st);
        if (wm == 3 && S <= 3 * 384) return launch_shallow_t<7, 7, 3, 3, 1, 3>(P, mgroups, st);
    } else if (sh.Hf == 11 && sh.Wf == 11) {
        if (wm == 1 && S <= 12 * 256) return launch_shallow_t<11, 11, 3, 1, 2, 12>(P, mgroups, st);
        if (wm == 2 && S <= 6 * 512) return launch_shallow_t<11, 11, 3, 2, 2, 6>(P, mgroups, st);
        if (wm == 3 && S <= 4 * 768) return launch_shallow_t<11, 11, 3, 3, 2, 4>(P, mgroups, st);
    } else if (sh.Hf == 3 && sh.Wf == 3) {
        if (wm == 1 && S <= 2 * 128) return launch_shallow_t<3, 3, 3, 1, 1, 2>(P, mgroups, st);
        if (wm == 2 && S <= 1 * 256) return launch_shallow_t<3, 3, 3, 2, 1, 1>(P, mgroups, st);
        if (wm == 3 && S <= 1 * 384) return launch_shallow_t<3, 3, 3, 3, 1, 1>(P, mgroups, st);
    }
    return hipErrorNotSupported;
}

}  // namespace im2win
