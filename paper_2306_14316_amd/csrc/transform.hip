// im2win data transformation (Section 3.1, Eq. 2) for gfx950:
//   What(i, r, m, k*Hf + u) = Ipad(i, r, m*s + u, k),  0<=k<Wp, 0<=u<Hf.
// A pure gather-copy, bound by HBM traffic: the input is read (each row about
// Hf/s times, re-reads served by the caches) and the tensor is written once.
// Values move as 32-bit words, so bit patterns survive; padding is +0.0.
#include "common.h"

namespace im2win {

struct TransformParams {
    const uint32_t *in;
    uint32_t *win;
    int Ci, Hi, Wi, Ho, Hf, s, p, Wp;
    uint32_t rowlen;      // Wp*Hf
    uint32_t total;       // N*Ci*Ho*rowlen
    uint32_t plane_in;    // Hi*Wi
    FastDiv d_rowlen, d_ho, d_hf;
};

// One thread writes VEC consecutive words of the tensor (one 16-byte store
// when VEC == 4).  The first word's coordinates come from three reciprocal
// divisions; the following ones are stepped with carries (u fastest, then the
// column k, then the row m, then the plane).
template <int VEC>
__global__ __launch_bounds__(256) void transform_kernel(TransformParams P)
{
    // consecutive blocks read overlapping input rows: keep them on one XCD (one L2)
    uint32_t y0 = (xcd_swizzle64(blockIdx.x, gridDim.x) * 256u + threadIdx.x) * VEC;
    if (y0 >= P.total) return;

    uint32_t row = fdiv(y0, P.d_rowlen);          // (i*Ci + r)*Ho + m
    uint32_t x = y0 - row * P.rowlen;             // k*Hf + u
    uint32_t plane = fdiv(row, P.d_ho);           // i*Ci + r
    int m = (int)(row - plane * (uint32_t)P.Ho);
    int k = (int)fdiv(x, P.d_hf);
    int u = (int)(x - (uint32_t)k * (uint32_t)P.Hf);
    const uint32_t *src = P.in + (size_t)plane * P.plane_in;

    uint32_t v[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        int h = m * P.s + u - P.p;
        int w = k - P.p;
        bool inside = (h >= 0) & (h < P.Hi) & (w >= 0) & (w < P.Wi) & (y0 + e < P.total);
        v[e] = inside ? src[h * P.Wi + w] : 0u;
        // step to the next word of the tensor
        if (++u == P.Hf) {
            u = 0;
            if (++k == P.Wp) {
                k = 0;
                if (++m == P.Ho) {
                    m = 0;
                    src += P.plane_in;
                }
            }
        }
    }

    if (VEC == 4) {
        if (y0 + 4 <= P.total) {
            *reinterpret_cast<uint4 *>(P.win + y0) = make_uint4(v[0], v[1], v[2], v[3]);
        } else {
            for (int e = 0; e < VEC; ++e)
                if (y0 + e < P.total) P.win[y0 + e] = v[e];
        }
    } else {
        P.win[y0] = v[0];
    }
}

// ---------------------------------------------------------------------------
// LDS-staged variant for tall windows.  With Hf rows per window, consecutive
// words of the tensor come from Hf different input rows, and the plain gather
// above touches many partly used cache lines per load.  Here a workgroup owns
// MR consecutive output rows of one (image, channel) plane: it reads the
// (MR-1)*s + Hf input rows they need into LDS with row-contiguous loads (the
// zero padding is materialised there), then writes its contiguous stretch of
// the tensor with 16-byte stores, reading LDS transposed (k*Hf + u  <-  row
// m*s + u, column k).  The host picks the LDS row pitch that spreads those
// transposed reads best over the banks.
struct TransformLdsParams {
    const uint32_t *in;
    uint32_t *win;
    int Hi, Wi, Ho, Hf, s, p, Wp;
    int MR;               // output rows per workgroup
    int RB;               // workgroups per plane = ceil(Ho / MR)
    int LW;               // LDS row pitch (>= Wp, chosen against bank conflicts)
    uint32_t rowlen;      // Wp*Hf
    uint32_t plane_in;    // Hi*Wi
    FastDiv d_rb, d_wp, d_rowlen, d_hf;
};

__global__ __launch_bounds__(256) void transform_lds_kernel(TransformLdsParams P)
{
    extern __shared__ __align__(16) unsigned char smem_t[];
    uint32_t *strip = reinterpret_cast<uint32_t *>(smem_t);   // [nrows][LW]

    const uint32_t lb = xcd_swizzle64(blockIdx.x, gridDim.x);   // neighbours in a plane share input rows: same XCD
    const uint32_t plane = fdiv(lb, P.d_rb);
    const int m0 = (int)(lb - plane * (uint32_t)P.RB) * P.MR;
    const int mr = min(P.MR, P.Ho - m0);
    const int nrows = (mr - 1) * P.s + P.Hf;
    const int h_lo = m0 * P.s - P.p;
    const uint32_t *src = P.in + (size_t)plane * P.plane_in;

    // ---- fill: padded input rows h_lo .. h_lo+nrows-1, columns 0..Wp-1 ----
    // Batches of FILL_U independent loads per thread, all issued before the first LDS store.
    constexpr int FILL_U = 8;
    const uint32_t nfill = (uint32_t)(nrows * P.Wp);
    for (uint32_t base = threadIdx.x; base < nfill; base += 256u * FILL_U) {
        uint32_t val[FILL_U], at[FILL_U];
#pragma unroll
        for (int j = 0; j < FILL_U; ++j) {
            const uint32_t idx = base + 256u * j;
            const uint32_t r = fdiv(idx, P.d_wp);
            const int k = (int)(idx - r * (uint32_t)P.Wp);
            const int hh = h_lo + (int)r, ww = k - P.p;
            const bool inside = (idx < nfill) & (hh >= 0) & (hh < P.Hi) & (ww >= 0) & (ww < P.Wi);
            val[j] = inside ? src[hh * P.Wi + ww] : 0u;
            at[j] = idx < nfill ? r * (uint32_t)P.LW + (uint32_t)k : ~0u;
        }
#pragma unroll
        for (int j = 0; j < FILL_U; ++j)
            if (at[j] != ~0u) strip[at[j]] = val[j];
    }
    __syncthreads();

    // ---- drain: tensor words [ybeg, yend) in 16-byte chunks aligned on the whole tensor ----
    const size_t ybeg = ((size_t)plane * P.Ho + (size_t)m0) * P.rowlen;
    const uint32_t nout = (uint32_t)mr * P.rowlen;
    const uint32_t head = (uint32_t)((4u - (uint32_t)(ybeg & 3u)) & 3u);   // words before the first aligned chunk
    uint32_t *dst = P.win + ybeg;
    auto word = [&](uint32_t y) -> uint32_t {   // tensor word ybeg + y
        const uint32_t ml = fdiv(y, P.d_rowlen);
        const uint32_t x = y - ml * P.rowlen;
        const uint32_t k = fdiv(x, P.d_hf);
        const uint32_t u = x - k * (uint32_t)P.Hf;
        return strip[(ml * (uint32_t)P.s + u) * (uint32_t)P.LW + k];
    };
    if (threadIdx.x < head && threadIdx.x < nout) dst[threadIdx.x] = word(threadIdx.x);
    const uint32_t nchunk = nout > head ? (nout - head) >> 2 : 0;
    for (uint32_t c = threadIdx.x; c < nchunk; c += 256) {
        const uint32_t y = head + 4u * c;
        uint32_t ml = fdiv(y, P.d_rowlen);
        uint32_t x = y - ml * P.rowlen;
        uint32_t k = fdiv(x, P.d_hf);
        uint32_t u = x - k * (uint32_t)P.Hf;
        uint32_t rowbase = ml * (uint32_t)P.s * (uint32_t)P.LW;
        uint32_t v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[e] = strip[rowbase + u * (uint32_t)P.LW + k];
            if (++u == (uint32_t)P.Hf) {
                u = 0;
                if (++k == (uint32_t)P.Wp) { k = 0; rowbase += (uint32_t)P.s * (uint32_t)P.LW; }
            }
        }
        *reinterpret_cast<uint4 *>(dst + y) = make_uint4(v[0], v[1], v[2], v[3]);
    }
    const uint32_t tail0 = head + 4u * nchunk;
    if (nout > head && threadIdx.x < nout - tail0) dst[tail0 + threadIdx.x] = word(tail0 + threadIdx.x);
}

// LDS row pitch for the drain's transposed reads: among the eight pitches from
// Wp up, the one with the fewest bank conflicts (32 banks of 4 bytes) over the
// first 32 lanes' four reads (lane L reads words 4L .. 4L+3 of the tensor row).
static int lds_pitch(int Wp, int Hf)
{
    int best = Wp, best_cost = 1 << 30;
    for (int lw = Wp; lw < Wp + 8; ++lw) {
        int cost = 0;
        for (int e = 0; e < 4; ++e) {
            int cnt[32] = {0}, worst = 0;
            for (int L = 0; L < 32; ++L) {
                const int x = 4 * L + e, k = (x / Hf) % Wp, u = x % Hf;
                const int b = (u * lw + k) & 31;
                if (++cnt[b] > worst) worst = cnt[b];
            }
            cost += worst;
        }
        if (cost < best_cost) { best_cost = cost; best = lw; }
    }
    return best;
}

// Output rows per workgroup for the LDS variant: as many as keep the strip within budget.
static int lds_rows_per_block(const Shape &sh, int LW, size_t budget_bytes)
{
    auto bytes = [&](int mr) {   // (64 bits: the stride has no upper bound)
        return ((unsigned long long)(mr - 1) * (unsigned long long)sh.s + (unsigned long long)sh.Hf) * (unsigned long long)LW * 4ull;
    };
    int mr = 16;
    while (mr > 1 && bytes(mr) > budget_bytes) mr >>= 1;
    if (bytes(mr) > budget_bytes) return 0;
    return mr;
}

hipError_t launch_transform(const float *in, float *win, const Shape &sh, hipStream_t st, LaunchPlan *plan)
{
    // Which kernel (measured on the layers of Table 2 and on sweeps of 3x3 shapes): tall windows
    // over wide rows take the LDS-staged kernel; so do short windows (3x3) once the tensors are
    // large -- past about the size of the 256 MB memory-side cache the plain gather drops from
    // 5 to 4.2 TB/s while the staged kernel holds 5.2-5.9 TB/s on rows of 48 words and more.
    // On small planes or small tensors the plain gather is as fast or faster.
    const unsigned long long moved =
        4ull * (unsigned long long)sh.N * sh.Ci * ((unsigned long long)sh.Hi * sh.Wi + (unsigned long long)sh.Ho * sh.rowlen);
    const bool tall = sh.Hf >= 5 && sh.Wp >= 64;
    const bool large = sh.Hf >= 3 && sh.Wp >= 48 && moved >= (192ull << 20);
    if ((tall || large) && (reinterpret_cast<uintptr_t>(win) & 15u) == 0) {
        const int LW = lds_pitch(sh.Wp, sh.Hf);
        const int MR = lds_rows_per_block(sh, LW, 32 * 1024);
        const long long blocks = MR ? (long long)sh.N * sh.Ci * ((sh.Ho + MR - 1) / MR) : 0;
        if (MR && blocks < (1LL << 31)) {
            TransformLdsParams Q;
            Q.in = reinterpret_cast<const uint32_t *>(in);
            Q.win = reinterpret_cast<uint32_t *>(win);
            Q.Hi = sh.Hi; Q.Wi = sh.Wi; Q.Ho = sh.Ho; Q.Hf = sh.Hf; Q.s = sh.s; Q.p = sh.p; Q.Wp = sh.Wp;
            Q.MR = MR; Q.RB = (sh.Ho + MR - 1) / MR; Q.LW = LW;
            Q.rowlen = (uint32_t)sh.rowlen;
            Q.plane_in = (uint32_t)(sh.Hi * sh.Wi);
            Q.d_rb = make_fastdiv((uint32_t)Q.RB);
            Q.d_wp = make_fastdiv((uint32_t)sh.Wp);
            Q.d_rowlen = make_fastdiv(Q.rowlen);
            Q.d_hf = make_fastdiv((uint32_t)sh.Hf);
            const size_t lds = (size_t)((MR - 1) * sh.s + sh.Hf) * LW * 4u;
            if (plan) { plan_record(plan, dim3((uint32_t)blocks), 256, lds, "transform_lds_kernel"); return hipSuccess; }
            hipLaunchKernelGGL(transform_lds_kernel, dim3((uint32_t)blocks), dim3(256), lds, st, Q);
            return hipGetLastError();
        }
    }

    TransformParams P;
    P.in = reinterpret_cast<const uint32_t *>(in);
    P.win = reinterpret_cast<uint32_t *>(win);
    P.Ci = sh.Ci; P.Hi = sh.Hi; P.Wi = sh.Wi; P.Ho = sh.Ho; P.Hf = sh.Hf;
    P.s = sh.s; P.p = sh.p; P.Wp = sh.Wp;
    P.rowlen = (uint32_t)sh.rowlen;
    P.total = (uint32_t)((size_t)sh.N * sh.Ci * sh.Ho * sh.rowlen);
    P.plane_in = (uint32_t)(sh.Hi * sh.Wi);
    P.d_rowlen = make_fastdiv(P.rowlen);
    P.d_ho = make_fastdiv((uint32_t)sh.Ho);
    P.d_hf = make_fastdiv((uint32_t)sh.Hf);

    bool vec4 = (reinterpret_cast<uintptr_t>(win) & 15u) == 0;
    if (vec4) {
        uint32_t chunks = (P.total + 3u) / 4u;
        uint32_t blocks = (chunks + 255u) / 256u;
        if (plan) { plan_record(plan, dim3(blocks), 256, 0, "transform_kernel<4>"); return hipSuccess; }
        hipLaunchKernelGGL(transform_kernel<4>, dim3(blocks), dim3(256), 0, st, P);
    } else {
        uint32_t blocks = (P.total + 255u) / 256u;
        if (plan) { plan_record(plan, dim3(blocks), 256, 0, "transform_kernel<1>"); return hipSuccess; }
        hipLaunchKernelGGL(transform_kernel<1>, dim3(blocks), dim3(256), 0, st, P);
    }
    return hipGetLastError();
}

}  // namespace im2win
