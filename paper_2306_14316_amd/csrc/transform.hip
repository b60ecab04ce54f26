// im2win data transformation (Section 3.1, Eq. 2) for gfx950:
//   What(i, r, m, k*Hf + u) = Ipad(i, r, m*s + u, k),  0<=k<Wp, 0<=u<Hf.
// A pure copy, bound by HBM traffic: the input is read (each row about Hf/s
// times, re-reads served by the caches) and the tensor is written once.
// Values move as 32-bit words, so bit patterns survive; padding is +0.0.
// Two kernels: a plain gather (one thread per 16 bytes of the tensor) and the
// assembling kernel that builds a workgroup's stretch of the tensor in LDS.
#include "common.h"
#include "runtime_cache.h"

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
// Assembling kernel: a workgroup builds its contiguous stretch of the tensor in LDS in final
// order and then copies it out linearly.  The stretch is MR consecutive output rows of one
// (image, channel) plane or, for small planes (MULTI), G whole consecutive planes.  Filling: a
// thread takes 16 bytes (four neighbouring columns) of one input row -- row-contiguous,
// 16-byte global loads, several in flight per thread -- and writes each of the four words to
// every place Eq. 2 gives it: input row h is row u = h + p - m*s of the windows of every
// output row m with 0 <= u < Hf, so word (h, k) lands at m*rowlen + k*Hf + u for up to
// ceil(Hf/s) rows m, LDS addresses that differ by the constant rowlen - s.  Draining: 16-byte
// LDS reads and 16-byte global stores with no index arithmetic at all; the LDS image is
// shifted by the stretch's alignment in the tensor so that chunks are 16-byte aligned on both
// sides.  All index arithmetic sits on the load side, a few instructions per 16 bytes loaded,
// each of which feeds up to 4*ceil(Hf/s) words of the tensor: a version that staged the input
// rows in LDS untransposed and decoded (row, column, window row) for every 16 bytes it stored
// was bound by the vector ALU, not by memory.
//
// HF, S: filter height and stride as compile-time constants (LDS offsets become immediates,
// divisions become shifts), or 0, 0 for the instance that reads them from the parameters.
// Threads form a TX x TY grid (TX a power of two >= the 16-byte pieces per input row): no
// division maps a thread to its row and columns.  The last piece of a row is moved left to end
// at the row's last word, so every piece is whole (the overlap rewrites equal values).
struct AssembleParams {
    const uint32_t *in;
    uint32_t *win;
    int Hi, Wi, Ho, Hf, s, p;
    int MR;               // output rows per workgroup (MULTI: Ho)
    int RB;               // workgroups per plane (MULTI: 1)
    int G;                // planes per workgroup (1 unless MULTI)
    int CPR;              // 16-byte pieces per input row = ceil(Wi / 4)
    int txl;              // log2(TX)
    uint32_t rowlen;      // Wp*Hf
    uint32_t plane_in;    // Hi*Wi
    uint32_t plane_out;   // Ho*rowlen
    uint32_t nplanes;     // N*Ci
    size_t in_elems;
    FastDiv d_rb, d_nrows, d_s, d_padrow, d_padplane;
};

typedef uint32_t uint32x4 __attribute__((ext_vector_type(4)));

template <int HF, int S, bool MULTI>
__global__ __launch_bounds__(256) void transform_assemble_kernel(AssembleParams P)
{
    extern __shared__ __align__(16) unsigned char smem_a[];
    uint32_t *buf = reinterpret_cast<uint32_t *>(smem_a);
    constexpr int FILL_U = 4;                       // independent 16-byte loads in flight per thread
    const int Hf = HF ? HF : P.Hf, s = S ? S : P.s;
    auto div_s = [&](uint32_t x) __attribute__((always_inline)) -> uint32_t {
        if (S == 1) return x;
        if (S == 2) return x >> 1;
        if (S == 4) return x >> 2;
        return fdiv(x, P.d_s);
    };

    const uint32_t lb = xcd_swizzle64(blockIdx.x, gridDim.x);   // neighbouring row blocks share input rows: same XCD
    const uint32_t pg = MULTI ? lb : fdiv(lb, P.d_rb);
    const uint32_t plane0 = MULTI ? pg * (uint32_t)P.G : pg;
    const int ng = MULTI ? (int)min((uint32_t)P.G, P.nplanes - plane0) : 1;
    const int m0 = MULTI ? 0 : (int)(lb - pg * (uint32_t)P.RB) * P.MR;
    const int mr = MULTI ? P.Ho : min(P.MR, P.Ho - m0);
    const int nrows = (mr - 1) * s + Hf;            // input rows (of the padded image) one plane's rows need
    const int h_lo = m0 * s - P.p;
    const size_t ybeg = ((size_t)plane0 * P.Ho + (size_t)m0) * P.rowlen;
    const uint32_t a = (uint32_t)(ybeg & 3u);       // LDS word i holds tensor word ybeg - a + i
    const uint32_t nout = (uint32_t)(ng - 1) * P.plane_out + (uint32_t)mr * P.rowlen;

    // descriptor on the first plane of the group (a group's planes span < 4 GiB: checked on the host)
    const size_t pbase = (size_t)plane0 * P.plane_in;
    const size_t left = (P.in_elems - pbase) * 4u;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t *>(P.in + pbase), 0, left < 0xffffffffull ? (uint32_t)left : 0xffffffffu, 0x00020000);

    // ---- zero padding: words [0, p*Hf) and [(p + Wi)*Hf, rowlen) of every row ----
    if (P.p > 0) {
        const uint32_t per = (uint32_t)(2 * P.p * Hf), half = (uint32_t)(P.p * Hf);
        const uint32_t per_plane = (uint32_t)mr * per;
        for (uint32_t idx = threadIdx.x; idx < (uint32_t)ng * per_plane; idx += 256) {
            const uint32_t g = MULTI ? fdiv(idx, P.d_padplane) : 0u;
            const uint32_t i2 = idx - g * per_plane;
            const uint32_t ml = fdiv(i2, P.d_padrow);
            const uint32_t c = i2 - ml * per;
            const uint32_t x = c < half ? c : (uint32_t)(P.Wi * Hf) + c;
            buf[a + g * P.plane_out + ml * P.rowlen + x] = 0u;
        }
    }

    // ---- fill ----
    const int tx = (int)threadIdx.x & ((1 << P.txl) - 1), ty = (int)threadIdx.x >> P.txl, TY = 256 >> P.txl;
    const int c4 = min(4 * tx, P.Wi - 4);           // first column of this thread's piece
    const bool col_ok = tx < P.CPR;
    const uint32_t colpos = a + (uint32_t)((P.p + c4) * Hf);
    const uint32_t step = P.rowlen - (uint32_t)s;   // LDS distance between the places of one word in rows m, m+1
    const int total_rows = ng * nrows;
    for (int rr0 = ty; rr0 < total_rows; rr0 += TY * FILL_U) {
        uint32x4 val[FILL_U];
        uint32_t at[FILL_U];
        int nml[FILL_U];
#pragma unroll
        for (int j = 0; j < FILL_U; ++j) {
            const int rr = rr0 + TY * j;
            const uint32_t g = MULTI ? fdiv((uint32_t)rr, P.d_nrows) : 0u;
            const uint32_t r = (uint32_t)rr - g * (uint32_t)nrows;   // row within the plane's strip
            const int hh = h_lo + (int)r;
            const bool live = col_ok & (rr < total_rows);
            const bool inside = live & (hh >= 0) & (hh < P.Hi);
            const uint32_t off = inside ? (g * P.plane_in + (uint32_t)(hh * P.Wi + c4)) * 4u : 0u;
            val[j] = __builtin_bit_cast(uint32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0));
            if (!inside) val[j] = (uint32x4){0u, 0u, 0u, 0u};
            // output rows ml with 0 <= r - ml*s < Hf, within this block
            const int ml_hi = min((int)div_s(r), mr - 1);
            const int ml_lo = (int)r >= Hf ? (int)div_s(r - (uint32_t)Hf) + 1 : 0;
            nml[j] = live ? ml_hi - ml_lo + 1 : 0;
            at[j] = colpos + g * P.plane_out + r + (uint32_t)ml_lo * step;
        }
#pragma unroll
        for (int j = 0; j < FILL_U; ++j) {
            uint32_t q = at[j];
            if (HF) {
                constexpr int JMAX = HF ? (HF + (S ? S : 1) - 1) / (S ? S : 1) : 1;
#pragma unroll
                for (int t = 0; t < JMAX; ++t) {
                    if (t < nml[j]) {
                        buf[q] = val[j].x;
                        buf[q + HF] = val[j].y;
                        buf[q + 2 * HF] = val[j].z;
                        buf[q + 3 * HF] = val[j].w;
                    }
                    q += step;
                }
            } else {
                for (int t = 0; t < nml[j]; ++t) {
                    buf[q] = val[j].x;
                    buf[q + (uint32_t)Hf] = val[j].y;
                    buf[q + 2u * (uint32_t)Hf] = val[j].z;
                    buf[q + 3u * (uint32_t)Hf] = val[j].w;
                    q += step;
                }
            }
        }
    }
    __syncthreads();

    // ---- drain: LDS words [a, a + nout) -> tensor words [ybeg, ybeg + nout) ----
    uint32_t *dst = P.win + (ybeg - a);
    const uint32_t end = a + nout;
    const uint32_t first_full = a ? 1u : 0u, nchunk_all = (end + 3u) >> 2;
    const uint32_t last_full = (end & 3u) ? nchunk_all - 1 : nchunk_all;   // chunks [first_full, last_full) are whole
    for (uint32_t c = first_full + threadIdx.x; c < last_full; c += 256)
        *reinterpret_cast<uint32x4 *>(dst + 4u * c) = *reinterpret_cast<const uint32x4 *>(buf + 4u * c);
    if (threadIdx.x < 4) {
        const uint32_t i0 = threadIdx.x;                    // word i0 of the head chunk
        if (a && i0 >= a && i0 < end) dst[i0] = buf[i0];
        const uint32_t i1 = 4u * last_full + threadIdx.x;   // ... of the tail chunk
        if (last_full < nchunk_all && last_full >= first_full && i1 < end) dst[i1] = buf[i1];
    }
}

template <int HF, int S>
static hipError_t launch_assemble_t(const AssembleParams &Q, bool multi, uint32_t blocks, size_t lds, hipStream_t st,
                                    LaunchPlan *plan)
{
    if (plan) {
        plan_record(plan, dim3(blocks), 256, lds, "transform_assemble_kernel<%d, %d, %s>", HF, S, tf(multi));
        return hipSuccess;
    }
    static KernelCache kc[2];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (multi) {
        if ((e = allow_dynamic_lds(kc[1], reinterpret_cast<const void *>(&transform_assemble_kernel<HF, S, true>), lds, dev)) != hipSuccess) return e;
        hipLaunchKernelGGL((transform_assemble_kernel<HF, S, true>), dim3(blocks), dim3(256), lds, st, Q);
    } else {
        if ((e = allow_dynamic_lds(kc[0], reinterpret_cast<const void *>(&transform_assemble_kernel<HF, S, false>), lds, dev)) != hipSuccess) return e;
        hipLaunchKernelGGL((transform_assemble_kernel<HF, S, false>), dim3(blocks), dim3(256), lds, st, Q);
    }
    return hipGetLastError();
}

// The assembling kernel.  hipErrorNotSupported when the layer is outside its reach: rows shorter
// than one 16-byte piece or longer than 256 of them, an im2win row too long for LDS, planes too
// large for 32-bit byte offsets, an unaligned tensor.
static hipError_t launch_transform_assemble(const float *in, float *win, const Shape &sh, hipStream_t st,
                                            LaunchPlan *plan, size_t budget = 24 * 1024)
{
    if ((reinterpret_cast<uintptr_t>(win) & 15u) != 0 || (reinterpret_cast<uintptr_t>(in) & 3u) != 0) return hipErrorNotSupported;
    const int CPR = (sh.Wi + 3) / 4;
    if (sh.Wi < 4 || CPR > 256) return hipErrorNotSupported;
    const unsigned long long row_bytes = (unsigned long long)sh.rowlen * 4ull;
    const unsigned long long plane_out_bytes = row_bytes * (unsigned long long)sh.Ho;
    const unsigned long long plane_in_bytes = (unsigned long long)sh.Hi * sh.Wi * 4ull;
    if (row_bytes + 32 > 64 * 1024 || plane_in_bytes >= (1ull << 32) - 16) return hipErrorNotSupported;
    const unsigned long long nplanes = (unsigned long long)sh.N * sh.Ci;

    AssembleParams Q;
    Q.in = reinterpret_cast<const uint32_t *>(in);
    Q.win = reinterpret_cast<uint32_t *>(win);
    Q.Hi = sh.Hi; Q.Wi = sh.Wi; Q.Ho = sh.Ho; Q.Hf = sh.Hf; Q.s = sh.s; Q.p = sh.p;
    Q.CPR = CPR;
    Q.txl = 0;
    while ((1 << Q.txl) < CPR) ++Q.txl;
    Q.rowlen = (uint32_t)sh.rowlen;
    Q.plane_in = (uint32_t)(sh.Hi * sh.Wi);
    Q.nplanes = (uint32_t)nplanes;
    Q.in_elems = (size_t)nplanes * Q.plane_in;
    bool multi = false;
    unsigned long long blocks, lds_words;
    if (2 * plane_out_bytes <= budget && plane_out_bytes < (1ull << 31)) {
        // small planes: G whole planes per workgroup
        unsigned long long G = budget / plane_out_bytes;
        if (G > nplanes) G = nplanes;
        if (G * plane_in_bytes >= (1ull << 32) - 16) return hipErrorNotSupported;
        multi = true;
        Q.G = (int)G; Q.MR = sh.Ho; Q.RB = 1;
        blocks = (nplanes + G - 1) / G;
        lds_words = G * ((unsigned long long)sh.Ho * sh.rowlen) + 8;
    } else {
        int mrmax = (int)(budget / row_bytes);
        if (mrmax < 1) mrmax = 1;
        if (mrmax > sh.Ho) mrmax = sh.Ho;
        const int nb = (sh.Ho + mrmax - 1) / mrmax;   // row blocks per plane, of equal height
        Q.G = 1; Q.MR = (sh.Ho + nb - 1) / nb; Q.RB = (sh.Ho + Q.MR - 1) / Q.MR;
        blocks = nplanes * (unsigned long long)Q.RB;
        lds_words = (unsigned long long)Q.MR * sh.rowlen + 8;
    }
    if (blocks >= (1ull << 31) || (unsigned long long)sh.Ho * sh.rowlen >= (1ull << 32)) return hipErrorNotSupported;
    Q.plane_out = (uint32_t)((unsigned long long)sh.Ho * sh.rowlen);
    const int nrows = (Q.MR - 1) * sh.s + sh.Hf;   // (MR <= Ho: at most Hp rows)
    Q.d_rb = make_fastdiv((uint32_t)Q.RB);
    Q.d_nrows = make_fastdiv((uint32_t)nrows);
    Q.d_s = make_fastdiv((uint32_t)sh.s);
    const uint32_t padrow = sh.p > 0 ? (uint32_t)(2 * sh.p * sh.Hf) : 1u;
    Q.d_padrow = make_fastdiv(padrow);
    Q.d_padplane = make_fastdiv(padrow * (uint32_t)Q.MR);
    const size_t lds = (size_t)lds_words * 4u;
    const uint32_t nb32 = (uint32_t)blocks;
    if (sh.Hf == 3 && sh.s == 1) return launch_assemble_t<3, 1>(Q, multi, nb32, lds, st, plan);
    if (sh.Hf == 5 && sh.s == 1) return launch_assemble_t<5, 1>(Q, multi, nb32, lds, st, plan);
    if (sh.Hf == 7 && sh.s == 2) return launch_assemble_t<7, 2>(Q, multi, nb32, lds, st, plan);
    if (sh.Hf == 11 && sh.s == 4) return launch_assemble_t<11, 4>(Q, multi, nb32, lds, st, plan);
    return launch_assemble_t<0, 0>(Q, multi, nb32, lds, st, plan);
}

hipError_t launch_transform(const float *in, float *win, const Shape &sh, hipStream_t st, LaunchPlan *plan)
{
    // The assembling kernel takes every layer it can (measured on the five benchmark layers and
    // the twelve of Table 2: 5.6-6.6 TB/s of tensor bytes, against 4.1-5.9 TB/s for the gather
    // below); the gather is the fallback for rows shorter than four words or longer than 1024,
    // im2win rows too long for LDS and tensors that are not 16-byte aligned.
    const hipError_t ae = launch_transform_assemble(in, win, sh, st, plan);
    if (ae != hipErrorNotSupported) return ae;

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
