// Comparison baselines for gfx950, kept beside the im2win path so that both
// can be timed on the same inputs:
//   - the direct convolution (Section 2.2): one thread per output element,
//     seven-loop arithmetic straight from the NCHW input;
//   - the GEMM-based convolution (Section 2.3): an explicit im2col matrix per
//     image, then one GEMM with the filter matrix on the fp32 matrix cores.
// Neither is part of the im2win hot path.
#include "conv_mfma_tile.h"

namespace im2win {

// ---------------------------------------------------------------------------
// Direct convolution, Eq. 1 evaluated per output element.
// ---------------------------------------------------------------------------
struct DirectParams {
    const float *in;
    const float *flt;
    float *out;
    int Ci, Hi, Wi, Ho, Wo, Co, Hf, Wf, s, p;
    uint32_t total;   // N*Co*Ho*Wo
    FastDiv d_wo, d_ho, d_co;
};

__global__ __launch_bounds__(256) void conv_direct_kernel(DirectParams P)
{
    const uint32_t o = blockIdx.x * 256u + threadIdx.x;   // flat NCHW output index
    if (o >= P.total) return;
    const uint32_t t = fdiv(o, P.d_wo);
    const int n = (int)(o - t * (uint32_t)P.Wo);
    const uint32_t t2 = fdiv(t, P.d_ho);
    const int m = (int)(t - t2 * (uint32_t)P.Ho);
    const uint32_t i = fdiv(t2, P.d_co);
    const uint32_t j = t2 - i * (uint32_t)P.Co;

    const float *img = P.in + (size_t)i * P.Ci * P.Hi * P.Wi;
    const float *f = P.flt + (size_t)j * P.Ci * P.Hf * P.Wf;
    float acc = 0.0f;
    for (int r = 0; r < P.Ci; ++r)
        for (int u = 0; u < P.Hf; ++u) {
            const int h = m * P.s + u - P.p;
            if (h < 0 || h >= P.Hi) continue;
            for (int v = 0; v < P.Wf; ++v) {
                const int w = n * P.s + v - P.p;
                if (w < 0 || w >= P.Wi) continue;
                acc = fmaf(img[((size_t)r * P.Hi + h) * P.Wi + w], f[(r * P.Hf + u) * P.Wf + v], acc);
            }
        }
    P.out[o] = acc;
}

hipError_t launch_conv_direct(const float *in, const float *flt, float *out, const Shape &sh,
                              hipStream_t st, LaunchPlan *plan)
{
    DirectParams P;
    P.in = in; P.flt = flt; P.out = out;
    P.Ci = sh.Ci; P.Hi = sh.Hi; P.Wi = sh.Wi; P.Ho = sh.Ho; P.Wo = sh.Wo; P.Co = sh.Co;
    P.Hf = sh.Hf; P.Wf = sh.Wf; P.s = sh.s; P.p = sh.p;
    P.total = (uint32_t)((size_t)sh.npix * sh.Co);
    P.d_wo = make_fastdiv((uint32_t)sh.Wo);
    P.d_ho = make_fastdiv((uint32_t)sh.Ho);
    P.d_co = make_fastdiv((uint32_t)sh.Co);
    if (plan) { plan_record(plan, dim3((P.total + 255u) / 256u), 256, 0, "conv_direct_kernel"); return hipSuccess; }
    hipLaunchKernelGGL(conv_direct_kernel, dim3((P.total + 255u) / 256u), dim3(256), 0, st, P);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// im2col (Section 2.3): col[gp][(r*Hf + u)*Wf + v] = Ipad(i, r, m*s + u, n*s + v)
// for pixel gp = (i*Ho + m)*Wo + n; rows of K = Ci*Hf*Wf floats, dense.
// One thread writes one group of four consecutive K entries of one row.
// ---------------------------------------------------------------------------
struct Im2colParams {
    const uint32_t *in;
    uint32_t *col;
    int Ci, Hi, Wi, Ho, Wo, Hf, Wf, s, p, K;
    uint32_t groups_per_row;   // ceil(K/4)
    uint32_t total_groups;     // npix * groups_per_row
    uint32_t howo;
    int vec4;                  // K % 4 == 0 and col 16-byte aligned
    FastDiv d_gpr, d_howo, d_wo, d_khw, d_wf;
};

__global__ __launch_bounds__(256) void im2col_kernel(Im2colParams P)
{
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;
    if (t >= P.total_groups) return;
    const uint32_t gp = fdiv(t, P.d_gpr);
    const int k0 = (int)(t - gp * P.groups_per_row) * 4;
    const uint32_t i = fdiv(gp, P.d_howo);
    const uint32_t pin = gp - i * P.howo;
    const int m = (int)fdiv(pin, P.d_wo);
    const int n = (int)(pin - (uint32_t)m * (uint32_t)P.Wo);
    int r = (int)fdiv((uint32_t)k0, P.d_khw);
    const uint32_t rem = (uint32_t)k0 - (uint32_t)r * (uint32_t)(P.Hf * P.Wf);
    int u = (int)fdiv(rem, P.d_wf);
    int v = (int)(rem - (uint32_t)u * (uint32_t)P.Wf);

    const uint32_t *img = P.in + (size_t)i * P.Ci * P.Hi * P.Wi;
    uint32_t val[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int h = m * P.s + u - P.p, w = n * P.s + v - P.p;
        const bool inside = (k0 + e < P.K) & (h >= 0) & (h < P.Hi) & (w >= 0) & (w < P.Wi);
        val[e] = inside ? img[((size_t)r * P.Hi + h) * P.Wi + w] : 0u;
        if (++v == P.Wf) {
            v = 0;
            if (++u == P.Hf) { u = 0; ++r; }
        }
    }
    uint32_t *dst = P.col + (size_t)gp * P.K + k0;
    if (P.vec4) {
        *reinterpret_cast<uint4 *>(dst) = make_uint4(val[0], val[1], val[2], val[3]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (k0 + e < P.K) dst[e] = val[e];
    }
}

hipError_t launch_im2col(const float *in, float *col, const Shape &sh, hipStream_t st)
{
    Im2colParams P;
    P.in = reinterpret_cast<const uint32_t *>(in);
    P.col = reinterpret_cast<uint32_t *>(col);
    P.Ci = sh.Ci; P.Hi = sh.Hi; P.Wi = sh.Wi; P.Ho = sh.Ho; P.Wo = sh.Wo; P.Hf = sh.Hf; P.Wf = sh.Wf;
    P.s = sh.s; P.p = sh.p; P.K = sh.K;
    P.groups_per_row = (uint32_t)((sh.K + 3) / 4);
    const unsigned long long groups = (unsigned long long)sh.npix * P.groups_per_row;
    if (groups >= (1ull << 31)) return hipErrorInvalidValue;
    P.total_groups = (uint32_t)groups;
    P.howo = (uint32_t)(sh.Ho * sh.Wo);
    P.vec4 = (sh.K % 4 == 0) && (reinterpret_cast<uintptr_t>(col) & 15u) == 0;
    P.d_gpr = make_fastdiv(P.groups_per_row);
    P.d_howo = make_fastdiv(P.howo);
    P.d_wo = make_fastdiv((uint32_t)sh.Wo);
    P.d_khw = make_fastdiv((uint32_t)(sh.Hf * sh.Wf));
    P.d_wf = make_fastdiv((uint32_t)sh.Wf);
    hipLaunchKernelGGL(im2col_kernel, dim3((P.total_groups + 255u) / 256u), dim3(256), 0, st, P);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// GEMM over the im2col matrix: O(i, j, pixel) = sum_k F[j][k] * col[gp][k].
// Both operands are K-contiguous.  64x64 output tile per workgroup, four waves
// of 32x32 (v_mfma_f32_32x32x2_f32), K blocks of 32 double-buffered in LDS.
// Tiles are stored [row][k] with a pitch of 36 floats, written and read as
// 16-byte groups: lane (row, h) takes K groups 2t+h, t = 0..3, and feeds entry e
// of its group to MFMA 4t+e.  The K order inside a block is therefore permuted,
// identically for both operands, which a sum does not mind.
// ---------------------------------------------------------------------------
constexpr int GK = 32;       // K block
constexpr int GP = GK + 4;   // LDS row pitch in floats

struct GemmParams {
    const float *flt;   // [Co][K]
    const float *col;   // [npix][K]
    float *out;
    int Co, K;
    uint32_t npix, howo;
    uint32_t tiles_m, nblocks;
    FastDiv d_tm, d_howo;
};

typedef float float4v __attribute__((ext_vector_type(4)));

template <bool VEC>
__device__ __forceinline__ float4v load_group(const float *row, bool row_ok, int k, int K)
{
    float4v g = {0.f, 0.f, 0.f, 0.f};
    if (VEC) {
        if (row_ok && k < K) g = *reinterpret_cast<const float4v *>(row + k);
    } else if (row_ok) {
        if (k + 0 < K) g.x = row[k + 0];
        if (k + 1 < K) g.y = row[k + 1];
        if (k + 2 < K) g.z = row[k + 2];
        if (k + 3 < K) g.w = row[k + 3];
    }
    return g;
}

template <bool VEC>
__global__ __launch_bounds__(256) void gemm_im2col_kernel(GemmParams P)
{
    __shared__ __align__(16) float lds[2][2][64 * GP];   // [stage][operand][row*GP + k]

    const uint32_t b = xcd_swizzle(blockIdx.x, P.nblocks);
    const uint32_t tn = fdiv(b, P.d_tm);
    const int m0 = (int)(b - tn * P.tiles_m) * 64;
    const uint32_t n0 = tn * 64u;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1, h = lane >> 5, l32 = lane & 31;

    // staging: a thread moves K group c of rows srow and srow+32 of both operands
    const int srow = tid >> 3, c4 = (tid & 7) * 4;
    const float *arow[2], *brow[2];
    bool aok[2], bok[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int j = m0 + srow + 32 * q;
        const uint32_t gp = n0 + (uint32_t)(srow + 32 * q);
        aok[q] = j < P.Co;
        bok[q] = gp < P.npix;
        arow[q] = P.flt + (size_t)(aok[q] ? j : 0) * P.K;
        brow[q] = P.col + (size_t)(bok[q] ? gp : 0) * P.K;
    }

    floatx16 acc = {0};
    float4v ga[2], gb[2];
    auto fetch = [&](int kb) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            ga[q] = load_group<VEC>(arow[q], aok[q], kb * GK + c4, P.K);
            gb[q] = load_group<VEC>(brow[q], bok[q], kb * GK + c4, P.K);
        }
    };
    auto stash = [&](int stage) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            *reinterpret_cast<float4v *>(&lds[stage][0][(srow + 32 * q) * GP + c4]) = ga[q];
            *reinterpret_cast<float4v *>(&lds[stage][1][(srow + 32 * q) * GP + c4]) = gb[q];
        }
    };

    const int nkb = (P.K + GK - 1) / GK;
    fetch(0);
    stash(0);
    __syncthreads();
    for (int kb = 0; kb < nkb; ++kb) {
        const int stage = kb & 1;
        if (kb + 1 < nkb) fetch(kb + 1);
        const float *A = &lds[stage][0][(wm * 32 + l32) * GP + 4 * h];
        const float *B = &lds[stage][1][(wn * 32 + l32) * GP + 4 * h];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float4v a = *reinterpret_cast<const float4v *>(A + 8 * t);
            const float4v bq = *reinterpret_cast<const float4v *>(B + 8 * t);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, bq.x, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, bq.y, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, bq.z, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, bq.w, acc, 0, 0, 0);
        }
        if (kb + 1 < nkb) stash(stage ^ 1);
        __syncthreads();
    }

    // epilogue: register v of lane (h, l32) is output channel 8*(v/4) + 4*h + v%4, pixel l32
    const uint32_t gp = n0 + (uint32_t)(wn * 32 + l32);
    if (gp < P.npix) {
        const uint32_t img = fdiv(gp, P.d_howo);
        const uint32_t pin = gp - img * P.howo;
        float *o = P.out + (size_t)img * P.Co * P.howo + pin;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int j = m0 + wm * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
            if (j < P.Co) o[(size_t)j * P.howo] = acc[v];
        }
    }
}

hipError_t launch_gemm_im2col(const float *col, const float *flt, float *out, const Shape &sh,
                              hipStream_t st)
{
    GemmParams P;
    P.flt = flt; P.col = col; P.out = out;
    P.Co = sh.Co; P.K = sh.K;
    P.npix = (uint32_t)sh.npix;
    P.howo = (uint32_t)(sh.Ho * sh.Wo);
    P.tiles_m = (uint32_t)((sh.Co + 63) / 64);
    const unsigned long long nb = (unsigned long long)P.tiles_m * ((P.npix + 63u) / 64u);
    if (nb >= (1ull << 31)) return hipErrorInvalidValue;
    P.nblocks = (uint32_t)nb;
    P.d_tm = make_fastdiv(P.tiles_m);
    P.d_howo = make_fastdiv(P.howo);
    const bool vec = (sh.K % 4 == 0) && ((reinterpret_cast<uintptr_t>(col) | reinterpret_cast<uintptr_t>(flt)) & 15u) == 0;
    if (vec)
        hipLaunchKernelGGL(gemm_im2col_kernel<true>, dim3(P.nblocks), dim3(256), 0, st, P);
    else
        hipLaunchKernelGGL(gemm_im2col_kernel<false>, dim3(P.nblocks), dim3(256), 0, st, P);
    return hipGetLastError();
}

}  // namespace im2win
