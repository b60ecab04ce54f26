// 1x1 convolution (no padding) on the fp32 matrix cores.  For such a layer with stride 1 the im2win
// tensor of Eq. 2 has the input's own layout -- every window is one element, row m of the tensor is
// row m of the input -- and the convolution is the GEMM O[Co x P] = F[Co x Ci] * I[Ci x P] over the
// P = N*H*W pixels, with I read channel plane by channel plane.  The generic two-stage kernel runs
// these layers at a third of the matrix peak: it copies its operands into LDS one word per lane, and
// the address path of the memory pipeline takes four lanes per cycle whatever their width, so two
// resident workgroups already saturate it.  This kernel moves the same bytes with 16-byte
// direct-to-LDS loads (buffer_load_dwordx4 ... lds, new on gfx950):
//   - tile 64 (or 128) channels x 64 pixels, K blocks of 32 (or 64) input channels (the last one may be
//     shorter), a ring of NST LDS stages; a workgroup runs its tiles as one sequence of blocks, the loads of
//     the next NST - 1 blocks (of the next tile, after a tile's last) in flight while the matrix cores work;
//     one barrier per block.  Two stages are the fastest: a third (loads two blocks ahead) costs a resident
//     workgroup per CU, and four workgroups hide each other's waits better than deeper prefetch does
//     (512 -> 512 channels at 14x14: 117 TFLOP/s with two stages, 112 with three, 97 with four);
//   - B (pixels): [channel][64 pixels], one wave instruction copies four channel rows (4 x 256
//     contiguous bytes of four planes) into 1 KB of LDS; a lane's B read is base + immediate;
//   - A (filter): [row][K1 k], pitch K1 floats, the 16-byte chunks of a row stored at slot
//     (chunk ^ (row & 7)) -- the permutation is applied to the source address of each lane, the
//     LDS side of a load is always the wave's 1 KB in lane order -- so that the 16-byte A reads of
//     eight neighbouring rows fall into eight different bank groups;
//   - K order inside a block: step 4q+i multiplies channel 8q+i on lanes 0-31 with channel 8q+4+i
//     on lanes 32-63, so one 16-byte A read serves four MFMAs of a lane half.
// Conditions (the launcher checks them, other layers keep their kernels): Hf = Wf = 1, pad 0, Ci a
// multiple of eight, Co a multiple of four, a 16-byte aligned filter.  With a stride above 1, planes whose
// pixel count is not a multiple of four or an unaligned source the pixels are copied one word per lane
// instead (GATHER below); the filter side and the MFMA loop are the same.
#include "conv_mfma_tile.h"
#include "runtime_cache.h"

namespace im2win {

typedef __attribute__((address_space(3))) void lds_void_t;
typedef float float4v_t __attribute__((ext_vector_type(4)));

// K1: input channels per K block (64 or 32); MT: blocks of 64 output channels per workgroup tile (1 or 2).
// floats per LDS stage: B [K1][NB], then A [MT * MB][K1]
template <int K1, int MT> constexpr int stage1_floats() { return K1 * NB + MT * MB * K1; }

struct OneByOneParams {
    const float *in;     // [N][Ci][howo]
    const float *flt;    // [Co][Ci]
    MfmaParams T;        // the fields the shared epilogue reads (out, out_elems, Co, howo, d_howo)
    int Ci;
    uint32_t npix, howo, tiles_m, ntiles;
    size_t in_elems, flt_elems;
    FastDiv d_howo, d_tm;
    // source geometry (GATHER instances): floats in a channel plane of `in`, between its rows that hold
    // consecutive output rows, and between the columns of neighbouring output pixels; output row length
    uint32_t plane, rowstep, colstep, Wo;
    FastDiv d_wo;
};

// LDS stages of the K blocks of 32 and largest tile height in blocks of 64 channels (build-time choices,
// measured; see the header and the launcher)
#ifndef ONE_BY_ONE_STAGES
#define ONE_BY_ONE_STAGES 2
#endif
#ifndef ONE_BY_ONE_MT
#define ONE_BY_ONE_MT 2
#endif

// What the loads need to know about a tile.
struct OneByOneTile {
    uint32_t P0, Pend;
    int m0;
    uint32_t b_voff;     // per lane: byte offset of its chunk of four pixels (and its channel of four)
    size_t b_tile;       // floats: plane 0 of the image of the tile's first pixel
};

// GATHER: the pixels of a tile are not contiguous in the source (a stride above 1: every s-th column of
// every row of the im2win tensor, every s-th row and column of the input in the workspace-free call) or
// do not come in groups of four.  B is then copied one word per lane -- lane = pixel, one channel row of
// 64 pixels per instruction, each lane fetching its own pixel -- into the same LDS layout; the filter
// still travels 16 bytes per lane.  (Eight such loads per wave and K block of 32 channels keep the
// address path of the memory pipeline busy for half of the block's MFMA time.)
// MT = 2: the workgroup's tile is 128 output channels x 64 pixels, every wave owns two 32x32 blocks (rows
// r and r + 64) whose MFMA chains are independent and share their pixel operand: half the pixel traffic and
// LDS reads per MFMA, and two chains to interleave.
template <int K1, bool GATHER, int NST, int MT>
__global__ __launch_bounds__(256) void conv_mfma_1x1_kernel(OneByOneParams P)
{
    static_assert(NST >= 2 && NST <= 4, "two to four LDS stages");
    static_assert(MT == 1 || MT == 2, "one or two blocks of 64 output channels");
    constexpr int STAGE1 = stage1_floats<K1, MT>();
    constexpr int CPR = K1 / 4;          // 16-byte chunks per filter row and block
    constexpr int RPI = 64 / CPR;        // filter rows per load instruction (a wave's 1 KB)
    constexpr int NI = K1 / 16;          // load instructions per wave, block and operand
    extern __shared__ __align__(16) unsigned char smem[];
    float *lds = reinterpret_cast<float *>(smem);   // NST stages

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int h = lane >> 5, l32 = lane & 31;

    // Persistent workgroups: the grid takes the tiles round by round, the workgroups of one XCD (every
    // eighth one) on neighbouring tiles, so that the channel blocks of a pixel tile -- consecutive
    // tile numbers -- read their shared pixels through one L2 at about the same time.
    const uint32_t tstep = gridDim.x, xcd = blockIdx.x % 8u;
    const uint32_t tile0 = xcd * (tstep / 8u) + min(xcd, tstep % 8u) + blockIdx.x / 8u;
    if (tile0 >= P.ntiles) return;

    // B: lane = (channel of four: lane / 16, chunk of four pixels: lane % 16).  The tile's pixels may
    // straddle images; a chunk never does (planes are a multiple of four pixels).  Chunks past the
    // layer's last pixel re-read its last chunk (their outputs are never stored).
    auto geometry = [&](uint32_t t) __attribute__((always_inline)) {
        OneByOneTile T;
        const uint32_t tile_n = fdiv(t, P.d_tm);
        T.m0 = (int)(t - tile_n * P.tiles_m) * (MT * MB);
        T.P0 = tile_n * NB;
        T.Pend = min(T.P0 + NB - 1, P.npix - 1);
        const uint32_t img0 = fdiv(T.P0, P.d_howo);
        T.b_tile = (size_t)img0 * P.Ci * P.plane;
        if constexpr (GATHER) {
            // lane = pixel of the tile; pixels past the layer's last re-read it (never stored)
            const uint32_t Pl = min(T.P0 + (uint32_t)lane, P.npix - 1u);
            const uint32_t img = fdiv(Pl, P.d_howo);
            const uint32_t pin = Pl - img * P.howo;
            const uint32_t m = fdiv(pin, P.d_wo), n = pin - m * P.Wo;
            T.b_voff = ((img - img0) * (uint32_t)P.Ci * P.plane + m * P.rowstep + n * P.colstep) * 4u;
        } else {
            const uint32_t Pl = min(T.P0 + 4u * (uint32_t)(lane & 15), P.npix - 4u);
            const uint32_t img = fdiv(Pl, P.d_howo);
            const uint32_t pin = Pl - img * P.howo;
            T.b_voff = ((img - img0) * (uint32_t)P.Ci * P.plane + pin + (uint32_t)(lane >> 4) * P.plane) * 4u;
        }
        return T;
    };
    // A: lane = (row of RPI: lane / CPR, slot: lane % CPR); instruction I of a wave covers rows RPI*I ..
    // RPI*I + RPI-1.  With four rows per instruction (RPI*I + r) & 7 = (4I & 4) | r: the slot permutation
    // has two forms, for even and odd I, and I = wave + 4j has the parity of the wave; with eight rows it
    // is r.  Row groups past Co re-read the last rows (their accumulators are never stored).
    const uint32_t Ci4 = (uint32_t)P.Ci * 4u;
    const int a_r = lane / CPR;
    const uint32_t a_voff = (uint32_t)a_r * Ci4 + (uint32_t)((lane % CPR) ^ ((RPI * (wave & 1) + a_r) & 7)) * 16u;
    auto desc = [](const float *base, size_t elems) __attribute__((always_inline)) {
        const size_t left = elems * 4u;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(base), 0,
                                                 left < 0xffffffffull ? left : 0xffffffffull, 0x00020000);
    };
    const __amdgpu_buffer_rsrc_t ra = desc(P.flt, P.flt_elems);
    const uint32_t plane4 = P.plane * 4u;

    // K block kb of tile T on its way into stage st: wave w issues instructions w, w+4, ... of each operand,
    // the same number for every block (the wait below counts them).  The last block may hold fewer than K1
    // channels (a multiple of eight): the channel groups it does not have re-read the layer's last channels,
    // and the filter chunks past the row's end bring whatever follows in memory (zeros past the tensor); both
    // land in slots no MFMA of that block reads.
    constexpr int LPI = (GATHER ? K1 / 4 : NI) + MT * NI;     // load instructions per wave and block
    auto issue = [&](const OneByOneTile &T, int kb, int st) __attribute__((always_inline)) {
        float *sB = lds + st * STAGE1, *sA = sB + K1 * NB;
        const __amdgpu_buffer_rsrc_t rb = desc(P.in + T.b_tile, P.in_elems - T.b_tile);
        if constexpr (GATHER) {
#pragma unroll
            for (int j = 0; j < K1 / 4; ++j) {
                const int c = wave + 4 * j;                   // channel c of the block: its 64 pixels
                const int ch = min(kb * K1 + c, P.Ci - 1);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_void_t *)(sB + c * NB), 4, T.b_voff,
                                                         (uint32_t)ch * plane4, 0, 0);
            }
        } else {
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int I = wave + 4 * j;                   // channels 4I .. 4I+3 of the block
                const int ch = min(kb * K1 + 4 * I, P.Ci - 4);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_void_t *)(sB + I * 256), 16, T.b_voff,
                                                         (uint32_t)ch * plane4, 0, 0);
            }
        }
#pragma unroll
        for (int j = 0; j < MT * NI; ++j) {
            const int I = wave + 4 * j;                       // filter rows RPI*I .. of the tile
            const int row = min(T.m0 + RPI * I, P.T.Co - RPI);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void_t *)(sA + I * 256), 16, a_voff,
                                                     (uint32_t)row * Ci4 + (uint32_t)kb * (K1 * 4), 0, 0);
        }
    };

    // operand bases of this lane, relative to a stage
    const int row = wm * 32 + l32;                            // filter row of the tile
    const int b_lane = wn * 32 + l32 + h * (4 * NB);          // pixel, plus the lane half's channel offset
    const int a_lane = K1 * NB + row * K1;
    const int nkb = (P.Ci + K1 - 1) / K1;

    // One flat sequence of K blocks over all of the workgroup's tiles.  The loads run NST - 1 blocks ahead of
    // the matrix cores -- into the next tile after a tile's last block, so a tile's stores go out while its
    // successor's first blocks arrive.  "Issue cursor": the block whose loads go out next.
    uint32_t t_i = tile0;
    int kb_i = 0;
    bool live = true;                                         // blocks are left to request
    OneByOneTile Ti = geometry(tile0);
    auto issue_next = [&](int st) __attribute__((always_inline)) {
        issue(Ti, kb_i, st);
        if (++kb_i == nkb) {
            kb_i = 0;
            t_i += tstep;
            if (t_i < P.ntiles) Ti = geometry(t_i); else live = false;
        }
    };
#pragma unroll
    for (int i = 0; i < NST - 1; ++i)
        if (live) issue_next(i);
    int st = 0;
    for (uint32_t t = tile0; t < P.ntiles; t += tstep) {
        floatx16 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][v] = 0.0f;
        for (int kb = 0; kb < nkb; ++kb) {
            // This wave's loads of the block have landed: memory operations retire in issue order, and after
            // the block's loads at most NST - 2 blocks' worth (and a tile's stores) were issued.  At the end
            // of the sequence, where fewer are in flight, wait for all.
            constexpr int AHEAD = LPI * (NST - 2);
            if (NST > 2 && live) __builtin_amdgcn_s_waitcnt(0x0F70 | (AHEAD & 15) | ((AHEAD >> 4) << 14));
            else __builtin_amdgcn_s_waitcnt(0x0F70);
            // everyone's have, and the stage read last is free again.  (A bare barrier instruction: a fence,
            // also one over LDS only, makes the compiler wait for every load in flight, since the loads
            // write LDS.  The wait above is what orders this wave's part of the block before the barrier;
            // the wave's LDS reads of the previous block were consumed by its MFMAs.)
            asm volatile("s_barrier" ::: "memory");
            int st_free = st + NST - 1;
            if (st_free >= NST) st_free -= NST;
            if (live) issue_next(st_free);
            const float *sS = lds + st * STAGE1;
            const float *bp = sS + b_lane;
            const float *ap = sS + a_lane;
            const int nq = min(K1, P.Ci - kb * K1) >> 3;   // groups of eight channels in this block
            // chunk 2q + h of the row sits at slot (2q + h) ^ (row & 7)
            if constexpr (MT == 2) {
                // whole blocks only (the launcher sees to it): all operand reads go out first -- LDS answers in
                // order, so an MFMA waits for its own operands only -- and the two blocks' chains alternate
                float4v_t a[MT][K1 / 8];
                float b[K1 / 2];
#pragma unroll
                for (int q = 0; q < K1 / 8; ++q) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        a[mt][q] = *reinterpret_cast<const float4v_t *>(ap + mt * (MB * K1) + 4 * ((2 * q + h) ^ (row & 7)));
#pragma unroll
                    for (int i = 0; i < 4; ++i) b[4 * q + i] = bp[(8 * q + i) * NB];
                }
#pragma unroll
                for (int q = 0; q < K1 / 8; ++q) {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
                            acc[mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mt][q][i], b[4 * q + i], acc[mt], 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int q = 0; q < K1 / 8; ++q) {
                    if (q >= nq) break;
                    const float4v_t a = *reinterpret_cast<const float4v_t *>(ap + 4 * ((2 * q + h) ^ (row & 7)));
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, bp[(8 * q + 0) * NB], acc[0], 0, 0, 0);
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, bp[(8 * q + 1) * NB], acc[0], 0, 0, 0);
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, bp[(8 * q + 2) * NB], acc[0], 0, 0, 0);
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, bp[(8 * q + 3) * NB], acc[0], 0, 0, 0);
                }
            }
            if (++st == NST) st = 0;
        }
        const uint32_t tile_n = fdiv(t, P.d_tm);
        const uint32_t P0 = tile_n * NB;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            store_tile_desc(P.T, acc[mt], P0, min(P0 + NB - 1, P.npix - 1), (int)(t - tile_n * P.tiles_m) * (MT * MB) + mt * MB,
                            wm, wn, h, l32);
    }
}

template <int K1, bool GATHER, int NST, int MT>
static hipError_t launch_1x1_t(OneByOneParams &P, const Shape &sh, hipStream_t st, LaunchPlan *plan)
{
    constexpr size_t lds = (size_t)NST * stage1_floats<K1, MT>() * sizeof(float);
    P.tiles_m = (uint32_t)((sh.Co + MT * MB - 1) / (MT * MB));
    P.d_tm = make_fastdiv(P.tiles_m);
    P.ntiles = ((P.npix + NB - 1) / NB) * P.tiles_m;
    constexpr int per_cu = (int)(160u * 1024u / lds) < 4 ? (int)(160u * 1024u / lds) : 4;   // resident workgroups per CU (LDS; four at most)
    int dev = 0, ncu = 0;
    hipError_t e = device_cus(&dev, &ncu);
    if (e != hipSuccess && plan) { e = hipSuccess; ncu = 256; }   // planning without a device: an MI355X's 256 compute units
    if (e != hipSuccess) return e;
    // Layers with up to 128 channels run persistent workgroups (as many as fit: 64 or 32 KB of LDS
    // each; whole groups of eight so that every XCD gets its share): a tile is then as short as the wait
    // for its first block, which only the prefetch across tiles hides (64 -> 256 channels at 56x56:
    // 67 -> 76 TFLOP/s).  With longer K loops one workgroup per tile is faster (512 -> 512 channels at
    // 14x14: 110 against 100 TFLOP/s): the hardware hands tiles out as workgroups finish, where the fixed
    // rounds leave some workgroups a tile short.
    uint32_t blocks = P.ntiles;
    if ((sh.Ci + 63) / 64 <= 2) {
        blocks = (uint32_t)(ncu * per_cu);
        if (blocks >= 8) blocks &= ~7u;
        if (blocks > P.ntiles) blocks = P.ntiles;
    }
    if (plan) { plan_record(plan, dim3(blocks), 256, lds, "conv_mfma_1x1_kernel<%d, %s, %d, %d>", K1, tf(GATHER), NST, MT); return hipSuccess; }
    static KernelCache kc;
    void (*kern)(OneByOneParams) = &conv_mfma_1x1_kernel<K1, GATHER, NST, MT>;
    if ((e = allow_dynamic_lds(kc, reinterpret_cast<const void *>(kern), lds, dev)) != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), lds, st, P);
    return hipGetLastError();
}

// Returns hipErrorNotSupported when the layer does not meet this kernel's conditions.  `src` is the
// im2win tensor of the layer -- for a 1x1 filter without padding: [N][Ci][Ho][Wi], the input rows m*s --
// or, with `implicit`, the NCHW input itself (workspace-free call).
hipError_t launch_conv_mfma_1x1(const float *src, const float *flt, float *out, const Shape &sh,
                                hipStream_t st, bool implicit, LaunchPlan *plan)
{
    if (sh.Hf != 1 || sh.Wf != 1 || sh.p != 0) return hipErrorNotSupported;
    if (sh.Ci % 8 != 0 || sh.Co % 4 != 0) return hipErrorNotSupported;   // (K steps come in groups of eight channels; filter rows are copied four at a time)
    if (reinterpret_cast<uintptr_t>(flt) % 16u != 0) return hipErrorNotSupported;
    const long long howo = (long long)sh.Ho * sh.Wo;
    const long long plane = implicit ? (long long)sh.Hi * sh.Wi : (long long)sh.Ho * sh.Wi;
    // 16-byte loads of the pixels: they are contiguous and come in whole groups of four
    const bool gather = sh.s != 1 || howo % 4 != 0 || reinterpret_cast<uintptr_t>(src) % 16u != 0;
    // 32-bit byte offsets: the images a tile's pixels span (two; more when a plane is smaller than a tile)
    // plus the channel offset of a load; the filter is addressed from its start
    const long long images = howo < NB ? NB / howo + 2 : 2;
    if ((images * sh.Ci + 8) * plane * 4LL >= (1LL << 32)) return hipErrorNotSupported;
    if ((long long)sh.Co * sh.Ci * 4LL >= (1LL << 32)) return hipErrorNotSupported;
    // (the epilogue's 32-bit output offsets: a tile's pixels within 4 GiB of its first image's first channel)
    if ((images * sh.Co + 64) * howo * 4LL >= (1LL << 32)) return hipErrorNotSupported;

    OneByOneParams P;
    P.in = src; P.flt = flt;
    P.Ci = sh.Ci;
    P.npix = (uint32_t)sh.npix;
    P.howo = (uint32_t)howo;
    P.tiles_m = (uint32_t)((sh.Co + MB - 1) / MB);
    P.in_elems = (size_t)sh.N * sh.Ci * (size_t)plane;
    P.flt_elems = (size_t)sh.Co * sh.Ci;
    P.d_howo = make_fastdiv(P.howo);
    P.d_tm = make_fastdiv(P.tiles_m);
    P.plane = (uint32_t)plane;
    // (with a single output row or column the step is never taken; a stride beyond the image then stays out
    // of the products -- the stride has no upper bound)
    P.rowstep = sh.Ho > 1 ? (uint32_t)(implicit ? sh.s * sh.Wi : sh.Wi) : 0u;
    P.colstep = sh.Wo > 1 ? (uint32_t)sh.s : 0u;
    P.Wo = (uint32_t)sh.Wo;
    P.d_wo = make_fastdiv(P.Wo);
    P.T = MfmaParams{};
    P.T.out = out; P.T.Co = sh.Co; P.T.howo = P.howo; P.T.d_howo = P.d_howo;
    P.T.out_elems = (size_t)sh.npix * sh.Co;
    P.ntiles = ((P.npix + NB - 1) / NB) * P.tiles_m;
    // K blocks of 32 channels leave room for four workgroups per CU, which hide each other's barriers and
    // load waits better than two with blocks of 64 (256 -> 256 channels at 28x28: 109 against 95 TFLOP/s);
    // they copy eight filter rows per instruction, hence for channel counts that are multiples of eight.
    if (sh.Co % 8 == 0) {
        constexpr int S = ONE_BY_ONE_STAGES;
        // Tiles of 128 output channels halve the pixel traffic; they pay where the pixel planes are large and
        // the K loop short (64 -> 256 and 256 -> 128 channels at 56x56: +3 to +4 %; 128 -> 512 at 28x28: +2 %)
        // and cost up to 3 % elsewhere (256 -> 256 at 28x28; 512 channels and more at 14x14 and 7x7).  Their
        // MFMA loop takes whole K blocks only.
        if (ONE_BY_ONE_MT == 2 && sh.Co % 128 == 0 && sh.Ci % 32 == 0 && (sh.Ci <= 128 || (sh.Ci <= 256 && howo >= 2048)))
            return gather ? launch_1x1_t<32, true, S, ONE_BY_ONE_MT>(P, sh, st, plan) : launch_1x1_t<32, false, S, ONE_BY_ONE_MT>(P, sh, st, plan);
        return gather ? launch_1x1_t<32, true, S, 1>(P, sh, st, plan) : launch_1x1_t<32, false, S, 1>(P, sh, st, plan);
    }
    return gather ? launch_1x1_t<64, true, 2, 1>(P, sh, st, plan) : launch_1x1_t<64, false, 2, 1>(P, sh, st, plan);
}

}  // namespace im2win
