// Measurement probes (declared in include/im2win_probe.h): the yardsticks the
// benchmark holds the path's kernels against, measured on the same device in the
// same process.  Not part of the im2win path.
//   - a register-resident v_mfma_f32_32x32x2_f32 loop: what the fp32 matrix pipes
//     deliver with no operand traffic at all;
//   - streaming kernels (read-only, write-only, copy) with 16-byte accesses and
//     several independent accesses in flight per thread: what HBM delivers to a
//     kernel that does nothing but move bytes.
#include "../../include/im2win_probe.h"
#include "common.h"
#include "runtime_cache.h"

namespace im2win {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

constexpr int PROBE_NACC = 4;   // independent accumulator blocks per wave: hides the MFMA latency

__global__ __launch_bounds__(256) void probe_mfma_f32_kernel(float *sink, int iters, float a0, float b0)
{
    floatx16 acc[PROBE_NACC];
#pragma unroll
    for (int i = 0; i < PROBE_NACC; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
    const float a = a0 + (float)threadIdx.x * 1e-9f, b = b0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < PROBE_NACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < PROBE_NACC; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    if (s == 123.456f) sink[0] = s;   // never true for the operands the host passes; keeps the chain alive
}

// MODE 0: copy, 1: read only, 2: write only.  NT: non-temporal accesses.  A block moves
// contiguous pieces of 256 threads x U x 16 bytes; a thread's U accesses are independent and
// each instruction of a wave covers 1 KiB of consecutive addresses.
template <int MODE, bool NT, int U>
__global__ __launch_bounds__(256) void probe_stream_kernel(const uint4v *__restrict__ src, uint4v *__restrict__ dst,
                                                           size_t n16, uint32_t fill)
{
    const size_t per_iter = (size_t)gridDim.x * 256u * U;
    uint4v keep = {0u, 0u, 0u, 0u};
    for (size_t base = (size_t)blockIdx.x * 256u * U; base < n16; base += per_iter) {
        uint4v v[U];
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const size_t i = base + (size_t)j * 256u + threadIdx.x;
            if (MODE != 2) {
                if (i < n16) v[j] = NT ? __builtin_nontemporal_load(src + i) : src[i];
                else v[j] = keep;
            } else {
                v[j] = (uint4v){fill, fill + (uint32_t)j, fill, fill};
            }
        }
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const size_t i = base + (size_t)j * 256u + threadIdx.x;
            if (MODE == 1) {
                keep |= v[j];
            } else if (i < n16) {
                if (NT) __builtin_nontemporal_store(v[j], dst + i);
                else dst[i] = v[j];
            }
        }
    }
    // read only: the words are OR-ed together and stored only if they are all ones, which the
    // buffers the benchmark passes never are
    if (MODE == 1 && (keep.x & keep.y & keep.z & keep.w) == 0xffffffffu && fill == 0x12345u) dst[0] = keep;
}

template <int MODE, bool NT>
static hipError_t launch_stream(const void *src, void *dst, size_t bytes, hipStream_t st)
{
    constexpr int U = 8;
    int dev = 0, ncu = 0;
    hipError_t e = device_cus(&dev, &ncu);
    if (e != hipSuccess) return e;
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 256u * U - 1) / (256u * U);
    const size_t cap = (size_t)ncu * 8;   // eight resident workgroups per compute unit, looping
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((probe_stream_kernel<MODE, NT, U>), dim3((uint32_t)blocks), dim3(256), 0, st,
                       reinterpret_cast<const uint4v *>(src), reinterpret_cast<uint4v *>(dst), n16, 0x3f800000u);
    return hipGetLastError();
}

}  // namespace im2win

extern "C" {

im2win_status im2win_probe_mfma_f32(float *sink_dev, int mfma_per_wave, double *flops, void *stream)
{
    if (!sink_dev || !flops) return IM2WIN_ERR_NULL;
    if (mfma_per_wave < im2win::PROBE_NACC || mfma_per_wave > (1 << 24)) return IM2WIN_ERR_SHAPE;
    int dev = 0, ncu = 0;
    if (im2win::device_cus(&dev, &ncu) != hipSuccess) return IM2WIN_ERR_HIP;
    const int iters = mfma_per_wave / im2win::PROBE_NACC;
    const unsigned blocks = (unsigned)ncu * 2u;   // two workgroups of four waves per compute unit
    hipLaunchKernelGGL(im2win::probe_mfma_f32_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                       sink_dev, iters, 1.0f, 1.0f);
    if (hipGetLastError() != hipSuccess) return IM2WIN_ERR_HIP;
    // one v_mfma_f32_32x32x2_f32 is a 32x32x2 block product: 2*32*32*2 flops
    *flops = (double)blocks * 4.0 * (double)iters * im2win::PROBE_NACC * 4096.0;
    return IM2WIN_OK;
}

im2win_status im2win_probe_stream(int mode, const void *src_dev, void *dst_dev, size_t bytes, void *stream)
{
    const int kind = mode & 3, nt = mode & IM2WIN_PROBE_NONTEMPORAL;
    if (kind == 3 || (mode & ~(3 | IM2WIN_PROBE_NONTEMPORAL))) return IM2WIN_ERR_UNSUPPORTED;
    if (!dst_dev || (kind != IM2WIN_PROBE_WRITE && !src_dev)) return IM2WIN_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0) return IM2WIN_ERR_SHAPE;
    if (((uintptr_t)src_dev | (uintptr_t)dst_dev) & 15u) return IM2WIN_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    using namespace im2win;
    if (kind == IM2WIN_PROBE_COPY) e = nt ? launch_stream<0, true>(src_dev, dst_dev, bytes, st) : launch_stream<0, false>(src_dev, dst_dev, bytes, st);
    else if (kind == IM2WIN_PROBE_READ) e = nt ? launch_stream<1, true>(src_dev, dst_dev, bytes, st) : launch_stream<1, false>(src_dev, dst_dev, bytes, st);
    else e = nt ? launch_stream<2, true>(src_dev, dst_dev, bytes, st) : launch_stream<2, false>(src_dev, dst_dev, bytes, st);
    return e == hipSuccess ? IM2WIN_OK : IM2WIN_ERR_HIP;
}

}  // extern "C"
