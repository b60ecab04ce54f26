/*
 * im2win_probe.h -- measurement probes of the MI355X (gfx950) im2win library.
 *
 * These calls are not part of the im2win path.  They run the two yardstick
 * kernels the benchmark reports the path's kernels against, on the same device
 * and in the same process: the rate of the fp32 matrix cores when every operand
 * already sits in registers (the ceiling of the convolution, Section 3.3's
 * micro-kernel with no memory traffic at all), and the rate at which a kernel
 * that only moves bytes streams through HBM (the ceiling of the im2win
 * transform of Section 3.1, which is a pure copy).
 *
 * Same conventions as im2win.h: device pointers on the current device, the
 * caller owns every buffer, calls enqueue on `stream` and never synchronise,
 * errors are returned and then nothing is launched.  The caller times the call
 * (HIP events on the same stream).
 */
#ifndef IM2WIN_PROBE_H_
#define IM2WIN_PROBE_H_

#include "im2win.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Register-resident fp32 MFMA loop: two workgroups of four waves per compute unit,
 * each wave issues `mfma_per_wave` (rounded down to a multiple of 4; 4 .. 2^24)
 * v_mfma_f32_32x32x2_f32 on four independent accumulator blocks.
 *   sink_dev  device, at least one float; never written in practice
 *   flops     host, receives the floating-point operations of the whole launch
 */
im2win_status im2win_probe_mfma_f32(float *sink_dev, int mfma_per_wave, double *flops, void *stream);

/*
 * Streaming kernel over `bytes` bytes (a multiple of 16; both pointers 16-byte
 * aligned), 16-byte accesses, eight independent accesses in flight per thread.
 *   mode      IM2WIN_PROBE_COPY   read src_dev, write dst_dev (2*bytes of traffic)
 *             IM2WIN_PROBE_READ   read src_dev only (dst_dev: at least 16 bytes, never
 *                                 written unless every word read is all ones)
 *             IM2WIN_PROBE_WRITE  write dst_dev only (src_dev may be NULL)
 *             optionally or-ed with IM2WIN_PROBE_NONTEMPORAL (non-temporal accesses)
 */
enum {
    IM2WIN_PROBE_COPY = 0,
    IM2WIN_PROBE_READ = 1,
    IM2WIN_PROBE_WRITE = 2,
    IM2WIN_PROBE_NONTEMPORAL = 4
};
im2win_status im2win_probe_stream(int mode, const void *src_dev, void *dst_dev, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* IM2WIN_PROBE_H_ */
