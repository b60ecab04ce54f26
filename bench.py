#!/usr/bin/env python3
"""Benchmark of the im2win hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input that is
already resident in HBM: the im2win transform followed by the convolution over
the im2win tensor.  The headline workload is the 3x3, 64-channel, 56x56 layer
at batch 32; with --layers all the other four layers are timed as well and
reported under "layers".

Prints ONE JSON line.  `value` is fp32 convolution TFLOP/s of the whole step
(2*N*Co*Ho*Wo*Ci*Hf*Wf flops / step time, transform included); the roofline
object is for the dominant kernel (the MFMA convolution) and is timed with HIP
events on the launch stream inside the timed region; cpu_baseline is the CPU
oracle timed on the host cores of the same box.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MATRIX_TFLOPS = 157.3   # MI355X dense fp32 MFMA: 256 CU x 256 flop/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0             # MI355X HBM3E

# HBM traffic of one launch of each kernel, bytes, keyed by layer name: measured with two
# rocprofv3 --pmc runs of this script (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch) and scaled by
# what the same counters read for a plain 256 MiB device copy in the same runs (factors 2.000 and
# 1.000).  The values are the TRAFFIC_BYTES lines of profiles/all_layers_default_bench.md, which
# gives the commands; tests/test_host_api.py holds the two to each other.  Layers that were not
# measured report null.
MEASURED_CONV_TRAFFIC_BYTES = {
    "cfg1_tiny_3x3": 209324,
    "cfg2_3x3_c64_56": 107723384,
    "cfg3_3x3_c256_14": 215418276,
    "cfg4_7x7_s2_c3_224": 689076020,
    "cfg5_11x11_s4_c3_227": 362789419}
MEASURED_TRANSFORM_TRAFFIC_BYTES = {
    "cfg1_tiny_3x3": 63485,
    "cfg2_3x3_c64_56": 105594963,
    "cfg3_3x3_c256_14": 113847631,
    "cfg4_7x7_s2_c3_224": 362295763,
    "cfg5_11x11_s4_c3_227": 298416819}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--layer", type=int, default=2, help="headline layer, 1..5 (default 2)")
    ap.add_argument("--layers", choices=["headline", "all"], default="all",
                    help="also time the other layers and list them under 'layers'")
    ap.add_argument("--table2", action="store_true",
                    help="also time the twelve layers of the paper's Table 2 at batch 128 (listed under 'table2')")
    ap.add_argument("--ablation", action="store_true",
                    help="also time the ablation variants of the convolution on the 3x3 layers (listed under 'ablation')")
    ap.add_argument("--baselines", action="store_true",
                    help="also time the comparison baselines (direct convolution; im2col + GEMM) on the five layers "
                         "(listed under 'baselines')")
    ap.add_argument("--extra", action="store_true",
                    help="also time layers off the specialised kernels' grid (ragged channel counts, 1x1, "
                         "asymmetric filters; listed under 'extra')")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (known traffic) so that a rocprofv3 --pmc "
                         "run of this command can scale FETCH_SIZE / WRITE_SIZE")
    return ap.parse_args()


def layer_flops(L):
    """The metric's flop count of a layer, 2*N*Co*Ho*Wo*Ci*Hf*Wf, with the output size the library derives."""
    import paper_2306_14316_amd as im2win
    Ho, Wo = im2win.im2win_out_shape(L.Hi, L.Wi, L.Hf, L.Wf, L.stride, L.pad)
    return 2 * L.N * L.Co * Ho * Wo * L.Ci * L.Hf * L.Wf


KERNEL_SAMPLES = 20   # launches per kernel timing batch, at least (whatever --steps says)


def time_layer(L, steps, warmup):
    """Run warmup + steps passes of transform+conv; returns timing dict (ms).

    Two separate measurements.  The step time is the wall clock around `steps` passes of the whole
    path, synchronised on both sides, with no events in between.  The per-kernel durations come
    right after, on the same stream and the same buffers: for each kernel, three batches of
    max(steps, KERNEL_SAMPLES) back-to-back launches between one pair of HIP events (an event
    pair around a single launch of a 20 us kernel reads several microseconds too long, and
    markers between the two kernels of a step keep them from being dispatched back to back; a
    kernel shorter than the host's launch period is queued behind a head start, see _event_ms);
    reported are the mean over all batches, the best and the median batch."""
    import torch
    import paper_2306_14316_amd as im2win
    from paper_2306_14316_amd import workloads

    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = L.dims
    I, F = workloads.make_inputs(L)
    dI, dF = I.cuda(), F.cuda()
    ws = im2win.im2win_workspace_bytes(N, Ci, Hi, Wi, Hf, Wf, s, p)
    col = im2win.im2col_footprint_bytes(N, Ci, Hi, Wi, Hf, Wf, s, p)
    Ho, Wo = im2win.im2win_out_shape(Hi, Wi, Hf, Wf, s, p)
    dW = torch.full((ws // 4,), float("nan"), dtype=torch.float32, device="cuda")
    dO = torch.full((N, Co, Ho, Wo), float("nan"), dtype=torch.float32, device="cuda")

    tr = lambda: im2win.im2win_transform(dI, dW, N, Ci, Hi, Wi, Hf, Wf, s, p)
    cv = lambda: im2win.conv2d_im2win_fwd(dW, dF, dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)

    def step():
        tr()
        cv()

    # Set-up, not part of the W warm-up steps: the first pass checks that every
    # output word is written, and a short burst brings the GPU clocks up (a cold
    # device needs a few milliseconds of load to leave its idle clock).
    step()
    torch.cuda.synchronize()
    if bool(torch.isnan(dO).any()) or bool(torch.isnan(dW).any()):
        raise RuntimeError("%s: an output element was never written" % L.name)
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < 0.05:
        for _ in range(20):
            step()
        torch.cuda.synchronize()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    # Each kernel's batches follow 20 ms of that kernel alone: the clocks take a few milliseconds to settle
    # when the load changes from memory-bound to matrix-bound work and back (without it the first batch of
    # the convolution after the transform's batches read up to 8 % long on some boxes).
    nk = max(steps, KERNEL_SAMPLES)
    _ramp(tr, 0.02)
    tr_b = [_event_ms(tr, nk) for _ in range(3)]
    _ramp(cv, 0.02)
    cv_b = [_event_ms(cv, nk) for _ in range(3)]
    # The workspace-free variant (strips built in LDS from the input): one call replaces the whole
    # step.  Timed the same way as the step, after the main measurement.
    imp_ms = None
    try:
        imp = lambda: im2win.conv2d_im2win_implicit_fwd(dI, dF, dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
        imp()
        torch.cuda.synchronize()
        for _ in range(max(5, warmup)):
            imp()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(steps):
            imp()
        torch.cuda.synchronize()
        imp_ms = (time.perf_counter() - t2) * 1e3 / steps
    except im2win.Im2winError:
        pass
    return dict(implicit_ms_per_step=imp_ms, ms_per_step=(t1 - t0) * 1e3 / steps,
                kernel_samples=3 * nk,
                transform_ms_avg=sum(tr_b) / 3, transform_ms_best=min(tr_b), transform_ms_median=sorted(tr_b)[1],
                conv_ms_avg=sum(cv_b) / 3, conv_ms_best=min(cv_b), conv_ms_median=sorted(cv_b)[1],
                workspace_bytes=ws, im2col_bytes=col,
                transform_alg_bytes=4 * N * Ci * Hi * Wi + ws,
                conv_alg_bytes=ws + 4 * Co * Ci * Hf * Wf + 4 * N * Co * Ho * Wo,
                flops=2 * N * Co * Ho * Wo * Ci * Hf * Wf, Ho=Ho, Wo=Wo)


def kernel_names(L):
    """(convolution kernel, transform kernel) of a layer, as the library's own dispatch names them."""
    import paper_2306_14316_amd as im2win
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = L.dims
    return (im2win.conv2d_im2win_fwd_launch_info(N, Ci, Hi, Wi, Co, Hf, Wf, s, p),
            im2win.im2win_transform_launch_info(N, Ci, Hi, Wi, Hf, Wf, s, p))


def layer_report(L, t):
    fl = t["flops"]
    conv_k, tr_k = kernel_names(L)
    return {
        "workload": L.name,
        "shape": {"N": L.N, "Ci": L.Ci, "Hi": L.Hi, "Wi": L.Wi, "Co": L.Co, "Hf": L.Hf, "Wf": L.Wf,
                  "stride": L.stride, "pad": L.pad},
        "conv_kernel": conv_k["kernel"], "transform_kernel": tr_k["kernel"],
        "step_tflops": fl / (t["ms_per_step"] * 1e-3) / 1e12,
        "conv_tflops_avg": fl / (t["conv_ms_avg"] * 1e-3) / 1e12,
        "conv_tflops_best": fl / (t["conv_ms_best"] * 1e-3) / 1e12,
        "conv_frac_of_fp32_matrix_peak": fl / (t["conv_ms_avg"] * 1e-3) / 1e12 / PEAK_FP32_MATRIX_TFLOPS,
        "transform_gbs_avg": t["transform_alg_bytes"] / (t["transform_ms_avg"] * 1e-3) / 1e9,
        "transform_frac_of_hbm_peak": t["transform_alg_bytes"] / (t["transform_ms_avg"] * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "ms_per_step": t["ms_per_step"], "kernel_samples": t["kernel_samples"],
        "conv_ms_avg": t["conv_ms_avg"], "conv_ms_best": t["conv_ms_best"], "conv_ms_median": t["conv_ms_median"],
        "transform_ms_avg": t["transform_ms_avg"], "transform_ms_best": t["transform_ms_best"],
        "transform_ms_median": t["transform_ms_median"],
        "workspace_bytes": t["workspace_bytes"], "im2col_bytes": t["im2col_bytes"],
        "conv_traffic_bytes": MEASURED_CONV_TRAFFIC_BYTES.get(L.name),
        "transform_traffic_bytes": MEASURED_TRANSFORM_TRAFFIC_BYTES.get(L.name),
        "workspace_free_ms_per_step": t["implicit_ms_per_step"],
        "workspace_free_step_tflops": (fl / (t["implicit_ms_per_step"] * 1e-3) / 1e12) if t["implicit_ms_per_step"] else None,
    }


def time_variants(L, steps):
    """Convolution-only timing of each ablation variant on one layer (HIP events, average of `steps`)."""
    import torch
    import paper_2306_14316_amd as im2win
    from paper_2306_14316_amd import workloads
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = L.dims
    I, F = workloads.make_inputs(L)
    dI, dF = I.cuda(), F.cuda()
    sz = im2win.layer_sizes(*L.dims)
    dW = torch.empty(sz["window_elems"], dtype=torch.float32, device="cuda")
    dO = torch.empty(sz["output_elems"], dtype=torch.float32, device="cuda")
    im2win.im2win_transform(dI, dW, N, Ci, Hi, Wi, Hf, Wf, s, p)
    names = {0: "default", 3: "narrow_loads (8-byte instead of 16-byte filter fetches)",
             5: "scalar_loads (4-byte filter fetches)",
             1: "no_pipeline (one LDS stage, no prefetch; matrix cores)",
             4: "valu_microkernel (no_pipeline's tiling with a 4x4 register tile per thread on the vector ALUs)",
             2: "no_mfma (Algorithm 2: one thread per output, no LDS, no register tile)"}
    out = {}
    _ramp(lambda: im2win.conv2d_im2win_fwd(dW, dF, dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p))
    for v, name in names.items():
        k = steps if v != 2 else max(2, steps // 10)
        try:
            for _ in range(10 if v != 2 else 1):
                im2win.conv2d_im2win_fwd_variant(dW, dF, dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p, v)
        except im2win.Im2winError:
            out[name] = None
            continue
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(k):
            im2win.conv2d_im2win_fwd_variant(dW, dF, dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p, v)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / k
        out[name] = {"conv_ms": ms, "conv_tflops": layer_flops(L) / (ms * 1e-3) / 1e12}
    return {"workload": L.name, "variants": out}


def _ramp(fn, seconds=0.05):
    import torch
    t = time.perf_counter()
    while time.perf_counter() - t < seconds:
        for _ in range(5):
            fn()
        torch.cuda.synchronize()


HOST_BOUND_MS = 0.030   # launches shorter than this may be paced by the host's launch rate, not by the GPU
_probe_sink = None


def _event_ms(fn, k, head_start=None):
    """Mean duration (ms) of k back-to-back launches of fn between one pair of HIP events.

    The host needs 10-20 us per launch through the Python binding, so a kernel shorter than that is
    measured at the host's pace with the GPU idle in between (a rocprofv3 trace of the same launches
    shows it).  When the first reading is below HOST_BOUND_MS the batch is therefore repeated behind
    a head start: the library's register-resident MFMA probe is queued first, sized to run while the
    host queues all k launches, the events go around the launches only, and the GPU then runs them
    back to back.  head_start=False / True forces one form."""
    import torch
    import paper_2306_14316_amd as im2win
    global _probe_sink

    def batch(ahead):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        if ahead:
            im2win.im2win_probe_mfma_f32(_probe_sink, max(2000, 800 * k))   # about 0.04 ms per launch to come
        e0.record()
        for _ in range(k):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / k

    if head_start is False:
        return batch(False)
    if _probe_sink is None:
        _probe_sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    if head_start:
        return batch(True)
    ms = batch(False)
    return batch(True) if ms < HOST_BOUND_MS else ms


def device_copy_gbs():
    """Bandwidth of a plain 256 MiB device-to-device copy of the runtime (bytes read + bytes written per second)."""
    import torch
    src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    _ramp(lambda: dst.copy_(src), 0.03)
    ms = min(_event_ms(lambda: dst.copy_(src), 10) for _ in range(3))
    del src, dst
    return 2.0 * 256 * 1024 * 1024 / (ms * 1e-3) / 1e9


def measured_stream_gbs(nbytes=256 * 1024 * 1024):
    """What this device's HBM delivers to the library's own streaming probe kernels (16-byte accesses,
    eight in flight per thread) over `nbytes`: read only, write only and copy, with ordinary and with
    non-temporal accesses.  GB/s of bytes moved (a copy moves 2 x nbytes); best of three batches of ten."""
    import torch
    import paper_2306_14316_amd as im2win
    src = torch.ones(nbytes // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    out = {}
    for name, mode, moved in (("read", im2win.PROBE_READ, nbytes), ("write", im2win.PROBE_WRITE, nbytes),
                              ("copy", im2win.PROBE_COPY, 2 * nbytes)):
        for nt in (0, im2win.PROBE_NONTEMPORAL):
            fn = lambda: im2win.im2win_probe_stream(mode | nt, src, dst, nbytes)
            _ramp(fn, 0.02)
            ms = min(_event_ms(fn, 10) for _ in range(3))
            out[name + ("_nontemporal" if nt else "")] = moved / (ms * 1e-3) / 1e9
    del src, dst
    return out


def measured_mfma_peak_tflops():
    """fp32 matrix rate of a register-resident v_mfma_f32_32x32x2_f32 loop on this device (the
    library's probe kernel: no operand traffic at all), best of three launches of about 2 ms."""
    import torch
    import paper_2306_14316_amd as im2win
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    per_wave = 40000
    _ramp(lambda: im2win.im2win_probe_mfma_f32(sink, per_wave), 0.05)
    best = 0.0
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        fl = im2win.im2win_probe_mfma_f32(sink, per_wave)
        e1.record()
        torch.cuda.synchronize()
        best = max(best, fl / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    return best


def time_baselines(L, steps):
    """The comparison baselines on one layer, beside the im2win path (HIP events, average of
    `steps` launches each): the direct convolution, and im2col followed by a GEMM."""
    import torch
    import paper_2306_14316_amd as im2win
    from paper_2306_14316_amd import workloads
    N, Ci, Hi, Wi, Co, Hf, Wf, s, p = L.dims
    I, F = workloads.make_inputs(L)
    dI, dF = I.cuda(), F.cuda()
    sz = im2win.layer_sizes(*L.dims)
    dO = torch.empty(sz["output_elems"], dtype=torch.float32, device="cuda")
    dW = torch.empty(sz["window_elems"], dtype=torch.float32, device="cuda")
    colb = im2win.im2col_footprint_bytes(N, Ci, Hi, Wi, Hf, Wf, s, p)
    res = {"workload": L.name, "im2win_workspace_bytes": dW.numel() * 4, "im2col_workspace_bytes": colb}

    def tf(ms):
        return layer_flops(L) / (ms * 1e-3) / 1e12

    f_t = lambda: im2win.im2win_transform(dI, dW, N, Ci, Hi, Wi, Hf, Wf, s, p)
    f_c = lambda: im2win.conv2d_im2win_fwd(dW, dF, dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    f_t()
    _ramp(f_c)
    t_ms, c_ms = _event_ms(f_t, steps), _event_ms(f_c, steps)
    res["im2win"] = {"transform_ms": t_ms, "conv_ms": c_ms, "conv_tflops": tf(c_ms), "total_tflops": tf(t_ms + c_ms)}

    col = torch.empty(colb // 4, dtype=torch.float32, device="cuda")
    f_i = lambda: im2win.im2col_transform(dI, col, N, Ci, Hi, Wi, Hf, Wf, s, p)
    f_g = lambda: im2win.conv2d_im2col_fwd(col, dF, dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    f_i()
    _ramp(f_g)
    i_ms, g_ms = _event_ms(f_i, steps), _event_ms(f_g, steps)
    res["im2col_gemm"] = {"transform_ms": i_ms, "conv_ms": g_ms, "conv_tflops": tf(g_ms), "total_tflops": tf(i_ms + g_ms)}
    del col

    f_d = lambda: im2win.conv2d_direct_fwd(dI, dF, dO, N, Ci, Hi, Wi, Co, Hf, Wf, s, p)
    f_d()
    d_ms = _event_ms(f_d, max(2, steps // 10))
    res["direct"] = {"conv_ms": d_ms, "total_tflops": tf(d_ms)}
    res["im2win_speedup_total"] = {"vs_im2col_gemm": (i_ms + g_ms) / (t_ms + c_ms), "vs_direct": d_ms / (t_ms + c_ms)}
    return res


def cpu_baseline(L):
    """The CPU oracle as it stands, timed on this machine's host cores on the same workload."""
    import oracle
    from paper_2306_14316_amd import workloads
    I, F = workloads.make_inputs(L)
    In, Fn = I.numpy(), F.numpy()
    cores = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
    t0 = time.perf_counter()
    oracle.im2win(In, L.Hf, L.Wf, L.stride, L.pad)
    oracle.conv2d_direct(In, Fn, L.stride, L.pad, with_bound=False)
    dt = time.perf_counter() - t0
    return {"value": layer_flops(L) / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "seconds": dt,
            "sample": "the whole %s workload (all %d images), one pass: im2win gather + seven-loop fp64 "
                      "direct convolution, OpenMP over (image, output channel)" % (L.name, L.N)}


def main():
    a = parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % a.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    import paper_2306_14316_amd as im2win
    from paper_2306_14316_amd import workloads
    im2win.load_library()

    if a.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")   # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    L = workloads.layer(a.layer)
    t = time_layer(L, a.steps, a.warmup)
    rep = layer_report(L, t)
    conv_tflops = rep["conv_tflops_avg"]
    traffic = MEASURED_CONV_TRAFFIC_BYTES.get(L.name)
    out = {
        "metric": "fp32 conv TFLOPS (2*N*Co*Ho*Wo*Ci*Hf*Wf / t), whole step = im2win transform + convolution",
        "value": rep["step_tflops"],
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": t["ms_per_step"],
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": L.name, **rep["shape"], "Ho": t["Ho"], "Wo": t["Wo"],
                   "gemm": {"M": L.Co, "N": L.N * t["Ho"] * t["Wo"], "K": L.Ci * L.Hf * L.Wf}},
        "workspace_bytes": t["workspace_bytes"], "im2col_bytes": t["im2col_bytes"],
        "conv_only_tflops": conv_tflops, "conv_only_tflops_best_of_steps": rep["conv_tflops_best"],
        "transform_gbs": rep["transform_gbs_avg"],
        "workspace_free_variant": {"ms_per_step": rep["workspace_free_ms_per_step"],
                                   "step_tflops": rep["workspace_free_step_tflops"],
                                   "note": "conv2d_im2win_implicit_fwd: one call, im2win strips built in LDS from the "
                                           "NCHW input, no workspace; not the headline (the step above is the paper's "
                                           "transform + convolution)"},
        "roofline": {"kernel": rep["conv_kernel"], "launch": kernel_names(L)[0], "bound": "mfma",
                     "achieved": conv_tflops,
                     "peak": PEAK_FP32_MATRIX_TFLOPS, "unit": "TFLOP/s",
                     "frac": conv_tflops / PEAK_FP32_MATRIX_TFLOPS, "traffic": traffic,
                     "flops_per_launch": t["flops"], "avg_launch_ms": t["conv_ms_avg"],
                     "launches_timed": t["kernel_samples"], "algorithmic_bytes": t["conv_alg_bytes"]},
        "roofline_transform": {"kernel": rep["transform_kernel"], "launch": kernel_names(L)[1], "bound": "hbm",
                               "achieved": rep["transform_gbs_avg"],
                               "peak": PEAK_HBM_GBS, "unit": "GB/s",
                               "frac": rep["transform_gbs_avg"] / PEAK_HBM_GBS,
                               "traffic": MEASURED_TRANSFORM_TRAFFIC_BYTES.get(L.name),
                               "bytes_per_launch": t["transform_alg_bytes"], "avg_launch_ms": t["transform_ms_avg"],
                               "launches_timed": t["kernel_samples"]},
        "paper_context": "paper reports ratios only, on an RTX 3090 at fp32, batch 128: im2win 3.5x im2col+cuBLAS, "
                         "1.1x (up to 1.8x) the fastest cuDNN algorithm, 5-155x a naive direct kernel",
    }
    # the two measured ceilings, from this device in this process
    peak = measured_mfma_peak_tflops()
    out["roofline"]["measured_mfma_peak_tflops"] = peak
    out["roofline"]["frac_of_measured_peak"] = conv_tflops / peak
    copy_gbs = device_copy_gbs()
    streams = measured_stream_gbs()
    best_stream = max(max(streams["copy"], streams["copy_nontemporal"]), copy_gbs)
    out["roofline_transform"]["measured_copy_gbs"] = copy_gbs
    out["roofline_transform"]["measured_stream_gbs"] = streams
    out["roofline_transform"]["frac_of_measured_copy"] = rep["transform_gbs_avg"] / best_stream
    if a.layers == "all":
        reps = []
        for other in workloads.LAYERS:
            if other.name == L.name:
                reps.append(rep)
            else:
                k = max(10, min(a.steps, 30))
                reps.append(layer_report(other, time_layer(other, k, min(a.warmup, 5))))
        for r in reps:
            r["conv_frac_of_measured_mfma_peak"] = r["conv_tflops_avg"] / peak
            r["transform_frac_of_measured_copy"] = r["transform_gbs_avg"] / best_stream
        out["layers"] = reps
    if a.ablation:
        out["ablation"] = [time_variants(workloads.layer(i), max(5, min(a.steps, 30))) for i in (2, 3)]
    if a.baselines:
        out["baselines"] = [time_baselines(l, max(5, min(a.steps, 20))) for l in workloads.LAYERS[1:]]
        if a.table2:   # the paper's comparison (Section 4.3) on its own twelve layers
            out["baselines_table2"] = [time_baselines(l, max(3, min(a.steps, 10))) for l in workloads.TABLE2]
    if a.table2:
        out["table2"] = [layer_report(t2, time_layer(t2, max(5, min(a.steps, 20)), 3)) for t2 in workloads.TABLE2]
    if a.extra:
        out["extra"] = [layer_report(x, time_layer(x, max(5, min(a.steps, 20)), 3)) for x in workloads.EXTRA]
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(L)
        if a.layers == "all":   # the oracle on every layer, whole workloads (a second or less each)
            for r, other in zip(out["layers"], workloads.LAYERS):
                cb = out["cpu_baseline"] if other.name == L.name else cpu_baseline(other)
                r["cpu_seconds"], r["cpu_tflops"], r["cpu_cores"] = cb["seconds"], cb["value"], cb["cores"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
