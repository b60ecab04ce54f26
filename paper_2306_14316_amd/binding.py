"""ctypes binding of the C ABI declared in include/im2win.h (same names).

Tensors are torch CUDA (ROCm) tensors used as raw device buffers; the current
torch stream is handed to the library as the hipStream_t.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libim2win.so")
_lib = None

EXPORTS = (
    "im2win_out_shape",
    "im2win_workspace_bytes",
    "im2col_footprint_bytes",
    "im2win_transform",
    "conv2d_im2win_fwd",
    "conv2d_im2win_fwd_basic",
    "conv2d_im2win_fwd_variant",
    "conv2d_im2win_implicit_fwd",
    "conv2d_direct_fwd",
    "im2col_transform",
    "conv2d_im2col_fwd",
    "im2win_status_str",
    "im2win_transform_launch_info",
    "conv2d_im2win_fwd_launch_info",
)
# measurement probes, declared in include/im2win_probe.h
PROBE_EXPORTS = ("im2win_probe_mfma_f32", "im2win_probe_stream")


class LaunchInfo(ctypes.Structure):
    """im2win_launch_info of the header."""
    _fields_ = [("kernel", ctypes.c_char * 160), ("grid_x", ctypes.c_uint), ("grid_y", ctypes.c_uint),
                ("block", ctypes.c_uint), ("lds_bytes", ctypes.c_size_t)]

    def as_dict(self):
        return {"kernel": self.kernel.decode(), "grid": [self.grid_x, self.grid_y], "block": self.block,
                "lds_bytes": self.lds_bytes}


class Im2winError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_str(status), status))


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libim2win.so (built in-tree by paper_2306_14316_amd.build); fails loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                "%s not found: build it with `python -m paper_2306_14316_amd.build` "
                "(or __graft_entry__.build())" % _LIB_PATH)
        lib = ctypes.CDLL(_LIB_PATH)
        i, vp, sp = ctypes.c_int, ctypes.c_void_p, ctypes.POINTER(ctypes.c_size_t)
        ip = ctypes.POINTER(ctypes.c_int)
        lib.im2win_out_shape.restype = i
        lib.im2win_out_shape.argtypes = [i] * 6 + [ip, ip]
        for name in ("im2win_workspace_bytes", "im2col_footprint_bytes"):
            getattr(lib, name).restype = i
            getattr(lib, name).argtypes = [i] * 8 + [sp]
        for name in ("im2win_transform", "im2col_transform"):
            getattr(lib, name).restype = i
            getattr(lib, name).argtypes = [vp, vp] + [i] * 8 + [vp]
        for name in ("conv2d_im2win_fwd", "conv2d_im2win_fwd_basic", "conv2d_direct_fwd", "conv2d_im2col_fwd",
                     "conv2d_im2win_implicit_fwd"):
            getattr(lib, name).restype = i
            getattr(lib, name).argtypes = [vp, vp, vp] + [i] * 9 + [vp]
        lib.conv2d_im2win_fwd_variant.restype = i
        lib.conv2d_im2win_fwd_variant.argtypes = [vp, vp, vp] + [i] * 10 + [vp]
        lib.im2win_status_str.restype = ctypes.c_char_p
        lib.im2win_status_str.argtypes = [i]
        lib.im2win_transform_launch_info.restype = i
        lib.im2win_transform_launch_info.argtypes = [i] * 8 + [ctypes.POINTER(LaunchInfo)]
        lib.conv2d_im2win_fwd_launch_info.restype = i
        lib.conv2d_im2win_fwd_launch_info.argtypes = [i] * 11 + [ctypes.POINTER(LaunchInfo)]
        lib.im2win_probe_mfma_f32.restype = i
        lib.im2win_probe_mfma_f32.argtypes = [vp, i, ctypes.POINTER(ctypes.c_double), vp]
        lib.im2win_probe_stream.restype = i
        lib.im2win_probe_stream.argtypes = [i, vp, vp, ctypes.c_size_t, vp]
        _lib = lib
    return _lib


def status_str(status: int) -> str:
    return load_library().im2win_status_str(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise Im2winError(status, where)


def im2win_out_shape(Hi, Wi, Hf, Wf, stride, pad):
    Ho, Wo = ctypes.c_int(), ctypes.c_int()
    _check(load_library().im2win_out_shape(Hi, Wi, Hf, Wf, stride, pad, ctypes.byref(Ho), ctypes.byref(Wo)),
           "im2win_out_shape")
    return Ho.value, Wo.value


def im2win_workspace_bytes(N, Ci, Hi, Wi, Hf, Wf, stride, pad) -> int:
    b = ctypes.c_size_t()
    _check(load_library().im2win_workspace_bytes(N, Ci, Hi, Wi, Hf, Wf, stride, pad, ctypes.byref(b)),
           "im2win_workspace_bytes")
    return b.value


def im2col_footprint_bytes(N, Ci, Hi, Wi, Hf, Wf, stride, pad) -> int:
    b = ctypes.c_size_t()
    _check(load_library().im2col_footprint_bytes(N, Ci, Hi, Wi, Hf, Wf, stride, pad, ctypes.byref(b)),
           "im2col_footprint_bytes")
    return b.value


def _window_elems(N, Ci, Hi, Wi, Hf, Wf, stride, pad) -> int:
    return im2win_workspace_bytes(N, Ci, Hi, Wi, Hf, Wf, stride, pad) // 4


def _out_elems(N, Co, Hi, Wi, Hf, Wf, stride, pad) -> int:
    Ho, Wo = im2win_out_shape(Hi, Wi, Hf, Wf, stride, pad)
    return N * Co * Ho * Wo


def layer_sizes(N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad) -> dict:
    """Ho, Wo and the element counts of the im2win tensor and the output, as the library derives them."""
    Ho, Wo = im2win_out_shape(Hi, Wi, Hf, Wf, stride, pad)
    return {"Ho": Ho, "Wo": Wo, "window_elems": _window_elems(N, Ci, Hi, Wi, Hf, Wf, stride, pad),
            "output_elems": N * Co * Ho * Wo}


def _dev_ptr(t, name: str, numel: int):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a torch tensor in GPU memory" % name)
    if t.dtype != torch.float32 or not t.is_contiguous():
        raise TypeError("%s must be contiguous fp32" % name)
    if t.numel() != numel:
        raise ValueError("%s has %d elements, expected %d" % (name, t.numel(), numel))
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def im2win_transform(input, window, N, Ci, Hi, Wi, Hf, Wf, stride, pad, stream=None):
    """window <- im2win(input); both are device tensors owned by the caller."""
    a = _dev_ptr(input, "input", N * Ci * Hi * Wi)
    w = _dev_ptr(window, "window", _window_elems(N, Ci, Hi, Wi, Hf, Wf, stride, pad))
    _check(load_library().im2win_transform(a, w, N, Ci, Hi, Wi, Hf, Wf, stride, pad, _stream(stream)),
           "im2win_transform")


def _conv(fn_name, window, filter, output, N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, stream):
    w = _dev_ptr(window, "window", _window_elems(N, Ci, Hi, Wi, Hf, Wf, stride, pad))
    f = _dev_ptr(filter, "filter", Co * Ci * Hf * Wf)
    o = _dev_ptr(output, "output", _out_elems(N, Co, Hi, Wi, Hf, Wf, stride, pad))
    fn = getattr(load_library(), fn_name)
    _check(fn(w, f, o, N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, _stream(stream)), fn_name)


def conv2d_im2win_fwd(window, filter, output, N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, stream=None):
    """output <- convolution over the im2win tensor on the fp32 matrix cores."""
    _conv("conv2d_im2win_fwd", window, filter, output, N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, stream)


def conv2d_im2win_fwd_basic(window, filter, output, N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, stream=None):
    """output <- the one-thread-per-output kernel (Algorithm 2)."""
    _conv("conv2d_im2win_fwd_basic", window, filter, output, N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, stream)


VARIANT_DEFAULT, VARIANT_NO_PIPELINE, VARIANT_NO_MFMA, VARIANT_NARROW_LOADS = 0, 1, 2, 3
VARIANT_VALU_MICROKERNEL, VARIANT_SCALAR_LOADS = 4, 5


def conv2d_im2win_fwd_variant(window, filter, output, N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, variant,
                              stream=None):
    """output <- the convolution computed by one of the ablation variants (VARIANT_*)."""
    w = _dev_ptr(window, "window", _window_elems(N, Ci, Hi, Wi, Hf, Wf, stride, pad))
    f = _dev_ptr(filter, "filter", Co * Ci * Hf * Wf)
    o = _dev_ptr(output, "output", _out_elems(N, Co, Hi, Wi, Hf, Wf, stride, pad))
    _check(load_library().conv2d_im2win_fwd_variant(w, f, o, N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad,
                                                     int(variant), _stream(stream)),
           "conv2d_im2win_fwd_variant")


def conv2d_im2win_implicit_fwd(input, filter, output, N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, stream=None):
    """output <- the im2win convolution straight from the NCHW input (no workspace)."""
    a = _dev_ptr(input, "input", N * Ci * Hi * Wi)
    f = _dev_ptr(filter, "filter", Co * Ci * Hf * Wf)
    o = _dev_ptr(output, "output", _out_elems(N, Co, Hi, Wi, Hf, Wf, stride, pad))
    _check(load_library().conv2d_im2win_implicit_fwd(a, f, o, N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad,
                                                      _stream(stream)),
           "conv2d_im2win_implicit_fwd")


def conv2d_direct_fwd(input, filter, output, N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, stream=None):
    """output <- the direct convolution (baseline): one thread per output, no workspace."""
    a = _dev_ptr(input, "input", N * Ci * Hi * Wi)
    f = _dev_ptr(filter, "filter", Co * Ci * Hf * Wf)
    o = _dev_ptr(output, "output", _out_elems(N, Co, Hi, Wi, Hf, Wf, stride, pad))
    _check(load_library().conv2d_direct_fwd(a, f, o, N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, _stream(stream)),
           "conv2d_direct_fwd")


def im2col_transform(input, col, N, Ci, Hi, Wi, Hf, Wf, stride, pad, stream=None):
    """col <- the stacked im2col matrices (baseline), N*Ho*Wo rows of Ci*Hf*Wf floats."""
    a = _dev_ptr(input, "input", N * Ci * Hi * Wi)
    c = _dev_ptr(col, "col", im2col_footprint_bytes(N, Ci, Hi, Wi, Hf, Wf, stride, pad) // 4)
    _check(load_library().im2col_transform(a, c, N, Ci, Hi, Wi, Hf, Wf, stride, pad, _stream(stream)),
           "im2col_transform")


def conv2d_im2col_fwd(col, filter, output, N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, stream=None):
    """output <- GEMM of the im2col matrix with the filter matrix (baseline)."""
    c = _dev_ptr(col, "col", im2col_footprint_bytes(N, Ci, Hi, Wi, Hf, Wf, stride, pad) // 4)
    f = _dev_ptr(filter, "filter", Co * Ci * Hf * Wf)
    o = _dev_ptr(output, "output", _out_elems(N, Co, Hi, Wi, Hf, Wf, stride, pad))
    _check(load_library().conv2d_im2col_fwd(c, f, o, N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, _stream(stream)),
           "conv2d_im2col_fwd")


def im2win_transform_launch_info(N, Ci, Hi, Wi, Hf, Wf, stride, pad) -> dict:
    """The kernel im2win_transform would launch for this layer (nothing is launched)."""
    info = LaunchInfo()
    _check(load_library().im2win_transform_launch_info(N, Ci, Hi, Wi, Hf, Wf, stride, pad, ctypes.byref(info)),
           "im2win_transform_launch_info")
    return info.as_dict()


def conv2d_im2win_fwd_launch_info(N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, variant=VARIANT_DEFAULT,
                                  workspace_free=False) -> dict:
    """The kernel conv2d_im2win_fwd_variant (or conv2d_im2win_implicit_fwd) would launch (nothing is launched)."""
    info = LaunchInfo()
    _check(load_library().conv2d_im2win_fwd_launch_info(N, Ci, Hi, Wi, Co, Hf, Wf, stride, pad, int(variant),
                                                         1 if workspace_free else 0, ctypes.byref(info)),
           "conv2d_im2win_fwd_launch_info")
    return info.as_dict()


PROBE_COPY, PROBE_READ, PROBE_WRITE, PROBE_NONTEMPORAL = 0, 1, 2, 4


def _raw_ptr(t, name: str):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or not t.is_contiguous():
        raise TypeError("%s must be a contiguous torch tensor in GPU memory" % name)
    return ctypes.c_void_p(t.data_ptr())


def im2win_probe_mfma_f32(sink, mfma_per_wave: int, stream=None) -> float:
    """Enqueue the register-resident fp32 MFMA loop; returns the flops of the launch."""
    fl = ctypes.c_double()
    _check(load_library().im2win_probe_mfma_f32(_dev_ptr(sink, "sink", sink.numel()), int(mfma_per_wave),
                                                 ctypes.byref(fl), _stream(stream)), "im2win_probe_mfma_f32")
    return fl.value


def im2win_probe_stream(mode: int, src, dst, nbytes: int, stream=None):
    """Enqueue a streaming kernel (PROBE_COPY / PROBE_READ / PROBE_WRITE, | PROBE_NONTEMPORAL) over nbytes."""
    for t, name in ((src, "src"), (dst, "dst")):
        if t is not None and t.numel() * t.element_size() < (nbytes if not (name == "dst" and (mode & 3) == PROBE_READ) else 16):
            raise ValueError("%s is smaller than %d bytes" % (name, nbytes))
    _check(load_library().im2win_probe_stream(int(mode), _raw_ptr(src, "src") if src is not None else None,
                                               _raw_ptr(dst, "dst"), int(nbytes), _stream(stream)),
           "im2win_probe_stream")
