"""CPU oracle for the im2win convolution path -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end of ``im2win_oracle.c`` (plain C, fp64 arithmetic,
OpenMP over independent outputs).  Only ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py`` may import this package; the GPU
library never does, and the two share no code.

Notation follows the paper (Section 2.1): I[N][Ci][Hi][Wi], F[Co][Ci][Hf][Wf],
O[N][Co][Ho][Wo], stride s; zero padding p is this build's extension.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "im2win_oracle.c")
_LIB = os.path.join(_HERE, "libim2win_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math) and return the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
               "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32, i64, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p
        lib.oracle_out_dim.restype = i32
        lib.oracle_out_dim.argtypes = [i32] * 4
        for name in ("oracle_im2win_elems", "oracle_im2col_elems"):
            getattr(lib, name).restype = i64
            getattr(lib, name).argtypes = [i32] * 8
        lib.oracle_conv2d_direct.restype = i32
        lib.oracle_conv2d_direct.argtypes = [vp, vp] + [i32] * 9 + [vp, vp]
        lib.oracle_conv2d_direct_at.restype = i32
        lib.oracle_conv2d_direct_at.argtypes = [vp, vp] + [i32] * 9 + [vp, i64, vp, vp]
        lib.oracle_im2win.restype = i32
        lib.oracle_im2win.argtypes = [vp, vp] + [i32] * 8
        lib.oracle_im2col.restype = i32
        lib.oracle_im2col.argtypes = [vp, vp] + [i32] * 7
        lib.oracle_conv2d_im2col_gemm.restype = i32
        lib.oracle_conv2d_im2col_gemm.argtypes = [vp, vp] + [i32] * 9 + [vp]
        lib.oracle_conv2d_over_im2win.restype = i32
        lib.oracle_conv2d_over_im2win.argtypes = [vp, vp] + [i32] * 9 + [vp]
        _lib = lib
    return _lib


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("oracle inputs are fp32 arrays, got %s" % a.dtype)
    return a


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _dims(I: np.ndarray, F: np.ndarray):
    if I.ndim != 4 or F.ndim != 4 or I.shape[1] != F.shape[1]:
        raise ValueError("expected I[N,Ci,Hi,Wi] and F[Co,Ci,Hf,Wf]")
    N, Ci, Hi, Wi = I.shape
    Co, _, Hf, Wf = F.shape
    return N, Ci, Hi, Wi, Co, Hf, Wf


def out_dim(size: int, f: int, s: int, p: int) -> int:
    """floor((size + 2p - f)/s) + 1, or -1 if the filter does not fit."""
    return int(_load().oracle_out_dim(size, f, s, p))


def out_shape(Hi, Wi, Hf, Wf, s, p):
    Ho, Wo = out_dim(Hi, Hf, s, p), out_dim(Wi, Wf, s, p)
    if Ho < 0 or Wo < 0:
        raise ValueError("filter does not fit the padded input")
    return Ho, Wo


def im2win_elems(N, Ci, Hi, Wi, Hf, Wf, s, p) -> int:
    return int(_load().oracle_im2win_elems(N, Ci, Hi, Wi, Hf, Wf, s, p))


def im2col_elems(N, Ci, Hi, Wi, Hf, Wf, s, p) -> int:
    return int(_load().oracle_im2col_elems(N, Ci, Hi, Wi, Hf, Wf, s, p))


def conv2d_direct(I, F, s: int, p: int, with_bound: bool = True):
    """Seven-loop direct convolution (Eq. 1); returns (O fp64, B fp64 or None)."""
    I, F = _f32(I), _f32(F)
    N, Ci, Hi, Wi, Co, Hf, Wf = _dims(I, F)
    Ho, Wo = out_shape(Hi, Wi, Hf, Wf, s, p)
    O = np.empty((N, Co, Ho, Wo), dtype=np.float64)
    B = np.empty_like(O) if with_bound else None
    rc = _load().oracle_conv2d_direct(_ptr(I), _ptr(F), N, Ci, Hi, Wi, Co, Hf, Wf, s, p,
                                      _ptr(O), _ptr(B) if with_bound else None)
    if rc != 0:
        raise ValueError("oracle_conv2d_direct failed: %d" % rc)
    return O, B


def conv2d_direct_at(I, F, s: int, p: int, idx):
    """The same definition at sampled outputs; idx is an int array [count,4] of (i,j,m,n)."""
    I, F = _f32(I), _f32(F)
    N, Ci, Hi, Wi, Co, Hf, Wf = _dims(I, F)
    out_shape(Hi, Wi, Hf, Wf, s, p)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    if idx.ndim != 2 or idx.shape[1] != 4:
        raise ValueError("idx must be [count,4]")
    O = np.empty(idx.shape[0], dtype=np.float64)
    B = np.empty_like(O)
    rc = _load().oracle_conv2d_direct_at(_ptr(I), _ptr(F), N, Ci, Hi, Wi, Co, Hf, Wf, s, p,
                                         _ptr(idx), idx.shape[0], _ptr(O), _ptr(B))
    if rc != 0:
        raise ValueError("oracle_conv2d_direct_at failed: %d" % rc)
    return O, B


def im2win(I, Hf: int, Wf: int, s: int, p: int) -> np.ndarray:
    """im2win tensor What[N][Ci][Ho][Wp*Hf] (Eq. 2), values copied bit for bit."""
    I = _f32(I)
    N, Ci, Hi, Wi = I.shape
    Ho, _ = out_shape(Hi, Wi, Hf, Wf, s, p)
    W = np.empty((N, Ci, Ho, (Wi + 2 * p) * Hf), dtype=np.float32)
    rc = _load().oracle_im2win(_ptr(I), _ptr(W), N, Ci, Hi, Wi, Hf, Wf, s, p)
    if rc != 0:
        raise ValueError("oracle_im2win failed: %d" % rc)
    return W


def im2col(Iimg, Hf: int, Wf: int, s: int, p: int) -> np.ndarray:
    """im2col matrix (Ho*Wo) x (Ci*Hf*Wf) of one image I'[Ci][Hi][Wi] (Section 2.3)."""
    Iimg = _f32(Iimg)
    Ci, Hi, Wi = Iimg.shape
    Ho, Wo = out_shape(Hi, Wi, Hf, Wf, s, p)
    M = np.empty((Ho * Wo, Ci * Hf * Wf), dtype=np.float64)
    rc = _load().oracle_im2col(_ptr(Iimg), _ptr(M), Ci, Hi, Wi, Hf, Wf, s, p)
    if rc != 0:
        raise ValueError("oracle_im2col failed: %d" % rc)
    return M


def conv2d_im2col_gemm(I, F, s: int, p: int) -> np.ndarray:
    """GEMM-based convolution through explicit im2col matrices (Section 2.3)."""
    I, F = _f32(I), _f32(F)
    N, Ci, Hi, Wi, Co, Hf, Wf = _dims(I, F)
    Ho, Wo = out_shape(Hi, Wi, Hf, Wf, s, p)
    O = np.empty((N, Co, Ho, Wo), dtype=np.float64)
    rc = _load().oracle_conv2d_im2col_gemm(_ptr(I), _ptr(F), N, Ci, Hi, Wi, Co, Hf, Wf, s, p, _ptr(O))
    if rc != 0:
        raise ValueError("oracle_conv2d_im2col_gemm failed: %d" % rc)
    return O


def conv2d_over_im2win(What, F, Hi: int, Wi: int, s: int, p: int) -> np.ndarray:
    """Convolution as dot products over the contiguous windows of the im2win tensor (Section 3.1-3.2)."""
    What, F = _f32(What), _f32(F)
    Co, Ci, Hf, Wf = F.shape
    N = What.shape[0]
    Ho, Wo = out_shape(Hi, Wi, Hf, Wf, s, p)
    if What.shape != (N, Ci, Ho, (Wi + 2 * p) * Hf):
        raise ValueError("im2win tensor has the wrong shape %s" % (What.shape,))
    O = np.empty((N, Co, Ho, Wo), dtype=np.float64)
    rc = _load().oracle_conv2d_over_im2win(_ptr(What), _ptr(F), N, Ci, Hi, Wi, Co, Hf, Wf, s, p, _ptr(O))
    if rc != 0:
        raise ValueError("oracle_conv2d_over_im2win failed: %d" % rc)
    return O
