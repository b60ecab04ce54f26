"""Seeded synthetic inputs for the five benchmark layers.

This module holds no arithmetic of the method: it only names the layer shapes
and draws the input and filter values.  It is the one module that both the GPU
tests/benchmark and the CPU oracle's callers use, so that both sides see the
same host arrays.

The layers stand in for the paper's benchmark layers (Table 2 gives shapes
only; the paper uses no dataset).  Layer 5 is Table 2's Conv1 at the paper's
batch of 128; layers 2-4 are the Conv9 / Conv11 / Conv3-like ResNet/VGG shapes
with the padding of their original networks.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Layer:
    name: str
    N: int
    Ci: int
    Hi: int
    Wi: int
    Co: int
    Hf: int
    Wf: int
    stride: int
    pad: int
    seed: int
    input_dist: str   # "uniform_pm1" | "uniform01" | "normal"
    filter_dist: str  # "uniform_pm1" | "he_normal"

    @property
    def dims(self):
        """Arguments in the order the C ABI takes them."""
        return (self.N, self.Ci, self.Hi, self.Wi, self.Co, self.Hf, self.Wf, self.stride, self.pad)


LAYERS = (
    Layer("cfg1_tiny_3x3", 1, 3, 32, 32, 16, 3, 3, 1, 0, 1001, "uniform_pm1", "uniform_pm1"),
    Layer("cfg2_3x3_c64_56", 32, 64, 56, 56, 64, 3, 3, 1, 1, 1002, "uniform01", "he_normal"),
    Layer("cfg3_3x3_c256_14", 128, 256, 14, 14, 256, 3, 3, 1, 1, 1003, "uniform01", "he_normal"),
    Layer("cfg4_7x7_s2_c3_224", 128, 3, 224, 224, 64, 7, 7, 2, 3, 1004, "normal", "he_normal"),
    Layer("cfg5_11x11_s4_c3_227", 128, 3, 227, 227, 96, 11, 11, 4, 0, 1005, "normal", "he_normal"),
)


# The twelve benchmark layers of the paper's Table 2 (unpadded, batch 128 as in Section 4.2).
# The paper does not say what values its tensors hold: N(0,1) inputs and He-normal filters here.
def _t2(name, Ci, Hi, Co, Hf, s, seed):
    return Layer("table2_" + name, 128, Ci, Hi, Hi, Co, Hf, Hf, s, 0, seed, "normal", "he_normal")


TABLE2 = (
    _t2("conv1", 3, 227, 96, 11, 4, 2001), _t2("conv2", 3, 231, 96, 11, 4, 2002),
    _t2("conv3", 3, 227, 64, 7, 2, 2003), _t2("conv4", 64, 224, 64, 7, 2, 2004),
    _t2("conv5", 96, 24, 256, 5, 1, 2005), _t2("conv6", 256, 12, 512, 3, 1, 2006),
    _t2("conv7", 3, 224, 64, 3, 1, 2007), _t2("conv8", 64, 112, 128, 3, 1, 2008),
    _t2("conv9", 64, 56, 64, 3, 1, 2009), _t2("conv10", 128, 28, 128, 3, 1, 2010),
    _t2("conv11", 256, 14, 256, 3, 1, 2011), _t2("conv12", 512, 7, 512, 3, 1, 2012),
)


# Layers off the specialised kernels' grid, timed by `bench.py --extra`: a channel count that is not a
# multiple of the pipelined kernel's K block, 1x1 layers (expanding, reducing, strided, 7x7 planes), row and
# column filters, a 4x4 stride-2 layer.
EXTRA = (
    Layer("extra_3x3_c60_56", 32, 60, 56, 56, 64, 3, 3, 1, 1, 3001, "uniform01", "he_normal"),
    Layer("extra_3x3_c100_28", 64, 100, 28, 28, 128, 3, 3, 1, 1, 3002, "uniform01", "he_normal"),
    Layer("extra_1x1_c256_28", 64, 256, 28, 28, 256, 1, 1, 1, 0, 3003, "uniform01", "he_normal"),
    Layer("extra_1x7_c64_28", 64, 64, 28, 28, 64, 1, 7, 1, 0, 3004, "uniform01", "he_normal"),
    Layer("extra_1x1_c64_56_co256", 64, 64, 56, 56, 256, 1, 1, 1, 0, 3005, "uniform01", "he_normal"),
    Layer("extra_1x1_c1024_14_co256", 64, 1024, 14, 14, 256, 1, 1, 1, 0, 3006, "uniform01", "he_normal"),
    Layer("extra_1x1_s2_c256_56_co512", 64, 256, 56, 56, 512, 1, 1, 2, 0, 3007, "uniform01", "he_normal"),
    Layer("extra_1x1_c2048_7_co512", 128, 2048, 7, 7, 512, 1, 1, 1, 0, 3008, "uniform01", "he_normal"),
    Layer("extra_7x1_c128_17_co192", 128, 128, 17, 17, 192, 7, 1, 1, 3, 3009, "uniform01", "he_normal"),
    Layer("extra_4x4_s2_c64_64_co128", 64, 64, 64, 64, 128, 4, 4, 2, 1, 3010, "uniform01", "he_normal"),
)


def layer(index_or_name) -> Layer:
    """Layer by 1-based index (1..5) or by name."""
    if isinstance(index_or_name, int):
        return LAYERS[index_or_name - 1]
    for l in LAYERS + TABLE2 + EXTRA:
        if l.name == index_or_name:
            return l
    raise KeyError(index_or_name)


def with_batch(l: Layer, N: int) -> Layer:
    """The same layer at another batch size (same seed: a prefix of nothing, new draws)."""
    return Layer(l.name + "_n%d" % N, N, l.Ci, l.Hi, l.Wi, l.Co, l.Hf, l.Wf, l.stride, l.pad,
                 l.seed, l.input_dist, l.filter_dist)


def make_inputs(l: Layer):
    """Host fp32 tensors (input I, filter F): input drawn first, then the filter,
    from one CPU generator seeded with the layer's seed."""
    g = torch.Generator(device="cpu")
    g.manual_seed(l.seed)
    ishape = (l.N, l.Ci, l.Hi, l.Wi)
    fshape = (l.Co, l.Ci, l.Hf, l.Wf)
    if l.input_dist == "uniform_pm1":
        I = torch.rand(ishape, generator=g, dtype=torch.float32) * 2.0 - 1.0
    elif l.input_dist == "uniform01":
        I = torch.rand(ishape, generator=g, dtype=torch.float32)
    elif l.input_dist == "normal":
        I = torch.randn(ishape, generator=g, dtype=torch.float32)
    else:
        raise ValueError(l.input_dist)
    if l.filter_dist == "uniform_pm1":
        F = torch.rand(fshape, generator=g, dtype=torch.float32) * 2.0 - 1.0
    elif l.filter_dist == "he_normal":
        sigma = math.sqrt(2.0 / (l.Ci * l.Hf * l.Wf))
        F = torch.randn(fshape, generator=g, dtype=torch.float32) * sigma
    else:
        raise ValueError(l.filter_dist)
    return I.contiguous(), F.contiguous()


def random_layer_inputs(seed: int, N, Ci, Hi, Wi, Co, Hf, Wf):
    """Small uniform[-1,1] tensors for edge-case tests."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    I = torch.rand((N, Ci, Hi, Wi), generator=g, dtype=torch.float32) * 2.0 - 1.0
    F = torch.rand((Co, Ci, Hf, Wf), generator=g, dtype=torch.float32) * 2.0 - 1.0
    return I.contiguous(), F.contiguous()
