"""Seeded synthetic workloads: shapes and value distributions only.

This module holds none of the method's arithmetic.  It is the one piece that
both the HIP path's callers and the oracle's callers use, so that the two are
fed identical bits.  The five named layers stand in for the workloads the
paper measures (single- and three-channel image maps of Tables 1-2, GAN
generator layers of Table 3) whose images and trained weights are not
available; timing does not depend on the values.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

SEED_BASE = 220903704


@dataclass(frozen=True)
class Layer:
    name: str
    B: int
    Cin: int
    Cout: int
    N: int          # input map edge
    n: int          # kernel edge
    dtype: str      # "f32" | "bf16" | "f16" (16-bit operands, fp32 accumulate and output)
    in_dist: str    # "uniform" | "normal" | "relu_normal"
    w_std: float = 0.02
    P: int = 0      # padding factor on the up-sampled map

    @property
    def M(self) -> int:
        """Output edge: (2N-1) + 2P - n + 1 (Section 1)."""
        return 2 * self.N - 1 + 2 * self.P - self.n + 1

    @property
    def in_shape(self):
        return (self.B, self.Cin, self.N, self.N)

    @property
    def w_shape(self):
        return (self.Cout, self.Cin, self.n, self.n)

    @property
    def out_shape(self):
        return (self.B, self.Cout, self.M, self.M)


# The five benchmark layers, in the order the baseline lists them.
LAYERS = (
    Layer("cfg1_tiny_1ch", 1, 1, 1, 32, 3, "f32", "uniform"),
    Layer("cfg2_1ch_bandwidth", 64, 1, 1, 512, 5, "f32", "normal"),
    Layer("cfg3_gan_n4", 128, 512, 256, 16, 4, "f32", "relu_normal"),
    Layer("cfg4_deep_n5", 64, 1024, 512, 8, 5, "f32", "relu_normal"),
    Layer("cfg5_late_bf16", 32, 256, 128, 64, 3, "bf16", "relu_normal"),
)


# Shapes the paper itself measures, all with padding factor 2: the 224 x 224 x 3 image maps of
# Tables 1-2 reduced to one output channel with 3 x 3, 4 x 4 and 5 x 5 kernels, and the
# DCGAN / DiscoGAN generator layers 2-5 of Table 3 (4 x 4 kernels), here at a batch of 64.
PAPER_LAYERS = (
    Layer("table1_224x224x3_n3_p2", 16, 3, 1, 224, 3, "f32", "uniform", P=2),
    Layer("table1_224x224x3_n4_p2", 16, 3, 1, 224, 4, "f32", "uniform", P=2),
    Layer("table1_224x224x3_n5_p2", 16, 3, 1, 224, 5, "f32", "uniform", P=2),
    # the same image layers at a batch that fills the chip (about 3700 tiles at 16 images are two rounds of workgroups)
    Layer("table1_224x224x3_n3_p2_b256", 256, 3, 1, 224, 3, "f32", "uniform", P=2),
    Layer("table1_224x224x3_n5_p2_b256", 256, 3, 1, 224, 5, "f32", "uniform", P=2),
    Layer("table3_dcgan_l2_4to8", 64, 1024, 512, 4, 4, "f32", "relu_normal", P=2),
    Layer("table3_dcgan_l3_8to16", 64, 512, 256, 8, 4, "f32", "relu_normal", P=2),
    Layer("table3_dcgan_l4_16to32", 64, 256, 128, 16, 4, "f32", "relu_normal", P=2),
    Layer("table3_dcgan_l5_32to64", 64, 128, 3, 32, 4, "f32", "relu_normal", P=2),
)


# Table 1's first row group: all 769 images of one class of the flower data set (224 x 224 x 3, one
# output channel, padding factor 2) with 5 x 5, 4 x 4 and 3 x 3 kernels.  Here: 769 synthetic images
# of that shape in one launch.  Entries: kernel edge -> the total seconds Table 1 prints for the
# class (conventional on the GPU, proposed on the GPU, conventional on the CPU, proposed on the
# CPU; RTX 2070 and Xeon), context beside this library's figures, never a target.
TABLE1_CLASS_IMAGES = 769
TABLE1_CLASS_SECONDS = {
    5: (3.6233, 1.018, 61.388, 15.714),
    4: (2.715, 0.741, 38.978, 10.331),
    3: (1.7454, 0.4916, 22.491, 6.098),
}


def table1_class_layers():
    """[(Layer, paper seconds)] for the three kernel sizes of Table 1 on a whole class of images."""
    return [(Layer("table1_class769_n%d_p2" % n, TABLE1_CLASS_IMAGES, 3, 1, 224, n, "f32", "uniform", P=2), sec)
            for n, sec in TABLE1_CLASS_SECONDS.items()]


# Table 3's transpose-convolution layers of four generator families, one input sample each
# (the paper times the forward pass of a single sample): 4 x 4 kernels, padding factor 2, so every
# layer doubles its map (N -> 2N).  Entries: (layer number, N, Cin, Cout).  The second tuple holds
# the seconds Table 3 prints for that layer, as context beside this library's figures and never as
# a target: (conventional on the GPU, proposed on the GPU, conventional on the CPU, proposed on the
# CPU), measured by the authors on an RTX 2070 and a Xeon.
TABLE3_GENERATORS = {
    "dcgan_discogan": (
        ((2, 4, 1024, 512), (0.046753, 0.011541, 3.023, 0.727)),
        ((3, 8, 512, 256), (0.046085, 0.011381, 3.101, 0.6863)),
        ((4, 16, 256, 128), (0.043747, 0.011296, 2.90, 0.6598)),
        ((5, 32, 128, 3), (0.003049, 0.001551, 0.1363, 0.0371)),
    ),
    "art_gan": (
        ((2, 4, 512, 256), (0.011886, 0.005768, 0.7114, 0.1782)),
        ((3, 8, 256, 128), (0.011726, 0.002971, 0.7219, 0.1652)),
        ((4, 16, 128, 128), (0.021727, 0.00568, 1.3879, 0.316)),
        ((6, 32, 128, 3), (0.001582, 0.001532, 0.0359, 0.0075)),
    ),
    "gp_gan": (
        ((2, 4, 512, 256), (0.011847, 0.005787, 0.7114, 0.1782)),
        ((3, 8, 256, 128), (0.01171, 0.002952, 0.7219, 0.1652)),
        ((4, 16, 128, 64), (0.01167, 0.002895, 0.6995, 0.1611)),
        ((5, 32, 64, 3), (0.001574, 0.000852, 0.0659, 0.016)),
    ),
    "eb_gan": (
        ((2, 4, 2048, 1024), (0.188821, 0.046078, 16.0994, 3.598)),
        ((3, 8, 1024, 512), (0.176702, 0.045508, 14.193, 2.919)),
        ((4, 16, 512, 256), (0.172839, 0.045071, 16.587, 2.950)),
        ((5, 32, 256, 128), (0.172694, 0.042322, 12.197, 2.866)),
        ((6, 64, 128, 64), (0.175486, 0.041105, 11.745, 2.774)),
        ((7, 128, 64, 64), (0.349605, 0.082192, 22.398, 5.233)),
    ),
}


def table3_layers(model: str, B: int = 1):
    """Table 3's layers of one generator family as Layer records at batch B, with the seconds the
    table prints for each: a list of (Layer, (conv_gpu_s, prop_gpu_s, conv_cpu_s, prop_cpu_s))."""
    out = []
    for (num, N, Cin, Cout), paper_s in TABLE3_GENERATORS[model]:
        name = "table3_%s_l%d_%dto%d_b%d" % (model, num, N, 2 * N, B)
        out.append((Layer(name, B, Cin, Cout, N, 4, "f32", "relu_normal", P=2), paper_s))
    return out


def layer_by_name(name: str) -> Layer:
    for i, l in enumerate(LAYERS):
        if l.name == name or name in ("cfg%d" % (i + 1), str(i + 1)):
            return l
    for l in PAPER_LAYERS:
        if l.name == name:
            return l
    for l, _ in table1_class_layers():
        if l.name == name:
            return l
    # a generator layer of Table 3 at any batch: table3_<model>_l<k>_<N>to<2N>_b<B>
    for model in TABLE3_GENERATORS:
        prefix = "table3_%s_l" % model
        if name.startswith(prefix) and "_b" in name:
            tail = name.rsplit("_b", 1)[1]
            if tail.isdigit():
                for l, _ in table3_layers(model, int(tail)):
                    if l.name == name:
                        return l
    raise KeyError(name)


def layer_seed(layer: Layer) -> int:
    for i, l in enumerate(LAYERS + PAPER_LAYERS):
        if l is layer or l == layer:
            return SEED_BASE + i
    return SEED_BASE + 1000


def make_tensors(layer: Layer, seed: int | None = None):
    """(x, w) as CPU torch tensors in the layer's operand dtype.

    The input is drawn first, then the weights, from one seeded CPU generator.
    For "bf16" the fp32 draws are rounded once, to nearest even, to bfloat16:
    both the HIP path and the oracle consume those rounded bits.
    """
    g = torch.Generator(device="cpu")
    g.manual_seed(layer_seed(layer) if seed is None else seed)
    if layer.in_dist == "uniform":
        x = torch.rand(layer.in_shape, generator=g, dtype=torch.float32) * 2.0 - 1.0
    elif layer.in_dist == "normal":
        x = torch.randn(layer.in_shape, generator=g, dtype=torch.float32)
    elif layer.in_dist == "relu_normal":
        x = torch.randn(layer.in_shape, generator=g, dtype=torch.float32).clamp_(min=0.0)
    elif layer.in_dist == "integer":
        x = torch.randint(-4, 5, layer.in_shape, generator=g).to(torch.float32)
    else:
        raise ValueError(layer.in_dist)
    if layer.in_dist == "integer":
        w = torch.randint(-3, 4, layer.w_shape, generator=g).to(torch.float32)
    else:
        w = torch.randn(layer.w_shape, generator=g, dtype=torch.float32) * layer.w_std
    if layer.dtype == "bf16":
        x = x.to(torch.bfloat16)
        w = w.to(torch.bfloat16)
    elif layer.dtype == "f16":
        x = x.to(torch.float16)
        w = w.to(torch.float16)
    elif layer.dtype != "f32":
        raise ValueError(layer.dtype)
    return x.contiguous(), w.contiguous()


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of an fp32 / bf16 CPU tensor to a float64 numpy array."""
    return t.detach().cpu().to(torch.float64).numpy()
