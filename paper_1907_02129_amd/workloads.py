"""Seeded synthetic convolution workloads.

This module only describes problem shapes and draws random input / filter
tensors for them.  It holds none of the method's arithmetic (no output-size
formula, no convolution, no indirection logic) so that both the CPU oracle's
tests and the HIP path's tests can feed on exactly the same bytes without
sharing any code of the method itself.

Shapes use the notation of the paper's problem statement (Listing 1 and the
paragraph after it): batch N, input Hin x Win, input channels C, output
channels K, kernel R x S, stride SY/SX, dilation DY/DX, implicit zero padding
(top/left/bottom/right).  Tensors are NHWC and the filter is [K][R][S][C].

The data stands in for the conv layers of the networks the paper measures
(ResNet-18 / SqueezeNet 1.0, section "Models"): layer-like shapes, random
values, no trained weights.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np


@dataclass(frozen=True)
class ConvShape:
    name: str
    N: int
    Hin: int
    Win: int
    C: int
    K: int
    R: int
    S: int
    SY: int = 1
    SX: int = 1
    DY: int = 1
    DX: int = 1
    PT: int = 0
    PL: int = 0
    PB: int = 0
    PR: int = 0
    dtype: str = "bf16"          # "f32" | "bf16" | "u8i8"
    zero_point: int = 0          # u8i8 only: value of the padding row
    seed: int = 0
    in_scale: str = "unit"       # "unit" | "rsc": divide input by sqrt(R*S*C)
    dist: str = "normal"         # "normal" | "uniform"
    c_logical: int = 0           # >0: only the first c_logical channels are non-zero

    def with_(self, **kw) -> "ConvShape":
        return replace(self, **kw)


# The eight concrete shapes of the five benchmark configuration groups.
CONFIGS = {
    "cfg1_tiny_f32": ConvShape("cfg1_tiny_f32", 1, 8, 8, 4, 8, 3, 3, PT=1, PL=1, PB=1, PR=1,
                               dtype="f32", seed=0, dist="uniform"),
    "cfg2_3x3_c64": ConvShape("cfg2_3x3_c64", 32, 56, 56, 64, 64, 3, 3, PT=1, PL=1, PB=1, PR=1,
                              seed=1, in_scale="rsc"),
    "cfg3a_3x3_s2": ConvShape("cfg3a_3x3_s2", 32, 56, 56, 128, 256, 3, 3, SY=2, SX=2,
                              PT=1, PL=1, PB=1, PR=1, seed=2),
    "cfg3b_3x3_d2": ConvShape("cfg3b_3x3_d2", 16, 64, 64, 128, 128, 3, 3, DY=2, DX=2,
                              PT=2, PL=2, PB=2, PR=2, seed=3),
    "cfg3c_5x5_asym": ConvShape("cfg3c_5x5_asym", 8, 112, 112, 32, 64, 5, 5,
                                PT=2, PL=2, PB=1, PR=1, seed=4),
    "cfg4_int8_3x3": ConvShape("cfg4_int8_3x3", 32, 28, 28, 256, 256, 3, 3, PT=1, PL=1, PB=1, PR=1,
                               dtype="u8i8", zero_point=128, seed=5),
    "cfg5a_1x1": ConvShape("cfg5a_1x1", 32, 56, 56, 256, 64, 1, 1, seed=6),
    # first-layer conv: 3 real channels stored with a pixel stride of 4, the
    # fourth channel of input and filter is zero
    "cfg5b_7x7_s2": ConvShape("cfg5b_7x7_s2", 32, 224, 224, 4, 64, 7, 7, SY=2, SX=2,
                              PT=3, PL=3, PB=3, PR=3, seed=7, c_logical=3),
}



def _layer(model, tag, N, hw, C, K, k, stride, pad, seed, dtype="bf16"):
    return ConvShape(f"{model}.{tag}", N, hw, hw, C, K, k, k, SY=stride, SX=stride, PT=pad, PL=pad, PB=pad, PR=pad,
                     dtype=dtype, zero_point=128 if dtype == "u8i8" else 0, seed=seed)


def layer_type(s: ConvShape) -> str:
    """The row of the paper's Table 2 a shape belongs to, e.g. "3x3 stride-1"."""
    return f"{s.R}x{s.S} stride-{s.SY}"


def resnet18_layers(N: int = 32):
    """The distinct convolutions of ResNet-18 on 224 x 224 images, from the published architecture (a 7x7 stride-2
    stem to 112 x 112, a stride-2 pooling to 56 x 56, then four stages of 3x3 convolutions with 64, 128, 256, 512
    channels at 56, 28, 14, 7 pixels; each later stage opens with a stride-2 3x3 convolution and a stride-2 1x1
    projection on the shortcut).  Identical parameter sets appear once, as in the paper's Table 2."""
    out = [_layer("resnet18", "conv1", N, 224, 3, 64, 7, 2, 3, 1000)]
    hw, c = 56, 64
    out.append(_layer("resnet18", "stage1.3x3", N, hw, c, c, 3, 1, 1, 1001))
    for i, k in enumerate((128, 256, 512)):
        out.append(_layer("resnet18", f"stage{i + 2}.3x3s2", N, hw, c, k, 3, 2, 1, 1010 + 3 * i))
        out.append(_layer("resnet18", f"stage{i + 2}.1x1s2", N, hw, c, k, 1, 2, 0, 1011 + 3 * i))
        hw, c = hw // 2, k
        out.append(_layer("resnet18", f"stage{i + 2}.3x3", N, hw, c, c, 3, 1, 1, 1012 + 3 * i))
    return out


def squeezenet10_layers(N: int = 32):
    """The distinct convolutions of SqueezeNet 1.0 on 224 x 224 images, from the published architecture: an unpadded
    7x7 stride-2 stem with 96 filters (109 x 109), eight fire modules (a 1x1 squeeze, then a 1x1 and a padded 3x3
    expand side by side) with 3x3 stride-2 ceiling-mode poolings after the stem, fire4 and fire8 (54, 27, 13
    pixels), and a 1x1 classifier convolution with 1000 filters.  Identical parameter sets appear once."""
    out = [_layer("squeezenet", "conv1", N, 224, 3, 96, 7, 2, 0, 2000)]
    # (module, pixels, input channels, squeeze filters, expand filters per branch)
    fires = [(2, 54, 96, 16, 64), (3, 54, 128, 16, 64), (4, 54, 128, 32, 128), (5, 27, 256, 32, 128),
             (6, 27, 256, 48, 192), (7, 27, 384, 48, 192), (8, 27, 384, 64, 256), (9, 13, 512, 64, 256)]
    seen = set()
    for m, hw, cin, sq, ex in fires:
        for tag, c, k, r in ((f"fire{m}.squeeze", cin, sq, 1), (f"fire{m}.expand1x1", sq, ex, 1),
                             (f"fire{m}.expand3x3", sq, ex, 3)):
            key = (hw, c, k, r)
            if key in seen:
                continue
            seen.add(key)
            out.append(_layer("squeezenet", tag, N, hw, c, k, r, 1, r // 2, 2000 + 10 * m + r))
    out.append(_layer("squeezenet", "conv10", N, 13, 512, 1000, 1, 1, 0, 2100))
    return out


# The configuration the headline metric is quoted on.
HEADLINE = "cfg2_3x3_c64"


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = b + 0x7FFF + ((b >> 16) & 1)
    return (b >> 16).astype(np.uint16)


def make_tensors(shape: ConvShape):
    """Draw (input NHWC, filter KRSC) for a shape.

    dtype "f32"  -> float32 arrays
    dtype "bf16" -> uint16 arrays holding bfloat16 bit patterns (rounded once, here)
    dtype "u8i8" -> uint8 input in 0..255, int8 filter in -127..127
    """
    rng = np.random.Generator(np.random.PCG64(shape.seed))
    ishape = (shape.N, shape.Hin, shape.Win, shape.C)
    fshape = (shape.K, shape.R, shape.S, shape.C)
    if shape.dtype == "u8i8":
        x = rng.integers(0, 256, size=ishape, dtype=np.uint8)
        w = rng.integers(-127, 128, size=fshape, dtype=np.int8)
        return x, w
    red = float(np.sqrt(shape.R * shape.S * (shape.c_logical or shape.C)))
    if shape.dist == "uniform":
        x = rng.uniform(-1.0, 1.0, size=ishape).astype(np.float32)
        w = rng.uniform(-1.0, 1.0, size=fshape).astype(np.float32)
    else:
        x = rng.standard_normal(size=ishape, dtype=np.float32)
        w = rng.standard_normal(size=fshape, dtype=np.float32) / np.float32(red)
        if shape.in_scale == "rsc":
            x = x / np.float32(red)
    if shape.c_logical:
        x[..., shape.c_logical:] = 0
        w[..., shape.c_logical:] = 0
    if shape.dtype == "bf16":
        return f32_to_bf16_bits(x), f32_to_bf16_bits(w)
    return x, w


def random_small_shape(rng: np.random.Generator, dtype: str = "f32", *, c_mult: int = 1,
                       max_hw: int = 9, max_ck: int = 5) -> ConvShape:
    """A random tiny shape (possibly with strides, dilation, asymmetric padding).

    Shapes whose padded input is smaller than the dilated kernel are re-drawn,
    so that every returned shape has at least one output pixel.
    """
    while True:
        R, S = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        DY, DX = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        PT, PL, PB, PR = (int(v) for v in rng.integers(0, 4, size=4))
        Hin, Win = int(rng.integers(1, max_hw + 1)), int(rng.integers(1, max_hw + 1))
        if Hin + PT + PB < DY * (R - 1) + 1 or Win + PL + PR < DX * (S - 1) + 1:
            continue
        return ConvShape(
            "rand", int(rng.integers(1, 3)), Hin, Win,
            int(rng.integers(1, max_ck + 1)) * c_mult, int(rng.integers(1, max_ck + 1)), R, S,
            SY=int(rng.integers(1, 4)), SX=int(rng.integers(1, 4)), DY=DY, DX=DX,
            PT=PT, PL=PL, PB=PB, PR=PR, dtype=dtype,
            zero_point=128 if dtype == "u8i8" else 0,
            seed=int(rng.integers(0, 2**31 - 1)), dist="uniform" if dtype == "f32" else "normal")
