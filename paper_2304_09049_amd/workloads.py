"""Seeded synthetic inputs for the 2-bit lookup-table GEMM / convolution.

This module serves BOTH the CPU oracle's tests and the GPU path's tests and
benchmark, and therefore holds none of the method's arithmetic: it draws code
arrays, level tables and scales, and names the benchmark shapes.  It imports
neither the oracle nor the GPU binding.

The shapes stand in for convolution layers of ResNet18 / ResNet50 / VGG16 (the
paper measures trained 2-bit layers of such networks, Sec. 5.1); codes are
synthetic because neither the trained weights nor the image data exist here.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

# Level tables in code order 0..3.  Signed ("bipolar") weights and unsigned
# ("unipolar") activations, the two encodings Sec. 5.3 says the table handles alike.
LEVELS_W_SIGNED = (-2, -1, 0, 1)
LEVELS_A_UNSIGNED = (0, 1, 2, 3)


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str                      # "gemm" or "conv"
    M: int                         # output channels / weight rows
    N: int                         # output pixels x batch / activation rows
    K: int                         # reduction length
    # convolution geometry (kind == "conv")
    B: int = 0
    H: int = 0
    W: int = 0
    Cin: int = 0
    Cout: int = 0
    KH: int = 1
    KW: int = 1
    stride: Tuple[int, int] = (1, 1)
    pad: Tuple[int, int] = (0, 0)
    act_dist: str = "uniform"      # "uniform" or "relu_skew"
    levels: str = "fixed"          # "fixed" (signed w / unsigned a) or "random_int8"
    lut_entry: str = "i8"          # "i8" or "i16"
    scale: bool = False            # per-output-channel fp32 scale epilogue
    seed: int = 0

    @property
    def ops(self) -> int:
        return 2 * self.M * self.N * self.K

    @property
    def algorithmic_bytes(self) -> int:
        """Packed weights + packed activations (un-expanded input for conv) + output (+ scales)."""
        w = self.M * self.K // 4
        a = (self.B * self.H * self.W * self.Cin // 4) if self.kind == "conv" else self.N * self.K // 4
        out = 4 * self.M * self.N
        return w + a + out + (4 * self.M if self.scale else 0)


def _conv(name, B, H, W, Cin, Cout, KH, KW, stride, pad, **kw) -> Workload:
    OH = (H + 2 * pad[0] - KH) // stride[0] + 1
    OW = (W + 2 * pad[1] - KW) // stride[1] + 1
    return Workload(name=name, kind="conv", M=Cout, N=B * OH * OW, K=KH * KW * Cin, B=B, H=H, W=W,
                    Cin=Cin, Cout=Cout, KH=KH, KW=KW, stride=stride, pad=pad, **kw)


def gemm_large(N: int) -> Workload:
    """M = K = 8192 GEMM with seeded int8 levels in [-8, 7] and an int16 table, at a given N."""
    return Workload(name=f"gemm_8192x{N}x8192_i16", kind="gemm", M=8192, N=N, K=8192,
                    levels="random_int8", lut_entry="i16")


CONFIGS = {
    # configs[0]: single small GEMM
    "gemm_64x196x576": Workload(name="gemm_64x196x576", kind="gemm", M=64, N=196, K=576),
    # configs[1]: ResNet18-style 3x3, stride 1, pad 1, batch 1, 56x56x64 -> 64, fp32 scale epilogue
    "resnet18_conv3x3_b1": _conv("resnet18_conv3x3_b1", 1, 56, 56, 64, 64, 3, 3, (1, 1), (1, 1), scale=True),
    # configs[2]: ResNet50-style bottleneck 1x1, batch 32, 56x56x256 -> 64, post-ReLU-like skew
    "resnet50_conv1x1_b32": _conv("resnet50_conv1x1_b32", 32, 56, 56, 256, 64, 1, 1, (1, 1), (0, 0),
                                  act_dist="relu_skew"),
    # configs[3]: VGG16-style 3x3, stride 1, pad 1, batch 16, 56x56x256 -> 256
    "vgg16_conv3x3_b16": _conv("vgg16_conv3x3_b16", 16, 56, 56, 256, 256, 3, 3, (1, 1), (1, 1)),
    # configs[4]: large GEMM, non-uniform int16 table, N swept
    "gemm_8192x1x8192_i16": gemm_large(1),
    "gemm_8192x16x8192_i16": gemm_large(16),
    "gemm_8192x256x8192_i16": gemm_large(256),
    "gemm_8192x8192x8192_i16": gemm_large(8192),
}

# the workload bench.py's headline line is quoted on: the largest ResNet-shaped layer of the set (the batch-1 3x3 layer
# is a 3.5 us kernel whose time is mostly launch latency)
HEADLINE = "resnet50_conv1x1_b32"


@dataclass
class Inputs:
    workload: Workload
    levels_w: np.ndarray           # int8[4]
    levels_a: np.ndarray           # int8[4]
    Wc: np.ndarray                 # uint8 codes, [M][K] or [Cout][KH][KW][Cin]
    Ac: np.ndarray                 # uint8 codes, [N][K] or [B][H][W][Cin]
    scale: Optional[np.ndarray] = field(default=None)   # float32[M] or None


def draw_codes(rng: np.random.Generator, shape, dist: str = "uniform", nlev: int = 4) -> np.ndarray:
    """Codes in 0..nlev-1 (nlev = 4: the paper's 2-bit codes; 8, 16: its 3- and 4-bit extension).
    "uniform": every code equally likely.  "relu_skew" (2-bit only): code 0 with probability 1/2, codes 1..3 with 1/6 each."""
    if dist == "uniform":
        return rng.integers(0, nlev, size=shape, dtype=np.uint8)
    if dist == "relu_skew":
        r = rng.integers(0, 6, size=shape, dtype=np.uint8)   # 0,1,2 -> code 0; 3,4,5 -> codes 1,2,3
        return np.where(r < 3, 0, r - 2).astype(np.uint8)
    raise ValueError(f"unknown code distribution {dist!r}")


def draw_levels(rng: np.random.Generator, kind: str):
    if kind == "fixed":
        return (np.array(LEVELS_W_SIGNED, dtype=np.int8), np.array(LEVELS_A_UNSIGNED, dtype=np.int8))
    if kind == "random_int8":
        # 4 + 4 independent uniform integers in [-8, 7]; duplicates allowed
        lw = rng.integers(-8, 8, size=4).astype(np.int8)
        la = rng.integers(-8, 8, size=4).astype(np.int8)
        return lw, la
    raise ValueError(f"unknown level recipe {kind!r}")


def make_inputs(w: Workload, seed: Optional[int] = None) -> Inputs:
    """Draw every array of one workload from one generator seeded with ``seed`` (default: the workload's)."""
    rng = np.random.default_rng(w.seed if seed is None else seed)
    lw, la = draw_levels(rng, w.levels)
    if w.kind == "gemm":
        Wc = draw_codes(rng, (w.M, w.K))
        Ac = draw_codes(rng, (w.N, w.K), w.act_dist)
    else:
        Wc = draw_codes(rng, (w.Cout, w.KH, w.KW, w.Cin))
        Ac = draw_codes(rng, (w.B, w.H, w.W, w.Cin), w.act_dist)
    scale = rng.uniform(0.01, 0.1, size=w.M).astype(np.float32) if w.scale else None
    return Inputs(workload=w, levels_w=lw, levels_a=la, Wc=Wc, Ac=Ac, scale=scale)


def small_gemm(M: int, N: int, K: int, seed: int = 0, levels: str = "fixed", dist: str = "uniform") -> Inputs:
    """An ad-hoc GEMM case for tests."""
    return make_inputs(Workload(name=f"gemm_{M}x{N}x{K}", kind="gemm", M=M, N=N, K=K, levels=levels,
                                act_dist=dist, seed=seed))


def small_conv(B, H, W, Cin, Cout, KH, KW, stride=(1, 1), pad=(0, 0), seed: int = 0,
               levels: str = "fixed", scale: bool = False) -> Inputs:
    """An ad-hoc convolution case for tests."""
    return make_inputs(_conv(f"conv_{B}x{H}x{W}x{Cin}_{Cout}_{KH}x{KW}", B, H, W, Cin, Cout, KH, KW,
                             tuple(stride), tuple(pad), seed=seed, levels=levels, scale=scale))
