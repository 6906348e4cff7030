"""Generators for the five benchmark configurations (all seeded, all synthetic).

Pattern table.  Bit (3*r + s) of a mask is tap (r, s) of the 3x3 kernel.
IDs 0-3 are the four Sparse Convolution Patterns of the paper's SCP-design
section (centre + three of the four edge neighbours); IDs 4-11 are extra 4-tap
masks that contain the centre, standing in for the "random patterns with 4
non-zero elements" of the pattern-count experiment (Tables 1-2).
"""
from __future__ import annotations

import dataclasses
from typing import List

import numpy as np

PATTERN_TABLE = np.array(
    [0x03A, 0x09A, 0x0B8, 0x0B2,          # the four SCPs
     0x01B, 0x036, 0x0D8, 0x1B0,          # 2x2 blocks containing the centre
     0x113, 0x074, 0x191, 0x05C],         # centre + diagonal pair + one edge tap
    dtype=np.uint16)
DENSE_MASK = np.uint16(0x1FF)


def base_seed(config_index: int) -> int:
    return 190905073 * 10 + int(config_index)


@dataclasses.dataclass(frozen=True)
class LayerSpec:
    name: str
    n: int
    c_in: int
    c_out: int
    h: int
    w: int
    stride: int = 1
    pad: int = 1
    dtype: str = "f32"            # "f32" | "bf16"
    num_patterns: int = 8
    pattern_dist: str = "zipf"    # "uniform" | "zipf" | "dense"
    keep_div: float = 3.6         # connectivity compression k: keep 1/k of the kernels
    count_dist: str = "pm30"      # "bernoulli" | "pm30" | "geometric" | "all"
    relu: bool = True
    pool_after: bool = False      # 2x2 max-pool follows this layer (VGG block end)

    @property
    def h_out(self) -> int:
        return (self.h + 2 * self.pad - 3) // self.stride + 1

    @property
    def w_out(self) -> int:
        return (self.w + 2 * self.pad - 3) // self.stride + 1


def vgg16_conv_shapes():
    """(c_in, c_out, spatial, pool_after) of VGG-16's 13 conv layers at 224x224."""
    return [(3, 64, 224, False), (64, 64, 224, True),
            (64, 128, 112, False), (128, 128, 112, True),
            (128, 256, 56, False), (256, 256, 56, False), (256, 256, 56, True),
            (256, 512, 28, False), (512, 512, 28, False), (512, 512, 28, True),
            (512, 512, 14, False), (512, 512, 14, False), (512, 512, 14, True)]


def resnet50_conv3x3_shapes():
    """(c, spatial_in, stride) of ResNet-50's sixteen 3x3 convs (stride on the 3x3)."""
    out = []
    out += [(64, 56, 1)] * 3
    out += [(128, 56, 2)] + [(128, 28, 1)] * 3
    out += [(256, 28, 2)] + [(256, 14, 1)] * 5
    out += [(512, 14, 2)] + [(512, 7, 1)] * 2
    return out


def config_layers(config_index: int, batch: int | None = None) -> List[LayerSpec]:
    """Layer list of benchmark configuration 1..5."""
    if config_index == 1:
        return [LayerSpec("c1_16x16", batch or 1, 16, 16, 16, 16, num_patterns=8,
                          pattern_dist="uniform", keep_div=2.0, count_dist="bernoulli",
                          relu=False)]
    if config_index == 2:
        return [LayerSpec("c2_vgg256_56", batch or 1, 256, 256, 56, 56, relu=False)]
    if config_index == 3:
        layers = []
        for i, (ci, co, s, pool) in enumerate(vgg16_conv_shapes()):
            if i == 0:
                layers.append(LayerSpec(f"vgg_conv{i+1}", batch or 1, ci, co, s, s,
                                        num_patterns=1, pattern_dist="dense",
                                        keep_div=1.0, count_dist="all", pool_after=pool))
            else:
                layers.append(LayerSpec(f"vgg_conv{i+1}", batch or 1, ci, co, s, s,
                                        pool_after=pool))
        return layers
    if config_index == 4:
        return [LayerSpec(f"rn50_3x3_{i+1}_c{c}_s{st}", batch or 32, c, c, sp, sp,
                          stride=st, dtype="bf16", keep_div=2.5)
                for i, (c, sp, st) in enumerate(resnet50_conv3x3_shapes())]
    if config_index == 5:
        return [LayerSpec("c5_stress512_28", batch or 64, 512, 512, 28, 28,
                          num_patterns=12, pattern_dist="uniform", keep_div=8.0,
                          count_dist="geometric", relu=False)]
    raise ValueError("config_index must be 1..5")


def _kept_counts(spec: LayerSpec, rng: np.random.Generator) -> np.ndarray:
    f, c = spec.c_out, spec.c_in
    m = c / spec.keep_div
    if spec.count_dist == "all":
        return np.full(f, c, dtype=np.int64)
    if spec.count_dist == "pm30":
        u = rng.uniform(-0.3, 0.3, size=f)
        return np.clip(np.rint(m * (1.0 + u)), 0, c).astype(np.int64)
    if spec.count_dist == "geometric":
        return np.minimum(c, rng.geometric(1.0 / m, size=f)).astype(np.int64)
    raise ValueError(spec.count_dist)


def make_layer(spec: LayerSpec, seed: int) -> dict:
    """Draw dense weights, per-kernel pattern ids, connectivity, table and bias.

    Draw order (fixed): weights, bias, pattern ids, connectivity.
    """
    rng = np.random.default_rng(seed)
    f, c = spec.c_out, spec.c_in
    sigma = np.sqrt(2.0 / (9.0 * c))
    w = (rng.standard_normal((f, c, 3, 3)) * sigma).astype(np.float32)
    bias = (rng.standard_normal(f) * 0.1).astype(np.float32)
    if spec.pattern_dist == "dense":
        table = np.array([DENSE_MASK], dtype=np.uint16)
        pid = np.zeros((f, c), dtype=np.uint8)
    else:
        p = spec.num_patterns
        table = PATTERN_TABLE[:p].copy()
        if spec.pattern_dist == "uniform":
            prob = np.full(p, 1.0 / p)
        elif spec.pattern_dist == "zipf":
            prob = 1.0 / np.arange(1, p + 1)
            prob /= prob.sum()
        else:
            raise ValueError(spec.pattern_dist)
        pid = rng.choice(p, size=(f, c), p=prob).astype(np.uint8)
    if spec.count_dist == "bernoulli":
        conn = (rng.random((f, c)) < 1.0 / spec.keep_div).astype(np.uint8)
    else:
        counts = _kept_counts(spec, rng)
        conn = np.zeros((f, c), dtype=np.uint8)
        for i in range(f):
            conn[i, rng.choice(c, size=int(counts[i]), replace=False)] = 1
    return dict(w=w, bias=bias, pattern_id=pid, conn=conn, table=table)


def to_bf16_values(x: np.ndarray) -> np.ndarray:
    """Round fp32 data to the nearest bf16-representable values (kept as fp32).

    Uses PyTorch's CPU cast as the library primitive, so that bf16 activations
    handed to both the oracle and the HIP path are the very same numbers.
    """
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def make_input(spec: LayerSpec, seed: int, layout: str = "nchw") -> np.ndarray:
    """Activations max(N(0,1), 0) of shape NCHW (or NHWC), fp32 (bf16-valued for bf16)."""
    rng = np.random.default_rng(seed + 7919)
    x = rng.standard_normal((spec.n, spec.c_in, spec.h, spec.w), dtype=np.float32)
    np.maximum(x, 0.0, out=x)
    if spec.dtype == "bf16":
        x = to_bf16_values(x)
    if layout == "nhwc":
        x = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
    return x


def nnz_of_layer(layer: dict) -> int:
    """Number of stored (non-pruned) weights: sum over kept kernels of popcount(mask)."""
    pop = np.array([bin(int(m)).count("1") for m in layer["table"]], dtype=np.int64)
    return int((pop[layer["pattern_id"]] * (layer["conn"] != 0)).sum())
