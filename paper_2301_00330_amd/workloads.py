"""Layer tables and seeded synthetic inputs of the benchmark configurations.

This module serves both the CPU oracle's tests and the GPU path, so it holds
none of the method's arithmetic: only shapes and random draws.  The paper
trains on ImageNet / VOC / Cityscapes crops; those are not available, and the
backward path has no data-dependent control flow, so seeded tensors with the
layer shapes and value distributions below stand in for them.

Distributions: "N(0, s)" means standard deviation s.  Kaiming-normal weights
are N(0, sqrt(2 / fan_in)) with fan_in = (C_in / groups) * K_h * K_w.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List

import torch

SEED_BASE = 230100330


@dataclass(frozen=True)
class Layer:
    name: str
    C_in: int
    C_out: int
    H: int
    W: int
    K: int = 1
    stride: int = 1
    pad: int = 0
    dilation: int = 1
    groups: int = 1
    count: int = 1       # how many times the shape occurs in the network tail

    def out_hw(self):
        e = lambda v: (v + 2 * self.pad - self.dilation * (self.K - 1) - 1) // self.stride + 1
        return e(self.H), e(self.W)


@dataclass(frozen=True)
class Config:
    cfg_id: int
    name: str
    N: int
    layers: tuple
    dtypes: tuple        # subset of ("f32", "bf16")
    rs: tuple            # patch sizes
    x_dist: str          # "normal" | "relu"  (|N(0,1)|, a post-ReLU activation)
    w_dist: str          # "normal" | "kaiming"
    gy_std: float
    chain: tuple = ()    # layer indices, back to front, when the layers form a stack with nothing
                         # between them (stride 1, same map): they can hand each other reduced maps
    chain_clip: tuple = ()   # per layer: upper bound of the clipped ReLU that produced its input
                             # (6 for ReLU6), or 0 where no non-linearity precedes the layer


def _pw(name, ci, co, hw, count=1):
    return Layer(name, ci, co, hw, hw, count=count)


def _dw(name, c, hw, stride=1, count=1):
    return Layer(name, c, c, hw, hw, K=3, stride=stride, pad=1, groups=c, count=count)


def _c3(name, ci, co, hw, stride=1, dilation=1, count=1):
    return Layer(name, ci, co, hw, hw, K=3, stride=stride, pad=dilation, dilation=dilation, count=count)


CONFIGS = {
    1: Config(1, "single 3x3 conv", 1, (_c3("conv3x3_16", 16, 16, 16),), ("f32",), (2,), "normal", "normal", 1.0),
    2: Config(2, "MobileNetV2 inverted-residual block @56x56", 32,
              (_pw("expand_24_144", 24, 144, 56), _dw("dw_144", 144, 56), _pw("project_144_24", 144, 24, 56)),
              ("f32", "bf16"), (2, 4), "normal", "kaiming", 1e-2, chain=(2, 1, 0), chain_clip=(0.0, 6.0, 6.0)),
    3: Config(3, "ResNet-18 tail", 64,
              (_c3("conv_256_256@14", 256, 256, 14), _c3("conv_256_512_s2@14", 256, 512, 14, stride=2),
               _c3("conv_512_512@7", 512, 512, 7, count=3)),
              ("bf16",), (2, 4), "relu", "kaiming", 1.0),
    4: Config(4, "DeepLabV3 head @64x64", 8,
              (_pw("pw_2048_256", 2048, 256, 64), _c3("atrous_d12", 256, 256, 64, dilation=12),
               _c3("atrous_d24", 256, 256, 64, dilation=24), _c3("atrous_d36", 256, 256, 64, dilation=36)),
              ("bf16",), (2, 4, 8), "relu", "kaiming", 1e-3),
    5: Config(5, "MobileNetV2 tail (last conv layers, 14x14 and 7x7)", 128,
              (_pw("pw_320_1280@7", 320, 1280, 7), _pw("pw_960_320@7", 960, 320, 7),
               _dw("dw_960@7", 960, 7, count=3), _pw("pw_160_960@7", 160, 960, 7, count=3),
               _pw("pw_960_160@7", 960, 160, 7, count=2), _pw("pw_576_160@7", 576, 160, 7),
               _dw("dw_576_s2@14", 576, 14, stride=2), _pw("pw_96_576@14", 96, 576, 14),
               _pw("pw_576_96@14", 576, 96, 14), _dw("dw_576@14", 576, 14)),
              ("f32", "bf16"), (2,), "relu", "kaiming", 1e-2),
}

# The paper's own on-device test cases (Supp. E, Table 7): C -> C 3x3, stride 1,
# pad 1, batch 32, fp32, patch 2 and 4.  Table 7 lists width x height.
PAPER_CASES = Config(7, "on-device test cases of Table 7", 32,
                     tuple(Layer(f"T{i}_{c}@{h}x{w}", c, c, h, w, K=3, pad=1) for i, (c, w, h) in enumerate(
                         [(128, 120, 160), (256, 60, 80), (512, 30, 40), (512, 14, 14), (256, 14, 14),
                          (128, 28, 28), (64, 56, 56)])),
                     ("f32",), (2, 4), "relu", "kaiming", 1.0)
CONFIGS[7] = PAPER_CASES


def torch_dtype(name: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def layer_seed(cfg: Config, layer_index: int) -> int:
    return SEED_BASE + 1000 * cfg.cfg_id + layer_index


def make_inputs(cfg: Config, layer: Layer, dtype: str, N: int | None = None, seed: int | None = None):
    """Seeded CPU tensors (x, w, g_y) of one layer, already rounded to `dtype`."""
    N = cfg.N if N is None else N
    if seed is None:
        seed = layer_seed(cfg, cfg.layers.index(layer) if layer in cfg.layers else 0)
    g = torch.Generator(device="cpu").manual_seed(seed)
    Hy, Wy = layer.out_hw()
    x = torch.randn((N, layer.C_in, layer.H, layer.W), generator=g, dtype=torch.float32)
    if cfg.x_dist == "relu":
        x = x.abs_()
    cg = layer.C_in // layer.groups
    w = torch.randn((layer.C_out, cg, layer.K, layer.K), generator=g, dtype=torch.float32)
    if cfg.w_dist == "kaiming":
        w *= math.sqrt(2.0 / (cg * layer.K * layer.K))
    g_y = torch.randn((N, layer.C_out, Hy, Wy), generator=g, dtype=torch.float32) * cfg.gy_std
    td = torch_dtype(dtype)
    return x.to(td), w.to(td), g_y.to(td)


def integer_coded(shape, seed: int, lo: int = -8, hi: int = 8, dtype: str = "f32"):
    """Small integers as floats: every sum of a few thousand of them is exact in
    fp32, so results do not depend on summation order (bit-exact layout tests)."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    return torch.randint(lo, hi + 1, shape, generator=g).to(torch_dtype(dtype))


def all_layers(cfg: Config) -> List[Layer]:
    return list(cfg.layers)
