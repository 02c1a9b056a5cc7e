"""Seeded synthetic inputs and the benchmark layer shapes.

This module serves both the GPU path's tests/bench and the CPU oracle, and so
holds none of the convolution arithmetic: only layer shapes, a counter-based
random stream per tensor, and the bf16 <-> fp32 bit conversions needed to hand
both sides the same values.

The workloads stand in for the CNNs of the public benchmark suite the MXNet
paper times in its Section 4 ("Raw performance"): same layer shapes, random
values.  None of that suite's files are reproduced.
"""
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

SEED = 151201274
TENSOR_X, TENSOR_W, TENSOR_DY = 0, 1, 2


@dataclass(frozen=True)
class Layer:
    name: str
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int
    pad: int
    w_sigma: Optional[float]  # None -> He-normal sqrt(2/(C*R*S)); unused for uniform configs

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def flops_per_pass(self) -> int:
        return 2 * self.N * self.K * self.P * self.Q * self.C * self.R * self.S

    def dims(self) -> Tuple[int, ...]:
        return (self.N, self.C, self.H, self.W, self.K, self.R, self.S, self.stride, self.pad)

    def with_batch(self, n: int) -> "Layer":
        return Layer(self.name, n, self.C, self.H, self.W, self.K, self.R, self.S,
                     self.stride, self.pad, self.w_sigma)


@dataclass(frozen=True)
class Config:
    index: int          # position in the benchmark's config list
    name: str
    dtype: str          # "f32" or "bf16"
    dist: str           # "uniform" (x,w,dy ~ U[-1,1]) or "normal" (x,dy ~ N(0,1), w ~ N(0,sigma))
    layers: Tuple[Layer, ...]


def _L(name, N, C, HW, K, RS, stride, pad, sigma=None):
    return Layer(name, N, C, HW, HW, K, RS, RS, stride, pad, sigma)


CONFIGS: List[Config] = [
    Config(0, "single_f32", "f32", "uniform", (
        _L("conv", 2, 16, 16, 32, 3, 1, 1),)),
    Config(1, "alexnet_b128", "bf16", "normal", (
        _L("conv1", 128, 3, 224, 64, 11, 4, 2, 0.1),
        _L("conv2", 128, 64, 27, 192, 5, 1, 2, 0.1),
        _L("conv3", 128, 192, 13, 384, 3, 1, 1, 0.1),
        _L("conv4", 128, 384, 13, 256, 3, 1, 1, 0.1),
        _L("conv5", 128, 256, 13, 256, 3, 1, 1, 0.1))),
    Config(2, "inception3a_b128", "bf16", "normal", (
        _L("1x1_192_64", 128, 192, 28, 64, 1, 1, 0),
        _L("1x1_192_96", 128, 192, 28, 96, 1, 1, 0),
        _L("3x3_96_128", 128, 96, 28, 128, 3, 1, 1),
        _L("1x1_192_16", 128, 192, 28, 16, 1, 1, 0),
        _L("5x5_16_32", 128, 16, 28, 32, 5, 1, 2),
        _L("1x1_192_32_poolproj", 128, 192, 28, 32, 1, 1, 0))),
    Config(3, "vgg_a_b64", "bf16", "normal", (
        _L("conv1_1", 64, 3, 224, 64, 3, 1, 1),
        _L("conv2_1", 64, 64, 112, 128, 3, 1, 1),
        _L("conv3_1", 64, 128, 56, 256, 3, 1, 1),
        _L("conv3_2", 64, 256, 56, 256, 3, 1, 1),
        _L("conv4_1", 64, 256, 28, 512, 3, 1, 1),
        _L("conv4_2", 64, 512, 28, 512, 3, 1, 1),
        _L("conv5_1", 64, 512, 14, 512, 3, 1, 1),
        _L("conv5_2", 64, 512, 14, 512, 3, 1, 1))),
    Config(4, "resnet_bottleneck_b256", "bf16", "normal", (
        _L("1x1_256_64_56", 256, 256, 56, 64, 1, 1, 0),
        _L("3x3_64_64_56", 256, 64, 56, 64, 3, 1, 1),
        _L("1x1_64_256_56", 256, 64, 56, 256, 1, 1, 0),
        _L("1x1s2_256_512", 256, 256, 56, 512, 1, 2, 0),
        _L("1x1_512_128_28", 256, 512, 28, 128, 1, 1, 0),
        _L("3x3_128_128_28", 256, 128, 28, 128, 3, 1, 1),
        _L("1x1_128_512_28", 256, 128, 28, 512, 1, 1, 0))),
]


# Beyond the benchmark's five configurations: the FullyConnected head of the AlexNet-style network
# (1x1 "images": the layer is the convolution with H = W = R = S = 1), He-normal weights.
EXTRA_CONFIGS: List[Config] = [
    Config(5, "alexnet_head_b128", "bf16", "normal", (
        _L("fc6", 128, 9216, 1, 4096, 1, 1, 0),
        _L("fc7", 128, 4096, 1, 4096, 1, 1, 0),
        _L("fc8", 128, 4096, 1, 1000, 1, 1, 0))),
]


def _rebatched(cfg: Config, index: int, name: str, n: int) -> Config:
    return Config(index, name, cfg.dtype, cfg.dist, tuple(L.with_batch(n) for L in cfg.layers))


# The batch size of the paper's own single-GPU comparison (Section 4, "Raw performance": batch 32): the
# AlexNet- and VGG-style stacks once more at that size, drawn from the same random streams as the full-size
# configs (a fresh draw of the smaller size, not a prefix).
EXTRA_CONFIGS += [
    _rebatched(CONFIGS[1], 1, "alexnet_b32", 32),
    _rebatched(CONFIGS[3], 3, "vgg_a_b32", 32),
]


def config_by_name(name: str) -> Config:
    for c in CONFIGS + EXTRA_CONFIGS:
        if c.name == name:
            return c
    raise KeyError(name)


# ---- bf16 <-> fp32 bit conversions (input preparation only) ----------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array whose every value is exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


# ---- random streams ---------------------------------------------------------

def stream(config_idx: int, layer_idx: int, tensor_id: int) -> np.random.Generator:
    """Independent counter-based (Philox) stream per (config, layer, tensor)."""
    key = (SEED << 20) ^ (config_idx << 12) ^ (layer_idx << 4) ^ tensor_id
    return np.random.Generator(np.random.Philox(key=key))


def uniform_pm1(shape, gen: np.random.Generator) -> np.ndarray:
    return (gen.random(size=shape, dtype=np.float32) * np.float32(2.0) - np.float32(1.0))


def normal(shape, sigma: float, gen: np.random.Generator) -> np.ndarray:
    a = gen.standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        a *= np.float32(sigma)
    return a


def layer_inputs(cfg: Config, layer_idx: int, batch: Optional[int] = None,
                 tensors=("x", "w", "dy")):
    """Dict of float32 arrays in NCHW / KCRS order for one layer of a config.

    For bf16 configs every value is already rounded to bf16 (held in fp32), so
    the oracle and the GPU path consume identical numbers.  `batch` overrides N
    (the first `batch` samples are NOT a prefix of the full batch; they are a
    fresh draw of that size from the same stream)."""
    L = cfg.layers[layer_idx]
    if batch is not None:
        L = L.with_batch(batch)
    shapes = {"x": (L.N, L.C, L.H, L.W), "w": (L.K, L.C, L.R, L.S), "dy": (L.N, L.K, L.P, L.Q)}
    ids = {"x": TENSOR_X, "w": TENSOR_W, "dy": TENSOR_DY}
    out = {}
    for t in tensors:
        g = stream(cfg.index, layer_idx, ids[t])
        if cfg.dist == "uniform":
            a = uniform_pm1(shapes[t], g)
        elif t == "w":
            sigma = L.w_sigma if L.w_sigma is not None else float(np.sqrt(2.0 / (L.C * L.R * L.S)))
            a = normal(shapes[t], sigma, g)
        else:
            a = normal(shapes[t], 1.0, g)
        if cfg.dtype == "bf16":
            a = round_to_bf16(a)
        out[t] = a
    return L, out


def random_case(seed: int, N, C, H, W, K, R, S, stride, pad, dtype="f32", dist="uniform"):
    """x, w, dy for an ad-hoc shape (parity sweeps); same rules as layer_inputs."""
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    g = np.random.Generator(np.random.Philox(key=(SEED << 20) ^ (0xABC << 32) ^ seed))
    shapes = [(N, C, H, W), (K, C, R, S), (N, K, P, Q)]
    if dist == "uniform":
        arrs = [uniform_pm1(s, g) for s in shapes]
    else:
        arrs = [normal(shapes[0], 1.0, g), normal(shapes[1], float(np.sqrt(2.0 / (C * R * S))), g),
                normal(shapes[2], 1.0, g)]
    if dtype == "bf16":
        arrs = [round_to_bf16(a) for a in arrs]
    return arrs


# ---- host <-> device plumbing (torch is used for device memory only) ---------

def to_device(a_f32: np.ndarray, dtype: str):
    """float32 numpy (already bf16-exact when dtype == "bf16") -> contiguous GPU tensor of that dtype."""
    import torch
    if dtype == "bf16":
        bits = f32_to_bf16_bits(a_f32).view(np.int16)
        return torch.from_numpy(bits).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a_f32, dtype=np.float32)).cuda()


def to_host_f64(t) -> np.ndarray:
    """GPU tensor (fp32 or bf16) -> float64 numpy, exactly."""
    import torch
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return bf16_bits_to_f32(bits).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)
