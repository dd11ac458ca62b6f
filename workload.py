"""Seeded synthetic workloads: the five GPT-2-block configurations, their tiling
recipe and the input generator.

This module is shared by the tests, the benchmark and the smoke check.  It holds
no arithmetic of the method itself: only shapes, tile extents and random draws.
Neither the CPU oracle nor the HIP library imports it; callers hand its arrays
to both.

Notation follows the paper's section 3: N_e embedding size, N_s sequence length,
N_b batch size, N_h number of heads, h = N_e / N_h head size; N_m is the MLP
hidden width of the GPT-2 block.  Tensors are indexed in the paper's axis order
(activations N_e x N_s x N_b, attention embeddings h x N_s x N_b x N_h, linear
weights N_d x N_e).
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

SEED_BASE = 250413236 * 1000


@dataclasses.dataclass(frozen=True)
class BlockConfig:
    index: int          # 1..5, enters the seed
    name: str
    dtype: str          # "f32" | "bf16"  (storage type of activations / GEMM inputs)
    N_e: int
    N_h: int
    N_m: int
    N_s: int
    N_b: int
    tile: int
    adam: bool
    eps: float = 1e-5
    gelu: str = "tanh"

    @property
    def h(self) -> int:
        return self.N_e // self.N_h

    @property
    def T(self) -> int:
        return self.N_s * self.N_b

    def replace(self, **kw) -> "BlockConfig":
        return dataclasses.replace(self, **kw)


CONFIGS = {
    1: BlockConfig(1, "C1", "f32", 128, 2, 512, 64, 2, 32, True),
    2: BlockConfig(2, "C2", "f32", 768, 12, 3072, 1024, 8, 256, False),
    3: BlockConfig(3, "C3", "bf16", 1024, 16, 4096, 1024, 16, 512, True),
    4: BlockConfig(4, "C4", "bf16", 1600, 25, 6400, 1024, 8, 400, False),
    5: BlockConfig(5, "C5", "bf16", 8192, 64, 32768, 1024, 4, 1024, True),
}

# Adam constants used by every config that takes an optimiser step.
ADAM = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)

# index -> (name, kind); the index enters the per-tensor seed
TENSOR_INDEX = [
    ("X", "act"), ("dOut", "act"),
    ("W_qkv", "weight"), ("W_o", "weight"), ("W_1", "weight"), ("W_2", "weight"),
    ("b_qkv", "bias"), ("b_o", "bias"), ("b_1", "bias"), ("b_2", "bias"),
    ("gamma1", "gain"), ("beta1", "bias"), ("gamma2", "gain"), ("beta2", "bias"),
]

PARAM_NAMES = [n for n, k in TENSOR_INDEX if k != "act"]


def tensor_shapes(cfg: BlockConfig) -> dict:
    e, m, s, b = cfg.N_e, cfg.N_m, cfg.N_s, cfg.N_b
    return {
        "X": (e, s, b), "dOut": (e, s, b),
        "W_qkv": (3 * e, e), "W_o": (e, e), "W_1": (m, e), "W_2": (e, m),
        "b_qkv": (3 * e,), "b_o": (e,), "b_1": (m,), "b_2": (e,),
        "gamma1": (e,), "beta1": (e,), "gamma2": (e,), "beta2": (e,),
    }


def round_through_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array -> nearest bf16 (library conversion) -> fp32 array."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def generate(cfg: BlockConfig, names=None) -> dict:
    """Seed-generated fp32 arrays in logical axis order.

    Each tensor has its own Philox stream, drawn in first-axis-fastest order:
    weights and biases N(0, 0.02^2), layer-norm gains 1 + N(0, 0.02^2), block
    input and upstream gradient N(0, 1).  For bf16 configurations the block
    input, the upstream gradient are rounded to bf16-representable values (the
    parameters stay fp32 masters; their bf16 copies are made by the path itself).
    """
    shapes = tensor_shapes(cfg)
    out = {}
    for i, (name, kind) in enumerate(TENSOR_INDEX):
        if names is not None and name not in names:
            continue
        shape = shapes[name]
        n = int(np.prod(shape))
        rng = np.random.Generator(np.random.Philox(SEED_BASE + 100 * cfg.index + i))
        z = rng.standard_normal(n)
        if kind == "act":
            v = z
        elif kind == "gain":
            v = 1.0 + 0.02 * z
        else:
            v = 0.02 * z
        a = np.asarray(v, dtype=np.float32).reshape(shape, order="F")
        if cfg.dtype == "bf16" and kind == "act":
            a = round_through_bf16(a.reshape(-1, order="F")).reshape(shape, order="F")
        out[name] = a
    return out


def base_tiles(cfg: BlockConfig) -> dict:
    """Base tile extents per axis kind (edge tiles are smaller).

    Embedding-like axes (N_e, 3 N_e, N_m) and the sequence axis are cut every
    `tile` elements; the batch and head-count axes stay whole; the head-size
    axis stays whole unless it is longer than `tile`.
    """
    t = cfg.tile
    return dict(e=min(cfg.N_e, t), e3=min(3 * cfg.N_e, t), m=min(cfg.N_m, t),
                s=min(cfg.N_s, t), b=cfg.N_b, j=cfg.N_h, i=min(cfg.h, t))


def causal_tile_pairs(cfg: BlockConfig):
    """Sequence-tile pairs (key tile, query tile) that hold at least one
    unmasked score under the causal rule key <= query."""
    ts = base_tiles(cfg)["s"]
    g = math.ceil(cfg.N_s / ts)
    return [(kt, qt) for qt in range(g) for kt in range(g) if kt * ts <= min(cfg.N_s, (qt + 1) * ts) - 1]


def model_flops(cfg: BlockConfig, tile_skip: bool = True, visible_only: bool = False) -> float:
    """Forward+backward flops of one block: weight GEMMs 3 * 24 T N_e^2 and
    attention products 3 * 4 N_s^2 N_e N_b, the latter counted only on the
    sequence-tile pairs that are actually computed when `tile_skip`, or only on
    the (key, query) pairs the causal mask leaves visible when `visible_only`
    (the fused kernels skip masked work below tile granularity, and the flops of
    their recomputation are not credited either)."""
    ts = base_tiles(cfg)["s"]
    g = math.ceil(cfg.N_s / ts)
    ext = [min(ts, cfg.N_s - i * ts) for i in range(g)]
    if visible_only:
        pairs = cfg.N_s * (cfg.N_s + 1) // 2
    elif tile_skip:
        pairs = sum(ext[kt] * ext[qt] for kt, qt in causal_tile_pairs(cfg))
    else:
        pairs = cfg.N_s * cfg.N_s
    # QKV 3 N_e^2, out-projection N_e^2, fc1 and fc2 N_e N_m each (= 24 T N_e^2 when N_m = 4 N_e)
    weight = 2.0 * cfg.T * (4.0 * cfg.N_e ** 2 + 2.0 * cfg.N_e * cfg.N_m)
    attn = 4.0 * pairs * cfg.N_e * cfg.N_b
    return 3.0 * (weight + attn)
