"""Seeded synthetic inputs shaped like the paper's BitNet b1.58 models.

This module only draws random inputs and names shapes.  It holds none of the
method's arithmetic (no quantization, no packing, no product): both the CPU
oracle's tests and the GPU path's tests/benchmarks consume the very same bits
produced here.

Shapes: Appendix A of arXiv 2410.16144 lists 12 dummy model configurations
(hidden size, intermediate size, layers); each decoder layer has 7 BitLinear
projections: Q, K, V, O (hidden -> hidden), gate and up (hidden -> ffn), down
(ffn -> hidden).  The benchmark configurations add three further layer shapes
("3B", "7B-bench", "100B-bench") that follow the same structure.
"""
from dataclasses import dataclass
from typing import List, Optional

import numpy as np

# (hidden_size, intermediate_size, num_hidden_layers) -- Appendix A, "Model Config".
PAPER_MODELS = {
    "125M": (768, 3072, 11),
    "350M": (1024, 3072, 24),
    "700M": (1536, 4096, 24),
    "1B": (2048, 3584, 24),
    "1.5B": (1536, 9216, 28),
    "2.5B": (2560, 6912, 30),
    "3.8B": (3840, 8192, 24),
    "7B": (4096, 12032, 32),
    "13B": (5120, 13824, 40),
    "30B": (6656, 16384, 60),
    "70B": (8192, 24576, 80),
    "100B": (8192, 45568, 72),
}

# num_attention_heads of the same 12 configurations (Appendix A); head size = hidden_size / heads.
PAPER_HEADS = {"125M": 12, "350M": 16, "700M": 16, "1B": 32, "1.5B": 32, "2.5B": 20, "3.8B": 32, "7B": 32,
               "13B": 40, "30B": 52, "70B": 64, "100B": 64}

# Layer shapes of the benchmark configurations (same 7-projection structure).
BENCH_MODELS = {
    "3B": (3200, 8640, 26),
    "7B-bench": (4096, 11008, 32),
    "100B-bench": (12288, 33792, 80),
}

PROJ_NAMES = ("q", "k", "v", "o", "gate", "up", "down")


@dataclass(frozen=True)
class Proj:
    name: str
    K: int  # input features
    N: int  # output features

    @property
    def packed_bytes(self) -> int:
        """Unpadded 2-bit size: the algorithmic bytes a GEMV must stream."""
        return self.N * self.K // 4


def layer_projections(hidden: int, ffn: int) -> List[Proj]:
    """The 7 BitLinear projections of one decoder layer, in execution order."""
    return [Proj("q", hidden, hidden), Proj("k", hidden, hidden), Proj("v", hidden, hidden),
            Proj("o", hidden, hidden), Proj("gate", hidden, ffn), Proj("up", hidden, ffn),
            Proj("down", ffn, hidden)]


def model_shape(name: str):
    if name in PAPER_MODELS:
        return PAPER_MODELS[name]
    return BENCH_MODELS[name]


def seed_for(config: int, layer: int = 0, matrix: int = 0) -> int:
    """Seed rule: config 1 uses seed 0; otherwise 1000*config + 10*layer + matrix."""
    if config == 1:
        return 0
    return 1000 * config + 10 * layer + matrix


def rng_for(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def ternary_weights(rng: np.random.Generator, N: int, K: int, p_zero: Optional[float] = None) -> np.ndarray:
    """[N,K] int8 in {-1,0,+1}.  p_zero=None: i.i.d. uniform over the three values;
    otherwise P(0)=p_zero and P(+1)=P(-1)=(1-p_zero)/2."""
    if p_zero is None:
        return rng.integers(-1, 2, size=(N, K), dtype=np.int8)
    u = rng.random((N, K), dtype=np.float32)
    half = np.float32((1.0 - p_zero) / 2.0)
    w = np.zeros((N, K), np.int8)
    w[u < half] = -1
    w[u >= np.float32(1.0) - half] = 1
    return w


def draw_w_scale(rng: np.random.Generator) -> np.float32:
    """A per-matrix fp32 scale standing in for an absmean: uniform in [0.01, 0.05]."""
    return np.float32(rng.uniform(0.01, 0.05))


def activations(rng: np.random.Generator, M: int, K: int, outlier_frac: float = 0.0,
                outlier_mult: float = 20.0) -> np.ndarray:
    """[M,K] fp32 ~ N(0,1); each element independently multiplied by outlier_mult
    with probability outlier_frac."""
    x = rng.standard_normal((M, K), dtype=np.float32)
    if outlier_frac > 0.0:
        mask = rng.random((M, K), dtype=np.float32) < np.float32(outlier_frac)
        x = np.where(mask, x * np.float32(outlier_mult), x).astype(np.float32)
    return x


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round-to-nearest-even.  Finite inputs only."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> fp32 (exact widening); for building test inputs only."""
    return (np.ascontiguousarray(h, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---- device-side generation for weights too large to stage on the host -------------

def ternary_weights_device(seed: int, N: int, K: int, device, p_zero: Optional[float] = None):
    """[N,K] int8 ternary tensor drawn on `device` with torch's generator (used when the
    matrix set is too large to draw on the host, e.g. the 100B-shape model)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    if p_zero is None:
        return torch.randint(-1, 2, (N, K), dtype=torch.int8, device=device, generator=g)
    u = torch.rand((N, K), dtype=torch.float32, device=device, generator=g)
    half = (1.0 - p_zero) / 2.0
    w = torch.zeros((N, K), dtype=torch.int8, device=device)
    w[u < half] = -1
    w[u >= 1.0 - half] = 1
    return w
