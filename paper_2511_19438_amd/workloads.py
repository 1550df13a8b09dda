"""Seeded synthetic inputs for the W4A16 GPTQ matrix multiply (numpy only).

This module holds no arithmetic of the method: it only draws random tensors in the
storage format of the problem statement and names the layer shapes that are measured.
Both the CPU oracle's tests and the HIP path's tests feed on it; it imports neither.

Storage format (all row-major, contiguous):
  x        float16 [M, K]                 activations, ~N(0, 1)
  qweight  int32   [K/8, N]               eight 4-bit codes per word along K; every code uniform in 0..15
  qzeros   int32   [K/group, N/8]         eight 4-bit zero points per word along N; uniform in 0..15
  scales   float16 [K/group, N]           uniform in [0.001, 0.01]
  g_idx    int32   [K] or None            act-order: group of row k = perm[k] // group for a random permutation

The packed words are drawn directly as uniform 32-bit integers: each of their eight
nibbles is then an independent uniform code in 0..15, which is the stated distribution,
and no packing code is needed here.

The layer shapes stand in for the GPTQ checkpoints of the Llama family that the paper
serves (Opt4GPTQ, Section 4.1): same K, N and group size, random values.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np

GROUP_SIZE = 128


@dataclass(frozen=True)
class Shape:
    name: str
    K: int
    N: int


# Llama-7B-shaped linear layers (hidden 4096, intermediate 11008).
LLAMA_7B: List[Shape] = [
    Shape("qkv", 4096, 12288),
    Shape("o", 4096, 4096),
    Shape("gate_up", 4096, 22016),
    Shape("down", 11008, 4096),
]

# Llama-70B-shaped linear layers (hidden 8192, intermediate 28672, 8 KV heads).
LLAMA_70B: List[Shape] = [
    Shape("qkv", 8192, 10240),
    Shape("o", 8192, 8192),
    Shape("gate_up", 8192, 57344),
    Shape("down", 28672, 8192),
]

ACT_ORDER_SHAPE = Shape("act_order", 4096, 11008)

DECODE_BATCHES = (1, 2, 4, 8, 16)
MID_BATCHES = (32, 64, 128)
PREFILL_BATCHES = (512, 2048)


def case_seed(config: int, shape_index: int = 0) -> int:
    """Seed of a benchmark configuration: config 0 uses seed 0, the others 1000*config + index."""
    return 0 if config == 0 else 1000 * config + shape_index


def make_weights(K: int, N: int, group_size: int = GROUP_SIZE, seed: int = 0,
                 act_order: bool = False) -> Dict[str, Optional[np.ndarray]]:
    """Quantized weights of one layer: qweight, qzeros, scales and (act-order only) g_idx."""
    if K % 8 or N % 8 or K % group_size:
        raise ValueError("K and N must be multiples of 8 and K a multiple of group_size")
    rng = np.random.default_rng([seed, 1])
    groups = K // group_size
    qweight = rng.integers(0, 2 ** 32, size=(K // 8, N), dtype=np.uint32).view(np.int32)
    qzeros = rng.integers(0, 2 ** 32, size=(groups, N // 8), dtype=np.uint32).view(np.int32)
    scales = rng.uniform(0.001, 0.01, size=(groups, N)).astype(np.float16)
    g_idx = None
    if act_order:
        perm = rng.permutation(K)
        g_idx = (perm // group_size).astype(np.int32)
    return {"qweight": qweight, "qzeros": qzeros, "scales": scales, "g_idx": g_idx}


def make_activations(M: int, K: int, seed: int = 0) -> np.ndarray:
    """x ~ N(0, 1) rounded to float16, shape [M, K]."""
    rng = np.random.default_rng([seed, 2])
    return rng.standard_normal((M, K), dtype=np.float32).astype(np.float16)


def make_case(M: int, K: int, N: int, group_size: int = GROUP_SIZE, seed: int = 0,
              act_order: bool = False) -> Dict[str, Optional[np.ndarray]]:
    """One full problem instance: weights plus activations."""
    case = make_weights(K, N, group_size, seed, act_order)
    case["x"] = make_activations(M, K, seed)
    return case


def one_hot_activations(M: int, K: int, hot: List[int]) -> np.ndarray:
    """x[m, :] = unit vector e_{hot[m]} (float16)."""
    x = np.zeros((M, K), np.float16)
    for m in range(M):
        x[m, hot[m] % K] = 1.0
    return x


def ternary_activations(M: int, K: int, seed: int = 0) -> np.ndarray:
    """x with entries drawn from {-1, 0, +1} (float16)."""
    rng = np.random.default_rng([seed, 3])
    return rng.integers(-1, 2, size=(M, K)).astype(np.float16)


def sample_positions(M: int, N: int, count: int, seed: int = 0):
    """`count` output positions (m, n), uniformly drawn; int32 arrays."""
    rng = np.random.default_rng([seed, 4])
    m_idx = rng.integers(0, M, size=count).astype(np.int32)
    n_idx = rng.integers(0, N, size=count).astype(np.int32)
    return m_idx, n_idx
