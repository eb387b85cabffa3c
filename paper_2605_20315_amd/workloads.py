"""Seeded synthetic inputs shaped like the prefill linear layers the paper accelerates.

The paper measures prefill of Qwen3-8B / Qwen3.5-9B class models (Section 4, Fig. 3); those
models and prompts are not available here, so these tensors stand in for them: token-major
BF16 activations with a few large "outlier" channels, and Gaussian weights, at the shapes of
Llama-3-8B-class and 32B-class linear layers.

This module holds no arithmetic of the quantization method itself: it only draws random
numbers and rounds them to BF16.  Both the CPU oracle's tests and the HIP path's tests and
benchmark take their inputs from here, so that they see identical bits.

Determinism: a tensor is generated in chunks of ``CHUNK_ROWS`` rows; chunk ``c`` of tensor
``t`` of layer ``l`` of config ``cfg`` uses ``numpy.random.default_rng([seed, cfg, l, t, c])``.
Chunks are independent, so they can be produced by several threads and the result does not
depend on the thread count.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

CHUNK_ROWS = 1024
_T_ACT, _T_WEIGHT, _T_COLS = 0, 1, 2


@dataclass(frozen=True)
class Layer:
    name: str
    K: int  # contraction (input features)
    N: int  # output features


@dataclass(frozen=True)
class Config:
    cfg_id: int
    name: str
    M: int
    layers: Tuple[Layer, ...]
    outlier_frac: float      # fraction of channels that are outliers (0 => fixed count below)
    outlier_count: int       # used when outlier_frac == 0
    outlier_gain: float
    weight_std: float        # 0 => K ** -0.5
    token_lognormal: bool    # per-token magnitude exp(N(0,1))
    student_t_down: bool     # Student-t(4) input for the "down" layer


LLAMA8B = (Layer("qkv", 4096, 6144), Layer("o", 4096, 4096),
           Layer("gate_up", 4096, 28672), Layer("down", 14336, 4096))
DENSE32B = (Layer("qkv", 5120, 7168), Layer("o", 5120, 5120),
            Layer("gate_up", 5120, 51200), Layer("down", 25600, 5120))


def ragged_lengths(seed: int = 0) -> np.ndarray:
    """24 sequence lengths uniform in [512, 8192] for the ragged multi-turn batch."""
    return np.random.default_rng(seed).integers(512, 8193, 24)


def configs(seed: int = 0) -> List[Config]:
    m5 = int(ragged_lengths(seed).sum())
    return [
        Config(0, "tiny", 256, (Layer("linear", 1024, 1024),), 0.0, 4, 20.0, 0.02, False, False),
        Config(1, "llama8b_m2048", 2048, LLAMA8B, 1e-3, 0, 20.0, 0.0, False, True),
        Config(2, "llama8b_m8192", 8192, LLAMA8B, 1e-3, 0, 20.0, 0.0, False, True),
        Config(3, "dense32b_m16384", 16384, DENSE32B, 1e-3, 0, 50.0, 0.0, True, False),
        Config(4, "ragged_llama8b", m5, (LLAMA8B[2], LLAMA8B[3]), 1e-3, 0, 20.0, 0.0, False, False),
    ]


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round binary32 to BF16 (nearest even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (h.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def outlier_columns(cfg: Config, layer_idx: int, seed: int = 0) -> np.ndarray:
    K = cfg.layers[layer_idx].K
    n = cfg.outlier_count if cfg.outlier_frac == 0 else int(round(cfg.outlier_frac * K))
    rng = np.random.default_rng([seed, cfg.cfg_id, layer_idx, _T_COLS])
    return np.sort(rng.choice(K, n, replace=False))


def _chunks(rows: int):
    return [(c, c * CHUNK_ROWS, min(rows, (c + 1) * CHUNK_ROWS))
            for c in range((rows + CHUNK_ROWS - 1) // CHUNK_ROWS)]


def activation(cfg: Config, layer_idx: int, seed: int = 0) -> np.ndarray:
    """X [M, K] as BF16 bit patterns (uint16)."""
    layer = cfg.layers[layer_idx]
    K = layer.K
    cols = outlier_columns(cfg, layer_idx, seed)
    heavy = cfg.student_t_down and layer.name == "down"
    out = np.empty((cfg.M, K), dtype=np.uint16)

    def work(job):
        c, r0, r1 = job
        rng = np.random.default_rng([seed, cfg.cfg_id, layer_idx, _T_ACT, c])
        n = r1 - r0
        if cfg.token_lognormal:
            mag = np.exp(rng.standard_normal(n)).astype(np.float32)
        if heavy:
            x = rng.standard_t(4, size=(n, K)).astype(np.float32)
        else:
            x = rng.standard_normal((n, K), dtype=np.float32)
        if cfg.token_lognormal:
            x *= mag[:, None]
        x[:, cols] *= np.float32(cfg.outlier_gain)
        out[r0:r1] = f32_to_bf16_bits(x)

    with ThreadPoolExecutor(_workers()) as ex:
        list(ex.map(work, _chunks(cfg.M)))
    return out


def weight(cfg: Config, layer_idx: int, seed: int = 0) -> np.ndarray:
    """W [N, K] as BF16 bit patterns (uint16); std 0.02 for the tiny config, else K**-0.5."""
    layer = cfg.layers[layer_idx]
    std = np.float32(cfg.weight_std if cfg.weight_std > 0 else layer.K ** -0.5)
    out = np.empty((layer.N, layer.K), dtype=np.uint16)

    def work(job):
        c, r0, r1 = job
        rng = np.random.default_rng([seed, cfg.cfg_id, layer_idx, _T_WEIGHT, c])
        w = rng.standard_normal((r1 - r0, layer.K), dtype=np.float32)
        w *= std
        out[r0:r1] = f32_to_bf16_bits(w)

    with ThreadPoolExecutor(_workers()) as ex:
        list(ex.map(work, _chunks(layer.N)))
    return out


def layer_flops(M: int, layer: Layer) -> float:
    return 2.0 * M * layer.N * layer.K
