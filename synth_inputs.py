"""Seeded synthetic inputs for the fine-grained W4A8 linear layer.

This module only draws random tensors and lists workload shapes.  It holds
none of the method's arithmetic (no quantisation, no scales, no GEMM), so the
CPU oracle and the HIP path can both be fed from it without sharing any code
that is under test.

The tensors stand in for the LLaMA-2 / LLaMA-3 / Mixtral linear layers the
paper evaluates (Sec. 5.1): the shapes are those models' projection shapes,
the values follow the usual initialisation scale of such layers plus the
activation-outlier channels that motivate per-token / group-wise quantisation.
Everything is drawn with numpy's PCG64 and cast to fp16 once; both sides get
the same fp16 arrays.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Tuple

import numpy as np

BASE_SEED = 20240514
GROUP = 128           # group size along K used in every experiment (Sec. 5.1)
ALPHA_LOG2 = 10       # default amplifier 2^10 (Sec. 4.1)


def seed_for(config: int, shape_index: int, stream: int = 0) -> int:
    """One seed per (config, shape, tensor stream)."""
    return BASE_SEED + 1000 * config + shape_index + 100003 * stream


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def activations_outlier(M: int, K: int, seed: int, outlier_frac: float = 0.01,
                        outlier_gain: float = 20.0) -> np.ndarray:
    """fp16 [M,K] ~ N(0,1); floor(outlier_frac*K) channels (same for all rows) are scaled by outlier_gain."""
    rng = _rng(seed)
    x = rng.standard_normal((M, K), dtype=np.float32)
    n_out = int(np.floor(outlier_frac * K))
    if n_out > 0:
        cols = rng.permutation(K)[:n_out]
        x[:, cols] *= np.float32(outlier_gain)
    return x.astype(np.float16)


def activations_student_t(M: int, K: int, seed: int, nu: float = 3.0) -> np.ndarray:
    """fp16 [M,K] heavy-tailed activations: Student-t with nu degrees of freedom (clipped to fp16 range)."""
    rng = _rng(seed)
    x = rng.standard_t(nu, size=(M, K)).astype(np.float32)
    np.clip(x, -60000.0, 60000.0, out=x)
    return x.astype(np.float16)


def weights_gaussian(N: int, K: int, seed: int, sigma: float = 0.02, outlier_col_frac: float = 0.0,
                     outlier_gain: float = 8.0) -> np.ndarray:
    """fp16 [N,K] (out-features x in-features) ~ N(0, sigma); optional outlier input-channel columns."""
    rng = _rng(seed)
    w = rng.standard_normal((N, K), dtype=np.float32)
    w *= np.float32(sigma)
    n_out = int(np.floor(outlier_col_frac * K))
    if n_out > 0:
        cols = _rng(seed + 7919).permutation(K)[:n_out]
        w[:, cols] *= np.float32(outlier_gain)
    return w.astype(np.float16)


def moe_routing(tokens: int, experts: int, topk: int, seed: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Uniform-random top-k router.

    Returns (token_of_row int32 [tokens*topk], expert_of_row int32 [tokens*topk], row_offsets int32 [experts+1]);
    rows are sorted by expert (stable in token order).
    """
    rng = _rng(seed)
    choice = np.empty((tokens, topk), dtype=np.int32)
    for t in range(tokens):
        choice[t] = rng.permutation(experts)[:topk]
    token = np.repeat(np.arange(tokens, dtype=np.int32), topk)
    expert = choice.reshape(-1)
    order = np.argsort(expert, kind="stable")
    counts = np.bincount(expert, minlength=experts)
    offsets = np.zeros(experts + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    return token[order].astype(np.int32), expert[order].astype(np.int32), offsets


@dataclasses.dataclass(frozen=True)
class Shape:
    name: str
    M: int
    K: int
    N: int


# Linear-layer shapes (K -> N) of the model families the paper measures.
LLAMA2_7B = {"qkv": (4096, 12288), "o_proj": (4096, 4096), "gate_up": (4096, 22016), "down": (11008, 4096)}
LLAMA2_70B = {"qkv": (8192, 10240), "o_proj": (8192, 8192), "gate": (8192, 28672), "up": (8192, 28672),
              "down": (28672, 8192)}
LLAMA3_8B = {"qkv": (4096, 6144), "gate_up": (4096, 28672), "down": (14336, 4096)}
MIXTRAL_8X7B = {"w1": (4096, 14336), "w3": (4096, 14336), "w2": (14336, 4096)}


def config_shapes(config: int) -> List[Shape]:
    """GEMM shapes of each benchmark configuration (index = position in the configuration list)."""
    if config == 0:
        return [Shape("dense4096", 8, 4096, 4096)]
    if config == 1:
        return [Shape(f"{n}_M{m}", m, k, nn) for m in (1, 16, 64) for n, (k, nn) in LLAMA2_7B.items()]
    if config == 2:
        return [Shape(f"{n}_M{m}", m, k, nn) for m in (1, 32, 2048) for n, (k, nn) in LLAMA2_70B.items()
                if n != "up"]
    if config == 3:
        return [Shape(f"{n}_M4096", 4096, k, nn) for n, (k, nn) in LLAMA3_8B.items()]
    if config == 4:
        return [Shape(f"{n}_E8", 1024, k, nn) for n, (k, nn) in MIXTRAL_8X7B.items()]
    raise ValueError(f"unknown config {config}")


def make_activations(config: int, M: int, K: int, seed: int) -> np.ndarray:
    if config == 3:
        return activations_student_t(M, K, seed)
    return activations_outlier(M, K, seed)


def make_weights(config: int, N: int, K: int, seed: int) -> np.ndarray:
    if config == 1:
        return weights_gaussian(N, K, seed, outlier_col_frac=0.005, outlier_gain=8.0)
    return weights_gaussian(N, K, seed)


def algorithmic_bytes(M: int, N: int, K: int, group: int = GROUP, scale_bytes: int = 4) -> int:
    """Bytes the layer must move once: packed int4 weights, group scales, int8 activations, fp16 output, row/col scales."""
    return N * K // 2 + N * (K // group) * scale_bytes + M * K + 2 * M * N + 4 * M + 4 * N


def algorithmic_ops(M: int, N: int, K: int) -> int:
    """int8 multiply and add operations of the contraction (2 per MAC)."""
    return 2 * M * N * K


def shapes_summary() -> Dict[int, List[Shape]]:
    return {c: config_shapes(c) for c in range(5)}
