"""Seeded synthetic inputs for the linear path: layer shapes of the model families
the paper serves (Section 5 "Experiment": Vicuna-7B / Llama-2-7B, Llama-3-8B; a
13B-shaped prefill chunk) and random weights / activations of those shapes.

This module holds no arithmetic of the method (no quantization, no products); it
serves both the CPU oracle's tests and the GPU path's tests, which otherwise share
nothing.  Everything is numpy on the host.
"""
import numpy as np

BASE_SEED = 250602006
GROUP = 128

# (K, N) of the four fused linears of one decoder layer.
LAYER_SHAPES = {
    "llama7b": {"qkv": (4096, 12288), "o": (4096, 4096), "gate_up": (4096, 22016), "down": (11008, 4096)},
    "llama3_8b": {"qkv": (4096, 6144), "o": (4096, 4096), "gate_up": (4096, 28672), "down": (14336, 4096)},
    "llama13b": {"qkv": (5120, 15360), "o": (5120, 5120), "gate_up": (5120, 27648), "down": (13824, 5120)},
}
LINEAR_ORDER = ("qkv", "o", "gate_up", "down")
_TENSOR_ID = {"x": 0, "qkv": 1, "o": 2, "gate_up": 3, "down": 4}


def rng_for(config_id: int, layer_id: int, tensor_id: int) -> np.random.Generator:
    return np.random.default_rng([BASE_SEED, int(config_id), int(layer_id), int(tensor_id)])


def activations(config_id: int, M: int, K: int, layer_id: int = 0, tensor_id: int = 0) -> np.ndarray:
    """x ~ N(0,1), drawn in fp32 and rounded to fp16.  [M,K] float16."""
    r = rng_for(config_id, layer_id, 100 + tensor_id)
    return r.standard_normal((M, K), dtype=np.float32).astype(np.float16)


def weights(config_id: int, K: int, N: int, layer_id: int = 0, tensor_id: int = 1,
            dist: str = "normal", std: float = 0.02) -> np.ndarray:
    """fp32 master weights [K,N]: N(0, std^2), or std * Student-t(nu=5) (heavy tails)."""
    r = rng_for(config_id, layer_id, tensor_id)
    if dist == "normal":
        w = r.standard_normal((K, N), dtype=np.float32)
        w *= np.float32(std)
        return w
    if dist == "student_t5":
        return (r.standard_t(5.0, size=(K, N)) * std).astype(np.float32)
    raise ValueError(dist)


def layer_weights(config_id: int, family: str, linear: str, layer_id: int = 0, dist: str = "normal") -> np.ndarray:
    K, N = LAYER_SHAPES[family][linear]
    return weights(config_id, K, N, layer_id, _TENSOR_ID[linear], dist)


def swapped_layers(n_layers: int, k: int, seed: int = BASE_SEED) -> np.ndarray:
    """Which layers hold the 4-bit variant when k of n_layers are swapped: the first
    k entries of one seeded permutation, so the sets are nested as k grows (the
    paper swaps layers one after another along a fixed sequence, Appendix A.2)."""
    perm = np.random.default_rng([seed, 5, 0, 999]).permutation(n_layers)
    return np.sort(perm[:k])


def w4_bytes(K: int, N: int, zeros: bool = True) -> int:
    """Bytes of one 4-bit layer record: packed codes + fp16 scales (+ packed zeros)."""
    b = K * N // 2 + (K // GROUP) * N * 2
    if zeros:
        b += (K // GROUP) * N // 2
    return b


def w8_bytes(K: int, N: int, zeros: bool = True) -> int:
    """Bytes of one 8-bit layer record: packed codes + fp16 scales (+ packed zeros)."""
    b = K * N + (K // GROUP) * N * 2
    if zeros:
        b += (K // GROUP) * N
    return b


def fp16_bytes(K: int, N: int) -> int:
    return 2 * K * N
