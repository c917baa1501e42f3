"""Seeded synthetic inputs for the quantized linear layer.

This module only draws random numbers and lists layer shapes.  It holds none of
the method's arithmetic (no quantizer, no contraction) and imports neither the
HIP binding nor the oracle, so both sides can take their inputs from it.

The layer shapes are the public dimensions of the three models the paper
evaluates (Section 6: Qwen2-1.5B, Qwen2-7B, Llama-3-8B; Table 1 lists the
Qwen2-7B dimensions).  The checkpoints themselves are not available, so weights
are N(0, 0.02) and activations N(0, 1) with a few outlier channels.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

GROUP = 64  # quantization group length along K

# name -> (N, K) for one transformer block, plus how many blocks the model has.
MODELS = {
    "qwen2-1.5b": {
        "blocks": 28,
        "layers": {
            "q": (1536, 1536), "k": (256, 1536), "v": (256, 1536), "o": (1536, 1536),
            "gate": (8960, 1536), "up": (8960, 1536), "down": (1536, 8960),
        },
        "lm_head": None,
        "prefill_m": 512,
    },
    "qwen2-7b": {
        "blocks": 28,
        "layers": {
            "q": (3584, 3584), "k": (512, 3584), "v": (512, 3584), "o": (3584, 3584),
            "gate": (18944, 3584), "up": (18944, 3584), "down": (3584, 18944),
        },
        "lm_head": (152064, 3584),
        "prefill_m": 1024,
    },
    "llama3-8b": {
        "blocks": 32,
        "layers": {
            "q": (4096, 4096), "k": (1024, 4096), "v": (1024, 4096), "o": (4096, 4096),
            "gate": (14336, 4096), "up": (14336, 4096), "down": (4096, 14336),
        },
        "lm_head": None,
        "prefill_m": 2048,
    },
}

_PROJ_INDEX = {"q": 0, "k": 1, "v": 2, "o": 3, "gate": 4, "up": 5, "down": 6, "lm_head": 7}
_MODEL_INDEX = {"qwen2-1.5b": 1, "qwen2-7b": 2, "llama3-8b": 3}

_ROWS_PER_CHUNK = 512


def layer_seed(model: str, block: int, proj: str) -> int:
    """Deterministic seed of one projection matrix of one block."""
    return 1_000_003 * _MODEL_INDEX[model] + 101 * block + _PROJ_INDEX[proj] + 1


def _n_threads() -> int:
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        n = os.cpu_count() or 1
    return max(1, min(16, n))


def weights(N: int, K: int, seed: int, std: float = 0.02) -> np.ndarray:
    """fp32 [N, K] ~ N(0, std).  Rows are drawn in chunks of 512, chunk c from
    ``default_rng([seed, c])``, so large matrices can be filled by several
    threads and still depend only on (N, K, seed)."""
    out = np.empty((N, K), dtype=np.float32)
    n_chunks = (N + _ROWS_PER_CHUNK - 1) // _ROWS_PER_CHUNK

    def fill(c: int) -> None:
        r0 = c * _ROWS_PER_CHUNK
        r1 = min(N, r0 + _ROWS_PER_CHUNK)
        rng = np.random.default_rng([seed, c])
        rng.standard_normal(out=out[r0:r1], dtype=np.float32)
        out[r0:r1] *= np.float32(std)

    if n_chunks == 1:
        fill(0)
    else:
        with ThreadPoolExecutor(_n_threads()) as pool:
            list(pool.map(fill, range(n_chunks)))
    return out


def outlier_channels(K: int, seed: int) -> np.ndarray:
    """Indices of the 0.1 % of K-channels that carry outliers (at least one)."""
    n_out = max(1, int(round(0.001 * K)))
    rng = np.random.default_rng([seed, 0x0A7])
    return np.sort(rng.choice(K, size=n_out, replace=False))


def activations(M: int, K: int, seed: int, outliers: bool = True) -> np.ndarray:
    """fp32 [M, K] ~ N(0, 1); with ``outliers`` the same 0.1 % of channels of
    every token are multiplied by 20."""
    rng = np.random.default_rng([seed, 0xAC7])
    x = rng.standard_normal((M, K), dtype=np.float32)
    if outliers:
        x[:, outlier_channels(K, seed)] *= np.float32(20.0)
    return x


def activations_f16(M: int, K: int, seed: int, outliers: bool = False) -> np.ndarray:
    """fp16 [M, K]: the fp32 draw of :func:`activations` stored as IEEE half
    (round to nearest even), i.e. what a caller with fp16 activations holds."""
    return activations(M, K, seed, outliers).astype(np.float16)


def config1():
    """Single decode layer of the first benchmark configuration: W [8960, 1536], x [1, 1536],
    plain N(0, 1) activations, seed 0."""
    return weights(8960, 1536, 0), activations(1, 1536, 0, outliers=False)


def block_layers(model: str, fused: bool = False):
    """[(name, N, K)] of one block.  ``fused`` concatenates along N the
    projections that share an input (q|k|v and gate|up): group quantization is
    independent per output row, so packing the concatenation equals
    concatenating the packings."""
    L = MODELS[model]["layers"]
    if not fused:
        return [(n, *L[n]) for n in ("q", "k", "v", "o", "gate", "up", "down")]
    return [
        ("qkv", L["q"][0] + L["k"][0] + L["v"][0], L["q"][1]),
        ("o", *L["o"]),
        ("gateup", L["gate"][0] + L["up"][0], L["gate"][1]),
        ("down", *L["down"]),
    ]


def fused_parts(name: str):
    return {"qkv": ("q", "k", "v"), "gateup": ("gate", "up")}.get(name, (name,))
