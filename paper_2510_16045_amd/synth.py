"""Seeded synthetic inputs for the AMS-Quant Linear: weight and activation matrices.

This module only draws random numbers and shapes them; it holds none of the
method's arithmetic (no quantization, packing or matmul) and imports nothing
but numpy, so that both the HIP path's tests/benchmark and the independent CPU
oracle's tests can be fed the same arrays.

The weight distributions follow the paper's observation that LLM weights are
bell-shaped (Sec. 2.2, weight-distribution figure): Gaussian N(0, 0.02) for
the 8B-shaped layers, heavy-tailed Student-t with sparse outliers for the
70B-shaped ones.  The layer shapes are (N_out, K_in) like Table 3's.
"""

from __future__ import annotations

import numpy as np

BASE_SEED = 2510_16045

# (N_out, K_in) of one Llama-3-8B decoder layer's Linear set at decode time
LLAMA8B_LAYERS = {
    "qkv": (6144, 4096),
    "o": (4096, 4096),
    "gate_up": (28672, 4096),
    "down": (4096, 14336),
}
LLAMA8B_LM_HEAD = (128256, 4096)  # the vocabulary projection of Llama-3-8B
LLAMA70B_LAYERS = {
    "o": (8192, 8192),
    "gate_up": (57344, 8192),
    "down": (8192, 28672),
}
# the paper's own efficiency shapes (Table 3): MLP-down layers
QWEN_DOWN_LAYERS = {
    "qwen3-4b": (2560, 9728),
    "qwen2.5-7b": (3584, 18944),
    "qwen3-32b": (5120, 25600),
}


def _rng(seed_offset: int, chunk: int | None = None) -> np.random.Generator:
    seed = BASE_SEED + int(seed_offset)
    return np.random.default_rng(seed if chunk is None else [seed, int(chunk)])


def _fill_by_chunks(out: np.ndarray, rows_per_chunk: int, seed_offset: int, draw) -> np.ndarray:
    """out[r0:r1] = draw(rng of chunk, r1 - r0) for consecutive row chunks.  Every chunk has its own
    generator, seeded by (seed, chunk index), so the result does not depend on how many threads draw."""
    import os
    from concurrent.futures import ThreadPoolExecutor

    N = out.shape[0]
    starts = list(range(0, N, rows_per_chunk))

    def one(c):
        r0 = starts[c]
        r1 = min(N, r0 + rows_per_chunk)
        out[r0:r1] = draw(_rng(seed_offset, c), r1 - r0)

    workers = min(16, len(os.sched_getaffinity(0)), len(starts))
    if workers <= 1:
        for c in range(len(starts)):
            one(c)
    else:
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(one, range(len(starts))))
    return out


def gaussian_weights(N: int, K: int, seed_offset: int = 0, std: float = 0.02) -> np.ndarray:
    """fp16 [N,K] drawn N(0, std) in fp32 then cast."""
    out = np.empty((N, K), dtype=np.float16)
    step = max(1, (1 << 22) // max(K, 1))  # chunked: bounds the fp32 temporaries, lets several cores draw
    return _fill_by_chunks(out, step, seed_offset, lambda rng, n: (rng.standard_normal((n, K), dtype=np.float32) * np.float32(std)).astype(np.float16))


def heavy_tail_weights(
    N: int, K: int, seed_offset: int = 0, std: float = 0.02, nu: float = 4.0, p_outlier: float = 1e-3, outlier_gain: float = 20.0
) -> np.ndarray:
    """fp16 [N,K]: std * Student-t(nu), a Bernoulli(p_outlier) subset scaled by outlier_gain."""

    def draw(rng, n):
        w = rng.standard_t(nu, size=(n, K)).astype(np.float32) * np.float32(std)
        mask = rng.random((n, K), dtype=np.float32) < np.float32(p_outlier)
        w = np.where(mask, w * np.float32(outlier_gain), w)
        return np.clip(w, -60000.0, 60000.0).astype(np.float16)

    out = np.empty((N, K), dtype=np.float16)
    step = max(1, (1 << 21) // max(K, 1))
    return _fill_by_chunks(out, step, seed_offset, draw)


def activations(M: int, K: int, seed_offset: int = 0, std: float = 1.0) -> np.ndarray:
    """fp16 [M,K] drawn N(0, std)."""
    rng = _rng(10_000 + seed_offset)
    return (rng.standard_normal((M, K), dtype=np.float32) * np.float32(std)).astype(np.float16)


def config1():
    """Smallest case: W 256x768 N(0,0.02), X 1x768 N(0,1) (FP4.25 in the baseline configs)."""
    return gaussian_weights(256, 768, 1), activations(1, 768, 1)


def config2():
    """Llama-3-8B q/o projection: W 4096x4096 N(0,0.02), X 1x4096 (FP5.33 in the baseline configs)."""
    return gaussian_weights(4096, 4096, 2), activations(1, 4096, 2)
