"""Seeded synthetic inputs shaped like the paper's workloads.

The paper measures on the trained weights of Gemma 27B, Qwen3 32B and
Llama3.3 70B with GSM8K prompts (Sec. VI-A).  Dequantisation never sees
prompts and its cost does not depend on the batch (Sec. II-A), so Gaussian
weights of the same projection shapes stand in for them.

This module holds no NF4 arithmetic: it only draws numbers and names shapes,
and it is the one module that both the CPU oracle's tests and the GPU path's
tests feed from.
"""
import numpy as np

# (rows, cols) of the decoder-layer projections, PyTorch Linear layout [out, in]
# flattened row-major; only the element count matters to dequantisation.
LLAMA33_70B = {  # hidden 8192, 64 q / 8 kv heads x 128, intermediate 28672, 80 layers
    "q": (8192, 8192), "k": (1024, 8192), "v": (1024, 8192), "o": (8192, 8192),
    "gate": (28672, 8192), "up": (28672, 8192), "down": (8192, 28672),
}
LLAMA33_70B_LAYERS = 80
LLAMA33_70B_SIGMA = 0.015

QWEN3_32B = {  # hidden 5120, 64 q / 8 kv heads x 128, intermediate 25600
    "q": (8192, 5120), "k": (1024, 5120), "v": (1024, 5120), "o": (5120, 8192),
    "gate": (25600, 5120), "up": (25600, 5120), "down": (5120, 25600),
}
QWEN3_32B_SIGMA = 0.02

GEMMA_27B = {  # hidden 5376, q 4096, kv 2048, intermediate 21504
    "q": (4096, 5376), "k": (2048, 5376), "v": (2048, 5376),
    "gate": (21504, 5376), "up": (21504, 5376), "down": (5376, 21504),
}
GEMMA_27B_SIGMA = 0.02

RAGGED_SIZES = (1, 63, 65, 1_000_003)

GEMV_SHAPES = ((8192, 28672), (28672, 8192))   # (N rows = outputs, K cols = inputs)
GEMV_BATCHES = (1, 4, 16)


def numel(shape):
    return int(shape[0]) * int(shape[1])


def gaussian_weights(n, sigma, seed, outlier_p=0.0, outlier_mult=8.0):
    """float32[n] ~ N(0, sigma^2); each element independently multiplied by
    outlier_mult with probability outlier_p."""
    rng = np.random.Generator(np.random.PCG64(seed))
    w = rng.standard_normal(n, dtype=np.float32)
    w *= np.float32(sigma)
    if outlier_p > 0.0:
        hit = rng.random(n, dtype=np.float32) < np.float32(outlier_p)
        w[hit] *= np.float32(outlier_mult)
    return w


def activations_fp16(batch, k, seed):
    """float16[batch][k] ~ N(0, 1), rounded to fp16."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.standard_normal((batch, k), dtype=np.float32).astype(np.float16)


def random_codes(nbytes, seed):
    """uint8[nbytes], every byte value equally likely (both nibbles uniform)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, 256, size=nbytes, dtype=np.uint8)


def positive_scales(count, seed, lo=1e-3, hi=1.0):
    """float32[count] log-uniform in [lo, hi): stand-in absmax values."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return np.exp(rng.uniform(np.log(lo), np.log(hi), size=count)).astype(np.float32)


def e2m1_codebook():
    """An FP4-style alternative to the NF4 levels, as input data for the codebook entry points: the 16 values of
    the 4-bit float with 1 sign, 2 exponent and 1 mantissa bit (code = s e e m), divided by the largest (6)."""
    mags = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=np.float64) / 6.0
    return np.concatenate([mags, -mags]).astype(np.float32)
