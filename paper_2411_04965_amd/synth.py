"""Seeded synthetic inputs shaped like the activations and weights of BitNet a4.8.

This module only draws random tensors.  It holds none of the method's
arithmetic (no quantizer, no ternarisation, no matmul), so that the CPU oracle
and the HIP path can both be fed from it without sharing any computation.

The distributions imitate what Section 2.1 says about a 7B BitNet b1.58:
inputs to the attention and FFN blocks look Gaussian, while the inputs to the
attention output projection and to the FFN down projection are sharply peaked
at zero with a few outlier channels.  They stand in for the paper's C4 /
RedPajama activations, which need trained checkpoints.

All generators return float32 numpy arrays.  Generators documented as "bf16"
return float32 values that are exactly representable in bfloat16, so a cast to
a bfloat16 tensor is lossless.
"""
import numpy as np

BASE_SEED = 20241104


def seed_for(config: int, index: int) -> int:
    """Seed convention: one stream per (config, tensor index)."""
    return BASE_SEED + 1000 * int(config) + int(index)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even.

    Storage conversion of generated data only (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32 (exact)."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def snap_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 data onto the bfloat16 grid, still stored as float32."""
    return from_bf16_bits(to_bf16_bits(x))


def gauss_outlier(M: int, K: int, n_out: int, factor: float, seed: int) -> np.ndarray:
    """N(0,1) float32 with `n_out` randomly chosen channels scaled by `factor`."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    ch = rng.choice(K, size=n_out, replace=False)
    x[:, ch] *= np.float32(factor)
    return x


def heavy(M: int, K: int, seed: int, frac: float = 0.005, scale: float = 10.0) -> np.ndarray:
    """bf16-valued N(0,1) with ~0.5% of the channels replaced by Student-t(2) * scale."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    n_out = max(1, int(round(frac * K)))
    ch = rng.choice(K, size=n_out, replace=False)
    x[:, ch] = (scale * rng.standard_t(2.0, size=(M, n_out))).astype(np.float32)
    return snap_bf16(x)


def glu_like(M: int, K: int, seed: int, keep: float = 0.45) -> np.ndarray:
    """bf16-valued stand-in for a down-projection input, drawn directly (no gating arithmetic).

    Each entry is zero with probability 1 - keep (more than half of a row in expectation),
    otherwise a `heavy` value times an independent chi-square(1) magnitude: sharply peaked
    at zero with a long tail and a few outlier channels, like the state behind a gated
    unit."""
    x = heavy(M, K, seed)
    rng = np.random.default_rng(seed + 500)
    mag = rng.gamma(0.5, 2.0, size=(M, K)).astype(np.float32)
    mask = rng.random((M, K)) < keep
    return snap_bf16(np.where(mask, x * mag, np.float32(0)).astype(np.float32))


def latent_weights(N: int, K: int, seed: int, std: float = 0.02) -> np.ndarray:
    """Latent full-precision weights W[N, K] ~ N(0, std^2), float32."""
    rng = np.random.default_rng(seed)
    return (std * rng.standard_normal((N, K))).astype(np.float32)


# Model shapes from the paper's Appendix A (hidden size, GLU size).
SHAPES = {
    "700M": (1536, 4096),
    "1.3B": (2048, 5460),
    "3B": (3200, 8640),
    "7B": (4096, 11008),
}


def projections(hidden: int, ffn: int):
    """(name, N, K, activation kind) of the projections in one block.

    kind 'a4' = per-token INT4 input, 'a8s' = top-50% + INT8 input."""
    return [
        ("qkv", 3 * hidden, hidden, "a4"),
        ("o", hidden, hidden, "a8s"),
        ("gate", ffn, hidden, "a4"),
        ("up", ffn, hidden, "a4"),
        ("down", hidden, ffn, "a8s"),
    ]
