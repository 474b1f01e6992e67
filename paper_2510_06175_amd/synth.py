"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path.

This module only draws random tensors of the right shape, dtype and value
structure; it contains none of the method's arithmetic (no transform, no
quantization, no attention) and imports neither the oracle nor the GPU
library.  Everything comes from ``numpy.random.Generator(PCG64(seed))``.

The tensors stand in for Llama-3.1-8B KV caches (32 query heads, 8 KV heads,
head dim 128; kernel sweep shapes of App. B.2), which would need model weights
and long-context text that are not available here.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

NUM_CENTROIDS = 256  # 8-bit codes: one uint8 index per sub-vector (Sec. 2.2)


@dataclass(frozen=True)
class Shape:
    """Problem shape in the paper's notation."""
    B: int            # batch
    Hq: int           # query heads
    Hkv: int          # KV heads
    D: int            # head dim
    N: int            # tokens in the cache
    d_k: int          # key sub-vector dim
    d_v: int          # value sub-vector dim
    b_k: int = 8      # key code width in bits (the m of the paper's "dnbm" names)
    b_v: int = 8      # value code width in bits

    @property
    def Mk(self) -> int:
        return self.D // self.d_k

    @property
    def Mv(self) -> int:
        return self.D // self.d_v

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def row_bytes_k(self) -> int:
        """Bytes of one token's key codes (Mk codes of b_k bits, end to end)."""
        return self.Mk * self.b_k // 8

    @property
    def row_bytes_v(self) -> int:
        return self.Mv * self.b_v // 8

    def index_bytes(self) -> int:
        """Compressed-KV bytes one decode step has to read."""
        return self.B * self.Hkv * self.N * (self.row_bytes_k + self.row_bytes_v)


# benchmark configurations (b2d4 = d 4, b4d2 = d 2; 8-bit codes in both)
TINY = Shape(B=1, Hq=1, Hkv=1, D=128, N=4096, d_k=4, d_v=4)
LLAMA8B_32K = Shape(B=1, Hq=32, Hkv=8, D=128, N=32768, d_k=4, d_v=4)
LLAMA8B_BATCH32 = Shape(B=32, Hq=32, Hkv=8, D=128, N=8192, d_k=4, d_v=4)
LLAMA8B_196K = Shape(B=1, Hq=32, Hkv=8, D=128, N=196608, d_k=4, d_v=4)
LLAMA8B_196K_B4D2 = Shape(B=1, Hq=32, Hkv=8, D=128, N=196608, d_k=2, d_v=2)
# head dim 64 (the paper's kernel sweep also covers it; Mistral / Qwen-class shapes), d = 4
HEADDIM64_196K = Shape(1, 32, 8, 64, 196608, 4, 4)
# keys at 4 bits per element (d = 2), values at 2 (d = 4): "more bits for the keys", Sec. 3.2
LLAMA8B_196K_KD2_VD4 = Shape(B=1, Hq=32, Hkv=8, D=128, N=196608, d_k=2, d_v=4)
# 1.5 bits per element: d = 8, 12-bit codes, one 4096-entry codebook per KV head (Sec. 4.1, Sec. 4.4)
LLAMA8B_196K_D8B12 = Shape(B=1, Hq=32, Hkv=8, D=128, N=196608, d_k=8, d_v=8, b_k=12, b_v=12)
ENCODE_64K = Shape(B=1, Hq=32, Hkv=8, D=128, N=65536, d_k=4, d_v=4)


def rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def codebooks(g: np.random.Generator, Hkv: int, M: int, d: int) -> np.ndarray:
    """Per-(KV head, sub-space) codebooks [Hkv, M, 256, d], fp16, centroids ~ N(0, 1)."""
    return g.standard_normal((Hkv, M, NUM_CENTROIDS, d), dtype=np.float32).astype(np.float16)


def shared_codebooks(g: np.random.Generator, Hkv: int, bits: int, d: int) -> np.ndarray:
    """One codebook of 2^bits centroids per KV head, shared by its sub-spaces: [Hkv, 2^bits, d], fp16 ~ N(0, 1)."""
    return g.standard_normal((Hkv, 1 << bits, d), dtype=np.float32).astype(np.float16)


def codebooks_for(g: np.random.Generator, Hkv: int, M: int, d: int, bits: int) -> np.ndarray:
    """The codebook tensor a side with `bits`-bit codes uses: per sub-space at 8 bits, shared above."""
    return codebooks(g, Hkv, M, d) if bits == 8 else shared_codebooks(g, Hkv, bits, d)


def queries(g: np.random.Generator, B: int, Hq: int, D: int) -> np.ndarray:
    """Decode-step queries [B, Hq, D], fp16 ~ N(0, 1)."""
    return g.standard_normal((B, Hq, D), dtype=np.float32).astype(np.float16)


def lognormal_lambda(g: np.random.Generator, Hkv: int, D: int, sigma: float = 0.5) -> np.ndarray:
    """Per-channel smoothing factors [Hkv, D], fp32 ~ LogNormal(0, sigma)."""
    return np.exp(sigma * g.standard_normal((Hkv, D))).astype(np.float32)


def random_indices(g: np.random.Generator, B: int, Hkv: int, n_cap: int, M: int) -> np.ndarray:
    """Uniform random uint8 codes [B, Hkv, n_cap, M]."""
    return g.integers(0, NUM_CENTROIDS, size=(B, Hkv, n_cap, M), dtype=np.uint8)


def random_code_rows(g: np.random.Generator, B: int, Hkv: int, n_cap: int, row_bytes: int) -> np.ndarray:
    """Uniform random code rows [B, Hkv, n_cap, row_bytes] as bytes.  With 2^b centroids every b-bit
    pattern is a valid code, so uniform random bytes are uniform random codes at any code width."""
    return g.integers(0, 256, size=(B, Hkv, n_cap, row_bytes), dtype=np.uint8)


def keys_with_outlier_channels(g: np.random.Generator, B: int, Hkv: int, T: int, D: int,
                               n_outlier: int, factor: float = 20.0):
    """Keys [B, Hkv, T, D] fp16 ~ N(0, 1) with `n_outlier` seeded channels per KV
    head scaled by `factor` (the few-large-channels structure of real key caches,
    Fig. 1 / Fig. 8).  Returns (keys, outlier_channels [Hkv, n_outlier])."""
    k = g.standard_normal((B, Hkv, T, D), dtype=np.float32)
    ch = np.stack([np.sort(g.choice(D, size=n_outlier, replace=False)) for _ in range(Hkv)])
    for h in range(Hkv):
        k[:, h, :, ch[h]] *= factor
    return k.astype(np.float16), ch


def values(g: np.random.Generator, B: int, Hkv: int, T: int, D: int) -> np.ndarray:
    """Values [B, Hkv, T, D] fp16 ~ N(0, 1)."""
    return g.standard_normal((B, Hkv, T, D), dtype=np.float32).astype(np.float16)


def decode_inputs(shape: Shape, seed: int, n_cap: int | None = None) -> dict:
    """Inputs of one decode step over a cache of uniform random codes
    (the 8B-shaped configurations): q, lam, cb_k, cb_v, k_idx, v_idx."""
    g = rng(seed)
    n_cap = shape.N if n_cap is None else n_cap
    return {
        "q": queries(g, shape.B, shape.Hq, shape.D),
        "lam": lognormal_lambda(g, shape.Hkv, shape.D),
        "cb_k": codebooks_for(g, shape.Hkv, shape.Mk, shape.d_k, shape.b_k),
        "cb_v": codebooks_for(g, shape.Hkv, shape.Mv, shape.d_v, shape.b_v),
        "k_idx": random_code_rows(g, shape.B, shape.Hkv, n_cap, shape.row_bytes_k),
        "v_idx": random_code_rows(g, shape.B, shape.Hkv, n_cap, shape.row_bytes_v),
    }


def residual_window(shape: Shape, seed: int, r_cap: int, n_outlier: int = 4) -> dict:
    """Full-precision window of the r_cap most recent tokens: raw fp16 keys (with outlier
    channels, as un-smoothed keys have) and raw values, [B, Hkv, r_cap, D] each."""
    g = rng(seed)
    k, _ = keys_with_outlier_channels(g, shape.B, shape.Hkv, r_cap, shape.D, n_outlier)
    return {"k_res": k, "v_res": values(g, shape.B, shape.Hkv, r_cap, shape.D)}


def encode_inputs(shape: Shape, seed: int, n_outlier: int) -> dict:
    """Inputs of a cache fill: raw keys (with outlier channels), raw values, codebooks,
    and the decode-step query.  The smoothing factors are NOT drawn here: where a
    configuration derives them from the keys (Eq. 4) the caller computes them."""
    g = rng(seed)
    k, ch = keys_with_outlier_channels(g, shape.B, shape.Hkv, shape.N, shape.D, n_outlier)
    return {
        "k": k,
        "outlier_channels": ch,
        "v": values(g, shape.B, shape.Hkv, shape.N, shape.D),
        "cb_k": codebooks_for(g, shape.Hkv, shape.Mk, shape.d_k, shape.b_k),
        "cb_v": codebooks_for(g, shape.Hkv, shape.Mv, shape.d_v, shape.b_v),
        "q": queries(rng(0), shape.B, shape.Hq, shape.D),
    }
