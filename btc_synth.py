"""Seeded synthetic inputs for the binary-codebook linear layer.

This module only draws random numbers and shapes them; it holds none of the
method's arithmetic (no packing, no decoding, no dot products).  Both the CPU
oracle's tests and the HIP path's tests/bench take their inputs from here.

A layer is (codebook, idx, alpha, mu) and an activation block x:

  codebook : uint32[K]       bit t of entry k is element t of sign pattern k
                             (1 => +1, 0 => -1), t < v
  idx      : int32[out][nchunks]   entry j of row i selects the pattern of the
                             j-th length-v chunk of weight row i
  alpha,mu : float32[out]    per-row scale and per-row mean
  x        : uint16[batch][in]     fp16 or bf16 bit patterns

Draw order is fixed: codebook -> idx -> alpha -> mu -> x -> outlier channels,
from one numpy Generator(PCG64(seed)) per layer, so a layer does not depend on
the order in which a sweep visits shapes.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np


def index_bits(K: int) -> int:
    """Smallest b with 2**b >= K (K >= 2)."""
    if K < 2:
        raise ValueError("K must be >= 2")
    return int(K - 1).bit_length()


def num_chunks(n_in: int, v: int) -> int:
    return (n_in + v - 1) // v


def words_per_row(n_in: int, v: int, K: int) -> int:
    return (num_chunks(n_in, v) * index_bits(K) + 31) // 32


@dataclasses.dataclass
class Layer:
    out: int
    n_in: int
    v: int
    K: int
    codebook: np.ndarray  # uint32[K]
    idx: np.ndarray       # int32[out][nchunks]
    alpha: np.ndarray     # float32[out]
    mu: np.ndarray        # float32[out]

    @property
    def b(self) -> int:
        return index_bits(self.K)

    @property
    def nchunks(self) -> int:
        return num_chunks(self.n_in, self.v)

    @property
    def wpr(self) -> int:
        return words_per_row(self.n_in, self.v, self.K)


def draw_codebook(rng: np.random.Generator, v: int, K: int) -> np.ndarray:
    """K sign patterns of length v as bit masks.

    K <= 2**v: K distinct patterns, drawn without replacement.
    K >  2**v: every pattern the same number of times (K must be a multiple of
    2**v), in a seeded shuffle -- a codebook with duplicates, as a 1024-entry
    codebook of length-9 patterns must be.
    """
    n_pat = 1 << v
    if K <= n_pat:
        if n_pat <= (1 << 22):
            cb = rng.choice(n_pat, size=K, replace=False)
        else:  # large v: rejection is cheap since K << 2**v
            seen: set = set()
            while len(seen) < K:
                seen.update(int(t) for t in rng.integers(0, n_pat, size=K - len(seen)))
            cb = rng.permutation(np.fromiter(seen, dtype=np.int64, count=K))
    else:
        if K % n_pat:
            raise ValueError("K > 2**v needs K a multiple of 2**v")
        cb = rng.permutation(np.tile(np.arange(n_pat), K // n_pat))
    return cb.astype(np.uint32)


def draw_indices(rng: np.random.Generator, out: int, nchunks: int, K: int,
                 dist: str = "uniform", zipf_s: float = 1.1) -> np.ndarray:
    """uniform: iid in [0,K).  zipf: bounded Zipf, P(rank r) ~ r**-s for
    r = 1..K, rank r -> index r-1, sampled by inverse CDF in fp64."""
    if dist == "uniform":
        return rng.integers(0, K, size=(out, nchunks), dtype=np.int32)
    if dist == "zipf":
        w = np.arange(1, K + 1, dtype=np.float64) ** (-zipf_s)
        cdf = np.cumsum(w)
        cdf /= cdf[-1]
        u = rng.random(size=(out, nchunks))
        idx = np.searchsorted(cdf, u, side="left")
        return np.minimum(idx, K - 1).astype(np.int32)
    raise ValueError(f"unknown index distribution {dist!r}")


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even), return the uint16 patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def draw_layer(seed: int, out: int, n_in: int, v: int, K: int,
               dist: str = "uniform") -> tuple[Layer, np.random.Generator]:
    rng = np.random.Generator(np.random.PCG64(seed))
    codebook = draw_codebook(rng, v, K)
    idx = draw_indices(rng, out, num_chunks(n_in, v), K, dist)
    alpha = np.abs(rng.normal(0.0, 0.02, size=out)).astype(np.float32)
    mu = rng.normal(0.0, 0.002, size=out).astype(np.float32)
    return Layer(out, n_in, v, K, codebook, idx, alpha, mu), rng


def draw_x(rng: np.random.Generator, batch: int, n_in: int, dtype: str = "f16",
           outlier_frac: float = 0.0, outlier_scale: float = 20.0) -> np.ndarray:
    """N(0,1) activations as fp16/bf16 bit patterns, uint16[batch][n_in].
    With outlier_frac > 0, floor(frac*n_in) distinct channels (the same for
    every batch row) are scaled by outlier_scale before rounding."""
    x = rng.normal(0.0, 1.0, size=(batch, n_in))
    n_outl = int(np.floor(outlier_frac * n_in))
    if n_outl > 0:
        ch = rng.choice(n_in, size=n_outl, replace=False)
        x[:, ch] *= outlier_scale
    if dtype == "f16":
        return x.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        return f32_to_bf16_bits(x.astype(np.float32))
    raise ValueError(dtype)


def make_case(seed: int, out: int, n_in: int, v: int, K: int, batch: int,
              dist: str = "uniform", x_dtype: str = "f16",
              outlier_frac: float = 0.0) -> tuple[Layer, np.ndarray]:
    layer, rng = draw_layer(seed, out, n_in, v, K, dist)
    x = draw_x(rng, batch, n_in, x_dtype, outlier_frac)
    return layer, x


# --- the five benchmark configurations (shapes, bit settings, distributions) ---

LLAMA2_7B = [(4096, 4096), (11008, 4096), (4096, 11008)]
LLAMA2_13B = [(5120, 5120), (13824, 5120), (5120, 13824)]
LLAMA2_70B = [(8192, 8192), (1024, 8192), (28672, 8192), (8192, 28672)]
SETTINGS_70B = [(9, 1024), (10, 512), (10, 128)]  # 1.11 / 0.9 / 0.7 bit


def config_cases(cfg: int) -> list[dict]:
    """Parameter dicts for make_case(), one per (shape, setting, batch)."""
    cases: list[dict] = []
    if cfg == 0:
        cases.append(dict(out=4096, n_in=4096, v=10, K=512, batch=1))
    elif cfg == 1:
        for (o, i) in LLAMA2_7B:
            for bt in (1, 4, 16):
                cases.append(dict(out=o, n_in=i, v=10, K=512, batch=bt, outlier_frac=0.01))
    elif cfg == 2:
        for (o, i) in LLAMA2_13B:
            cases.append(dict(out=o, n_in=i, v=10, K=256, batch=1, dist="zipf"))
    elif cfg == 3:
        for (o, i) in LLAMA2_13B:
            for m in (512, 2048):
                cases.append(dict(out=o, n_in=i, v=10, K=256, batch=m, x_dtype="bf16"))
    elif cfg == 4:
        for (v, K) in SETTINGS_70B:
            for (o, i) in LLAMA2_70B:
                cases.append(dict(out=o, n_in=i, v=v, K=K, batch=1))
    else:
        raise ValueError(cfg)
    for c in cases:
        c.setdefault("seed", 0)
    return cases


def draw_transform(seed: int, n1: int, n2: int, perturb: float = 0.02):
    """A synthetic transformation pair for an activation row of n1*n2 channels: sign bits of the diagonal
    sign matrix (uint32[ceil(n/32)], bit k set => sigma_k = +1, unused tail bits zero) and the two
    Kronecker factors P1 [n1][n1], P2 [n2][n2] (float32, row-major).  The factors stand in for learned
    invertible matrices: a random orthogonal matrix (QR of a Gaussian one) plus N(0, perturb) noise."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n = n1 * n2
    sigma = rng.integers(0, 2, size=n, dtype=np.uint32)
    bits = np.zeros((n + 31) // 32, dtype=np.uint32)
    for k in np.nonzero(sigma)[0]:
        bits[k >> 5] |= np.uint32(1) << np.uint32(k & 31)
    factors = []
    for m in (n1, n2):
        q, _ = np.linalg.qr(rng.standard_normal((m, m)))
        factors.append((q + perturb * rng.standard_normal((m, m))).astype(np.float32))
    return bits, factors[0], factors[1]
