"""Seeded synthetic inputs for the vocabulary-layer workloads.

This module only *generates data*: random hidden states, weight shards, labels,
token ids and upstream gradients with the shapes and value distributions of the
five benchmark configurations, plus bf16 <-> fp32 bit conversions.  It contains
none of the method's arithmetic (no logits, softmax, loss or gradients) and is
the only module imported by both the CPU oracle's tests and the GPU path's
harness, so that both sides receive bit-identical inputs.

Random numbers come from NumPy's counter-based Philox generator keyed by
(base seed, sub-stream id, index), so any shard of any tensor can be produced
on its own, in any order, without generating the tensors before it.

bf16 tensors are carried as ``uint16`` bit patterns (NumPy has no bf16 type).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 20241105

# sub-stream ids
STREAM_H = 1
STREAM_W = 2
STREAM_LABELS = 3
STREAM_PERM = 4
STREAM_GRAD = 5
STREAM_TABLE = 6


@dataclass(frozen=True)
class OutputConfig:
    """One output-layer workload: N tokens, hidden h, vocabulary V in p shards."""
    name: str
    N: int
    h: int
    V: int
    p: int
    dtype: str          # "f32" or "bf16": storage type of H and W
    h_std: float
    w_std: float
    labels: str         # "uniform" or "zipf"
    save_logits: bool   # True: logits stored in fwd; False: recomputed in bwd

    @property
    def Vs(self) -> int:
        return self.V // self.p

    @property
    def model_flops(self) -> float:
        # three dense products of 2*N*h*V flops each
        return 6.0 * self.N * self.h * self.V


@dataclass(frozen=True)
class EmbedConfig:
    """One input-embedding workload."""
    name: str
    N: int
    h: int
    V: int
    p: int
    dtype: str
    table_std: float
    grad_std: float
    ids: str            # "uniform" or "zipf"

    @property
    def Vs(self) -> int:
        return self.V // self.p


CONFIGS = {
    "cfg1_tiny": OutputConfig("cfg1_tiny", N=128, h=256, V=8192, p=2, dtype="f32",
                              h_std=1.0, w_std=0.02, labels="uniform", save_logits=True),
    "cfg2_llama": OutputConfig("cfg2_llama", N=4096, h=4096, V=32000, p=8, dtype="bf16",
                               h_std=1.0, w_std=0.02, labels="uniform", save_logits=True),
    "cfg3_large_vocab": OutputConfig("cfg3_large_vocab", N=4096, h=4096, V=128256, p=8,
                                     dtype="bf16", h_std=1.0, w_std=0.02, labels="zipf",
                                     save_logits=True),
    "cfg4_very_large_vocab": OutputConfig("cfg4_very_large_vocab", N=4096, h=8192, V=256000,
                                          p=16, dtype="bf16", h_std=1.0, w_std=0.01,
                                          labels="zipf", save_logits=False),
    "cfg5_embedding": EmbedConfig("cfg5_embedding", N=8192, h=4096, V=256000, p=8,
                                  dtype="bf16", table_std=0.02, grad_std=1.0, ids="zipf"),
}


# --------------------------------------------------------------------------- #
# bf16 bit helpers
# --------------------------------------------------------------------------- #
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns uint16 bit patterns.

    Inputs are finite here, so NaN handling is not needed.
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def as_f64(x: np.ndarray) -> np.ndarray:
    """Exact fp64 view of a stored tensor (uint16 = bf16 bits, else fp32)."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


def as_f32(x: np.ndarray) -> np.ndarray:
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x)
    return x.astype(np.float32)


# --------------------------------------------------------------------------- #
# generators
# --------------------------------------------------------------------------- #
def _rng(seed: int, stream: int, index: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64((stream << 32) | index)]))


def normal(shape, std: float, dtype: str, seed: int, stream: int, index: int = 0) -> np.ndarray:
    """N(0, std) tensor stored as fp32 ("f32") or as bf16 bit patterns ("bf16")."""
    g = _rng(seed, stream, index)
    x = g.standard_normal(size=shape, dtype=np.float32)
    x *= np.float32(std)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    if dtype == "f32":
        return x
    raise ValueError(dtype)


def zipf_ids(n: int, V: int, s: float, seed: int, stream: int = STREAM_LABELS) -> np.ndarray:
    """n ids in [0, V): ranks k = 1..V drawn with P(k) proportional to k**-s by inverse
    CDF on an fp64 cumulative table, then mapped through a seeded random permutation of
    the vocabulary (so hot ids are spread over the shards)."""
    w = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    u = _rng(seed, stream).random(n)
    rank = np.minimum(np.searchsorted(cdf, u, side="left"), V - 1)
    perm = _rng(seed, STREAM_PERM).permutation(V)
    return perm[rank].astype(np.int64)


def uniform_ids(n: int, V: int, seed: int, stream: int = STREAM_LABELS) -> np.ndarray:
    return _rng(seed, stream).integers(0, V, size=n, dtype=np.int64)


def make_labels(cfg, seed: int = BASE_SEED) -> np.ndarray:
    kind = cfg.labels if isinstance(cfg, OutputConfig) else cfg.ids
    if kind == "uniform":
        return uniform_ids(cfg.N, cfg.V, seed)
    if kind == "zipf":
        return zipf_ids(cfg.N, cfg.V, 1.1, seed)
    raise ValueError(kind)


def make_H(cfg: OutputConfig, seed: int = BASE_SEED) -> np.ndarray:
    return normal((cfg.N, cfg.h), cfg.h_std, cfg.dtype, seed, STREAM_H)


def make_W_shard(cfg: OutputConfig, r: int, seed: int = BASE_SEED) -> np.ndarray:
    """Rows [r*Vs, (r+1)*Vs) of the output embedding; each shard has its own counter
    stream, so shards can be generated one at a time."""
    return normal((cfg.Vs, cfg.h), cfg.w_std, cfg.dtype, seed, STREAM_W, r)


def make_table_shard(cfg: EmbedConfig, r: int, seed: int = BASE_SEED) -> np.ndarray:
    return normal((cfg.Vs, cfg.h), cfg.table_std, cfg.dtype, seed, STREAM_TABLE, r)


def make_grad_out(cfg: EmbedConfig, seed: int = BASE_SEED) -> np.ndarray:
    return normal((cfg.N, cfg.h), cfg.grad_std, cfg.dtype, seed, STREAM_GRAD)


def small_output_case(N: int, h: int, V: int, p: int, dtype: str = "f32", seed: int = 7,
                      labels: str = "uniform", w_std: float = 0.05):
    """Free-form small case for tests: returns (H, [W_0..W_{p-1}], labels)."""
    cfg = OutputConfig("small", N=N, h=h, V=V, p=p, dtype=dtype, h_std=1.0, w_std=w_std,
                       labels=labels, save_logits=True)
    return make_H(cfg, seed), [make_W_shard(cfg, r, seed) for r in range(p)], make_labels(cfg, seed)
