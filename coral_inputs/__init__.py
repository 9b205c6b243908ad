"""Seeded synthetic inputs for the weight-grouped LM head.

This module only draws random numbers, rounds them to the storage type and
lays out the vocabulary partition.  It holds none of the method's arithmetic
(no gate, no selection, no logits, no top-k): both the CPU oracle's tests and
the HIP path's tests feed from it, and neither of those imports the other.

Shapes follow the draft heads of the paper's Table 1 (Llama2-7B, Llama3-8B,
Qwen2.5-7B: hidden size d and vocabulary V); the (number of groups, active
groups) pairs lie inside the grid of the router ablation (Table 4), and the
candidate count is the ten candidates per draft token of the tree-decoding
discussion in the appendix on the LM head router.

Recipe (fixed; every draw comes from numpy's PCG64 seeded with
SeedSequence([seed, stream])):
  stream 0  lm_W      [V,H]  N(0, 0.02^2), float32 draws in consecutive blocks
                             of 8192 rows, then rounded to the storage type
  stream 1  gate_W    [G,H]  N(0, 0.02^2)
  stream 2  gate_bias [G]    N(0, bias_std^2) float32 (only if bias_std > 0)
  stream 3  perm      permutation of 0..V-1; group n owns
                             sorted(perm[n*v:(n+1)*v]) with v = V/G
                             (grouping="contiguous": perm is the identity)
  stream 4  router_W1 [H,H]  N(0, 0.02^2) (the router's first projection, Eq. 7;
                             drawn only by make_router_W1)
  stream 16+b  hidden batch b  [M,H]  N(0,1), optionally each row divided by
                             its RMS (float64 mean of squares), then rounded
bf16 storage = round-to-nearest-even of the float32 value, kept as uint16; f16 storage =
IEEE binary16 of the float32 value (nearest even), kept as uint16 as well.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np

_ROW_BLOCK = 8192


@dataclass(frozen=True)
class HeadConfig:
    name: str
    dtype: str              # "f32" or "bf16": storage type of hidden, gate_W, lm_W
    H: int                  # hidden size (paper's d)
    V: int                  # vocabulary size
    G: int                  # number of groups (paper's N)
    g: int                  # active groups per token (paper's top-n)
    Ms: Tuple[int, ...]     # draft tokens per step exercised for this shape
    k: int                  # candidates per token
    seed: int
    unit_rms: bool          # scale each hidden row to unit RMS before rounding
    bias_std: float = 0.0   # std of the per-group gate bias (0: no bias)
    grouping: str = "permuted"   # "permuted" or "contiguous"

    @property
    def v(self) -> int:
        return self.V // self.G

    def scaled(self, **kw) -> "HeadConfig":
        """Same recipe at another size (parity cases the oracle finishes fast)."""
        return replace(self, **kw)


CONFIGS = {
    "tiny_f32": HeadConfig("tiny_f32", "f32", 256, 8192, 16, 2, (4,), 8, 0, False),
    "llama2_7b": HeadConfig("llama2_7b", "bf16", 4096, 32000, 16, 2, (1, 4, 8), 10, 1, True),
    "llama3_8b": HeadConfig("llama3_8b", "bf16", 4096, 128256, 32, 4, (1, 4, 8, 16), 10, 2, True),
    "qwen25_7b": HeadConfig("qwen25_7b", "bf16", 3584, 152064, 32, 4, (1, 8, 16), 10, 3, True),
    "wide_tree": HeadConfig("wide_tree", "bf16", 4096, 128256, 64, 8, (64,), 16, 4, True,
                            bias_std=2.0),
    # The paper's own best router setting at the Llama3 shape (Table 4: 16 groups, top 2) with
    # its equal contiguous split of the vocabulary and the appendix's 10 candidates per step,
    # and the same with permuted groups (gathered rows against contiguous rows).
    "paper_point": HeadConfig("paper_point", "bf16", 4096, 128256, 16, 2, (1, 10), 10, 5, True,
                              grouping="contiguous"),
    "paper_point_permuted": HeadConfig("paper_point_permuted", "bf16", 4096, 128256, 16, 2, (1, 10),
                                       10, 5, True),
    # ... and in the paper's storage type (appendix "Backends": FP16)
    "paper_point_f16": HeadConfig("paper_point_f16", "f16", 4096, 128256, 16, 2, (1, 10), 10, 5, True,
                                  grouping="contiguous"),
}


@dataclass
class Head:
    cfg: HeadConfig
    lm_W: np.ndarray            # [V,H] float32, or uint16 holding bf16 bits
    gate_W: np.ndarray          # [G,H] same storage
    gate_bias: Optional[np.ndarray]   # [G] float32 or None
    group_offsets: np.ndarray   # [G+1] int32
    group_rows: np.ndarray      # [V] int32


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, stream])))


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round to nearest, ties to even."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """float32 values in the storage type's representation (fp32 as is, bf16 / fp16 as their
    bit patterns in uint16, rounded to nearest even)."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return to_bf16_bits(x)
    if dtype == "f16":                             # IEEE binary16 bits, round to nearest even
        return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)
    raise ValueError(f"unknown dtype {dtype!r}")


def make_partition(cfg: HeadConfig):
    """CSR partition of the vocabulary into G equal groups."""
    if cfg.V % cfg.G:
        raise ValueError("V must be divisible by G for the equal split")
    v = cfg.v
    if cfg.grouping == "contiguous":
        perm = np.arange(cfg.V, dtype=np.int64)
    elif cfg.grouping == "permuted":
        perm = _rng(cfg.seed, 3).permutation(cfg.V)
    else:
        raise ValueError(f"unknown grouping {cfg.grouping!r}")
    rows = np.sort(perm.reshape(cfg.G, v), axis=1).reshape(-1).astype(np.int32)
    offsets = (np.arange(cfg.G + 1, dtype=np.int64) * v).astype(np.int32)
    return offsets, rows


def make_head(cfg: HeadConfig) -> Head:
    r0 = _rng(cfg.seed, 0)
    store_dt = np.float32 if cfg.dtype == "f32" else np.uint16
    lm_W = np.empty((cfg.V, cfg.H), dtype=store_dt)
    for lo in range(0, cfg.V, _ROW_BLOCK):
        hi = min(cfg.V, lo + _ROW_BLOCK)
        blk = r0.standard_normal((hi - lo, cfg.H), dtype=np.float32)
        blk *= np.float32(0.02)
        lm_W[lo:hi] = to_storage(blk, cfg.dtype)
    gw = _rng(cfg.seed, 1).standard_normal((cfg.G, cfg.H), dtype=np.float32) * np.float32(0.02)
    gate_W = to_storage(gw, cfg.dtype)
    gate_bias = None
    if cfg.bias_std > 0:
        gate_bias = (_rng(cfg.seed, 2).standard_normal(cfg.G, dtype=np.float32)
                     * np.float32(cfg.bias_std)).astype(np.float32)
    offsets, rows = make_partition(cfg)
    return Head(cfg, lm_W, gate_W, gate_bias, offsets, rows)


def make_router_W1(cfg: HeadConfig) -> np.ndarray:
    """The router's square projection W1 [H,H] (row = output feature) in the config's storage type."""
    w = _rng(cfg.seed, 4).standard_normal((cfg.H, cfg.H), dtype=np.float32) * np.float32(0.02)
    return to_storage(w, cfg.dtype)


def make_hidden(cfg: HeadConfig, M: int, batch: int = 0) -> np.ndarray:
    """One batch of M draft hidden states, [M,H] in the config's storage type."""
    x = _rng(cfg.seed, 16 + batch).standard_normal((M, cfg.H), dtype=np.float32)
    if cfg.unit_rms:
        rms = np.sqrt(np.mean(x.astype(np.float64) ** 2, axis=1, keepdims=True))
        x = (x / rms).astype(np.float32)
    return to_storage(x, cfg.dtype)
