"""Seeded synthetic inputs for masked multi-head attention.

This module only *produces inputs*: mask descriptions, dense boolean masks built
from them, and Q/K/V tensors as raw fp16/bf16 bit patterns.  It holds none of the
attention arithmetic and none of the sparse-format logic, so that both the CPU
oracle and the HIP library can be fed the very same bytes.

Mask patterns follow the atomic/compound patterns of the paper (Sec. 2.1.2,
Fig. 1: causal, global, sliding window, random; Longformer and BigBird as
compounds) and Table 2 (band width = half-width on each side of the diagonal).

Mask composition rule (this build's definition, mirrored by the library's
description-based planner):

    M = (WINDOW or GLOBAL or STRIDED or BLOCK_RANDOM or BIGBIRD   [all-ones if none set])
        and CAUSAL (if set) and PADDING (if set)

Random components are drawn from a counter-based generator (splitmix64 finaliser
over (seed, head, block_row, block_col)) so that any implementation can
reproduce them without sharing state.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional, Sequence

import numpy as np

# flag bits (same numeric values as SMHA_MASK_* in include/smha.h)
CAUSAL = 1
WINDOW = 2
GLOBAL = 4
STRIDED = 8
BLOCK_RANDOM = 16
BIGBIRD = 32
PADDING = 64

_M64 = (1 << 64) - 1


def mix64(x: int) -> int:
    """splitmix64 output function on a Python int (mod 2^64)."""
    x = (x + 0x9E3779B97F4A7C15) & _M64
    z = x
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def block_hash(seed: int, head: int, br: int, bc: int) -> int:
    """64-bit hash of (seed, head, block_row, block_col)."""
    key = mix64((seed & _M64) ^ mix64(head))
    return mix64(key ^ (((br & 0xFFFFFFFF) << 32) | (bc & 0xFFFFFFFF)))


def hash_to_unit(h: int) -> float:
    """Top 53 bits of a hash as a double in [0, 1)."""
    return (h >> 11) * (1.0 / 9007199254740992.0)


@dataclass(frozen=True)
class MaskSpec:
    flags: int = 0
    window_left: int = 0      # keep j with i - j <= window_left
    window_right: int = 0     # keep j with j - i <= window_right
    n_global: int = 0         # rows < n_global and cols < n_global fully kept
    stride: int = 0           # keep j with j % stride == stride_phase
    stride_phase: int = 0
    block: int = 64           # block edge of BLOCK_RANDOM / BIGBIRD components
    keep_p: float = 0.0       # BLOCK_RANDOM: block kept iff u(hash) < keep_p, diagonal always
    n_window_blocks: int = 0  # BIGBIRD: odd count of block columns centred on the diagonal
    n_global_blocks: int = 0  # BIGBIRD: first block rows and block cols fully kept
    n_random_blocks: int = 0  # BIGBIRD: extra block cols per block row, smallest hash first
    seed: int = 0
    per_head: bool = False    # random components differ per head
    valid_len: Optional[tuple] = None  # PADDING: per-batch count of real tokens

    def n_batch_masks(self, B: int) -> int:
        return B if (self.flags & PADDING) and self.valid_len is not None and B > 1 else 1

    def n_head_masks(self, H: int) -> int:
        has_random = self.flags & (BLOCK_RANDOM | BIGBIRD)
        return H if (self.per_head and has_random) else 1


def mask_rows(spec: MaskSpec, S: int, head: int, valid: int, rows) -> np.ndarray:
    """bool [len(rows), S]: the given query rows of the S x S mask (the composition rule above,
    evaluated only where asked: long sequences never need the whole matrix)."""
    rows = np.asarray(rows, dtype=np.int64)
    i = rows[:, None]
    j = np.arange(S)[None, :]
    f = spec.flags
    additive = f & (WINDOW | GLOBAL | STRIDED | BLOCK_RANDOM | BIGBIRD)
    if not additive:
        m = np.ones((len(rows), S), dtype=bool)
    else:
        m = np.zeros((len(rows), S), dtype=bool)
    if f & WINDOW:
        m |= ((i - j) <= spec.window_left) & ((j - i) <= spec.window_right)
    if f & GLOBAL:
        m |= (i < spec.n_global) | (j < spec.n_global)
    if f & STRIDED:
        m |= (j % spec.stride) == spec.stride_phase
    if f & (BLOCK_RANDOM | BIGBIRD):
        bs = spec.block
        nb = -(-S // bs)
        keep = {}
        for br in sorted(set(int(r) // bs for r in rows)):
            row = np.zeros(nb, dtype=bool)
            if f & BLOCK_RANDOM:
                for bc in range(nb):
                    if br == bc or hash_to_unit(block_hash(spec.seed, head, br, bc)) < spec.keep_p:
                        row[bc] = True
            if f & BIGBIRD:
                big = np.zeros(nb, dtype=bool)
                half = (spec.n_window_blocks - 1) // 2
                if spec.n_window_blocks > 0:
                    big[max(0, br - half):min(nb, br + half + 1)] = True
                big[:min(nb, spec.n_global_blocks)] = True
                if br < spec.n_global_blocks:
                    big[:] = True
                cand = [bc for bc in range(nb) if not big[bc]]
                cand.sort(key=lambda bc: (block_hash(spec.seed, head, br, bc), bc))
                for bc in cand[:spec.n_random_blocks]:
                    big[bc] = True
                row |= big
            keep[br] = np.repeat(row, bs)[:S]
        for t, r in enumerate(rows):
            m[t] |= keep[int(r) // bs]
    if f & CAUSAL:
        m &= j <= i
    if f & PADDING:
        m &= (i < valid) & (j < valid)
    return m


def _one_mask(spec: MaskSpec, S: int, head: int, valid: int) -> np.ndarray:
    return mask_rows(spec, S, head, valid, np.arange(S))


def dense_mask(spec: MaskSpec, B: int, H: int, S: int) -> np.ndarray:
    """uint8 [Bm, Hm, S, S], 1 = attend.  Bm in {1, B}, Hm in {1, H}."""
    Bm, Hm = spec.n_batch_masks(B), spec.n_head_masks(H)
    out = np.empty((Bm, Hm, S, S), dtype=np.uint8)
    for b in range(Bm):
        valid = S
        if (spec.flags & PADDING) and spec.valid_len is not None:
            valid = int(spec.valid_len[b if Bm > 1 else 0])
        for h in range(Hm):
            out[b, h] = _one_mask(spec, S, h if Hm > 1 else 0, valid)
    return out


# ---------------------------------------------------------------------------
# Q/K/V as raw 16-bit patterns
# ---------------------------------------------------------------------------

def f64_to_f16_bits(x: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(x).astype(np.float16).view(np.uint16)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round to bfloat16 (nearest even on the float32 bit pattern)."""
    u = np.ascontiguousarray(x).astype(np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    return r.astype(np.uint16)


def bits_to_f64(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of fp16/bf16 bit patterns (used by tests for reporting)."""
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def qkv_bits(B: int, H: int, S: int, d: int, dtype: str, std: float, seed: int):
    """Three uint16 arrays [B, H, S, d]: Q, K, V ~ N(0, std^2) rounded to dtype."""
    rng = np.random.Generator(np.random.PCG64(seed))
    conv = f64_to_f16_bits if dtype == "f16" else f64_to_bf16_bits
    out = []
    for _ in range(3):
        x = rng.standard_normal((B, H, S, d)) * std
        out.append(conv(x))
    return tuple(out)


# ---------------------------------------------------------------------------
# The five benchmark configurations
# ---------------------------------------------------------------------------

@dataclass(frozen=True)
class Config:
    name: str
    B: int
    H: int
    S: int
    d: int
    dtype: str         # "f16" | "bf16"
    std: float
    mask: MaskSpec
    block: int = 64    # block size of the block-sparse format
    seed: int = 0


def _pad_lengths(seed: int, B: int, S: int, max_pad: int) -> tuple:
    return tuple(S - (mix64(mix64(seed) ^ (0x70616421 + b)) % (max_pad + 1)) for b in range(B))


def config(idx: int) -> Config:
    """idx in 1..5: the configurations this build is measured on."""
    if idx == 1:
        return Config("cfg1_tiny_window", 1, 2, 128, 64, "f16", 1.0,
                      MaskSpec(flags=WINDOW, window_left=16, window_right=16), 64, seed=1)
    if idx == 2:
        return Config("cfg2_longformer_bert", 8, 12, 512, 64, "f16", 1.0,
                      MaskSpec(flags=WINDOW | GLOBAL, window_left=64, window_right=64, n_global=8),
                      32, seed=2)
    if idx == 3:
        return Config("cfg3_strided_causal", 4, 16, 2048, 64, "f16", 1.0,
                      MaskSpec(flags=CAUSAL | WINDOW | STRIDED, window_left=127, window_right=0,
                               stride=128, stride_phase=0), 64, seed=3)
    if idx == 4:
        return Config("cfg4_random_blocks", 2, 16, 4096, 64, "bf16", 1.0,
                      MaskSpec(flags=BLOCK_RANDOM, block=64, keep_p=0.10, seed=4, per_head=True),
                      64, seed=4)
    if idx == 5:
        S = 8192
        return Config("cfg5_bigbird_8k", 1, 32, S, 128, "f16", 0.5,
                      MaskSpec(flags=BIGBIRD | PADDING, block=64, n_window_blocks=3,
                               n_global_blocks=2, n_random_blocks=3, seed=5,
                               valid_len=_pad_lengths(5, 1, S, 1023)), 64, seed=5)
    raise ValueError("config index must be 1..5")


def scaled(cfg: Config, **kw) -> Config:
    """A copy of a configuration with some fields replaced (smaller test variants)."""
    return replace(cfg, **kw)


# Table 2 patterns of the paper at sequence length 1024 (band = global = 32, fill 10 %).
def table2_spec(name: str) -> MaskSpec:
    if name == "causal":
        return MaskSpec(flags=CAUSAL)
    if name == "sliding_window":
        return MaskSpec(flags=WINDOW, window_left=32, window_right=32)
    if name == "longformer":
        return MaskSpec(flags=WINDOW | GLOBAL, window_left=32, window_right=32, n_global=32)
    if name == "bigbird":
        return MaskSpec(flags=WINDOW | GLOBAL | BLOCK_RANDOM, window_left=32, window_right=32,
                        n_global=32, block=32, keep_p=0.10, seed=1024)
    raise ValueError(name)


def scattered_spec(S: int, per_row: int, seed: int) -> "np.ndarray":
    """Dense mask with `per_row` pseudo-random columns per row plus the diagonal
    (a scattered, non-blocky pattern that favours the per-row format)."""
    m = np.zeros((1, 1, S, S), dtype=np.uint8)
    for i in range(S):
        m[0, 0, i, i] = 1
        for t in range(per_row):
            m[0, 0, i, block_hash(seed, 0, i, t) % S] = 1
    return m
