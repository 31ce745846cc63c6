"""Seeded synthetic inputs for GQLA decode attention.

This module only draws random numbers and rounds them to the storage type; it
holds none of the method's arithmetic and imports neither the CPU oracle nor
the HIP binding.  Both sides consume exactly the bits produced here.

Recipe (one config = one seed):
  stream 0            up-projection weights  W_UK, W_UV ~ N(0, 1/r_kv)   [g, r_kv, d_h]
  stream 1            step queries           q_C, q_R   ~ N(0, 1)        [B, s_q, h_q, d]
  stream 2            per-sequence lengths and the page permutation
  stream 1000 + b     sequence b's cache rows  c_kv | k_R ~ N(0, 1)      [L_b, r_kv + d_r]
Values are drawn in fp32; for bf16 configs they are rounded once
(round-to-nearest-even) to bf16 and those bits are what every consumer sees.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np


@dataclass(frozen=True)
class GqlaConfig:
    name: str
    B: int
    h_q: int
    g: int
    d_h: int
    r_kv: int
    d_r: int
    s_q: int
    dtype: str            # "f32" or "bf16"
    seed: int
    L: int = 0            # uniform context length (includes the s_q step tokens); 0 => ragged
    L_min: int = 0
    L_max: int = 0
    page_size: int = 64
    paged: bool = False   # True => randomly permuted page table
    d_v: int = 0          # per-head value dim; 0 => d_h

    @property
    def dv(self) -> int:
        return self.d_v if self.d_v > 0 else self.d_h

    @property
    def G(self) -> int:
        return self.h_q // self.g

    def with_(self, **kw) -> "GqlaConfig":
        return replace(self, **kw)


# The five workload shapes (index k uses seed 15250 + k).
CONFIGS = {
    "C0": GqlaConfig("C0", B=1, h_q=8, g=2, d_h=16, r_kv=32, d_r=8, s_q=1, dtype="f32",
                     seed=15250, L=64, page_size=16),
    "C1": GqlaConfig("C1", B=32, h_q=32, g=8, d_h=128, r_kv=512, d_r=64, s_q=1, dtype="bf16",
                     seed=15251, L=4096),
    "C2": GqlaConfig("C2", B=64, h_q=128, g=8, d_h=128, r_kv=512, d_r=64, s_q=1, dtype="bf16",
                     seed=15252, L=8192),
    "C3": GqlaConfig("C3", B=64, h_q=128, g=8, d_h=128, r_kv=512, d_r=64, s_q=2, dtype="bf16",
                     seed=15253, L=8192),
    "C4": GqlaConfig("C4", B=128, h_q=128, g=8, d_h=128, r_kv=512, d_r=64, s_q=2, dtype="bf16",
                     seed=15254, L_min=1024, L_max=32768, paged=True),
}


def rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.default_rng([seed, stream])


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern (uint16), round-to-nearest-even.  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(x: np.ndarray, dtype: str) -> np.ndarray:
    """Return the fp32 array holding exactly the values the storage type can represent."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(round_to_bf16_bits(x))
    raise ValueError(dtype)


def weights(cfg: GqlaConfig):
    r = rng(cfg.seed, 0)
    std = np.float32(cfg.r_kv ** -0.5)
    w_uk = r.standard_normal((cfg.g, cfg.r_kv, cfg.d_h), dtype=np.float32) * std
    w_uv = r.standard_normal((cfg.g, cfg.r_kv, cfg.dv), dtype=np.float32) * std
    return quantize(w_uk, cfg.dtype), quantize(w_uv, cfg.dtype)


def output_weights(cfg: GqlaConfig, d_model: int) -> np.ndarray:
    """W^O [d_model, h_q * d_h], storage-rounded."""
    r = rng(cfg.seed, 3)
    K = cfg.h_q * cfg.dv
    return quantize(r.standard_normal((int(d_model), K), dtype=np.float32) * np.float32(K ** -0.5), cfg.dtype)


def queries(cfg: GqlaConfig):
    r = rng(cfg.seed, 1)
    q_c = r.standard_normal((cfg.B, cfg.s_q, cfg.h_q, cfg.d_h), dtype=np.float32)
    q_r = r.standard_normal((cfg.B, cfg.s_q, cfg.h_q, cfg.d_r), dtype=np.float32)
    return quantize(q_c, cfg.dtype), quantize(q_r, cfg.dtype)


def seq_lens(cfg: GqlaConfig) -> np.ndarray:
    if cfg.L:
        return np.full((cfg.B,), cfg.L, dtype=np.int32)
    r = rng(cfg.seed, 2)
    return r.integers(cfg.L_min, cfg.L_max + 1, size=cfg.B).astype(np.int32)


def page_table(cfg: GqlaConfig, lens: np.ndarray):
    """(table int32[B, max_pages], num_pages).  Unused entries hold -1.

    paged=False: sequence b owns pages b*max_pages .. (identity).  paged=True: the
    pages the sequences need are one random permutation of 0..num_pages-1.
    """
    P = cfg.page_size
    need = (lens.astype(np.int64) + P - 1) // P
    max_pages = int(need.max())
    table = np.full((cfg.B, max_pages), -1, dtype=np.int32)
    if not cfg.paged:
        for b in range(cfg.B):
            table[b, : need[b]] = b * max_pages + np.arange(need[b])
        return table, cfg.B * max_pages
    total = int(need.sum())
    r = rng(cfg.seed, 2)
    r.integers(0, 2, size=cfg.B)          # keep the length draw and the permutation on separate states
    perm = r.permutation(total).astype(np.int32)
    at = 0
    for b in range(cfg.B):
        table[b, : need[b]] = perm[at: at + need[b]]
        at += int(need[b])
    return table, total


def sequence_rows(cfg: GqlaConfig, b: int, L_b: int) -> np.ndarray:
    """Cache rows of sequence b: fp32 array [L_b, r_kv + d_r] = c_kv | k_R, storage-rounded."""
    r = rng(cfg.seed, 1000 + b)
    rows = r.standard_normal((int(L_b), cfg.r_kv + cfg.d_r), dtype=np.float32)
    return quantize(rows, cfg.dtype)
