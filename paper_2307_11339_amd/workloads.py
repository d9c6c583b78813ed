"""Seeded synthetic workloads for the stacked-RNN forward pass.

This module only draws numbers and rounds them to the storage type. It contains none of
the RNN arithmetic, so both the CPU oracle's tests and the GPU path's tests can share it.

The paper evaluates on synthetic LSTM shapes described by the tuple
<num_of_layers, batch_size, io_size, seq_len> (Section 6.2, Table 6) and uses no dataset;
the five named configurations below follow the same idea at the sizes this library targets.

Draw order (fixed, one numpy PCG64 stream per workload):
    for layer l, for direction d:  W_ih, W_hh, b_ih, b_hh   each U(-k, k), k = 1/sqrt(H)
    x ~ N(0, 1)                    [T, B, I]
    h0 ~ N(0, h0_std) (if h0_std > 0, else zeros)   [L*D, B, H]
    c0 = zeros                     [L*D, B, H]
    lengths ~ U{len_min..T} (if len_min is set, else all T)
Values are drawn in float64, cast to float32 and, for bf16 workloads, rounded to bf16 with
round-to-nearest-even; every consumer receives the rounded values, so all sides see the
same stored bits.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional

import numpy as np

LSTM = 0
GRU = 1
F32 = 0
BF16 = 1

BASE_SEED = 230711339


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def round_to_storage(a: np.ndarray, dtype: int) -> np.ndarray:
    """float64 draw -> float32 value that is exactly representable in the storage type."""
    a32 = np.asarray(a, dtype=np.float64).astype(np.float32)
    if dtype == BF16:
        return bf16_bits_to_f32(f32_to_bf16_bits(a32))
    return a32


@dataclass(frozen=True)
class Config:
    name: str
    cell: int
    L: int
    D: int
    I: int
    H: int
    T: int
    B: int
    dtype: int
    seed: int
    h0_std: float = 0.0
    len_min: Optional[int] = None  # None: every sequence has length T

    @property
    def G(self) -> int:
        return 4 if self.cell == LSTM else 3

    def layer_input(self, l: int) -> int:
        return self.I if l == 0 else self.D * self.H

    def scaled(self, **kw) -> "Config":
        return replace(self, **kw)


# The five named workloads (C1..C5).
CONFIGS = {
    "C1": Config("C1", LSTM, L=1, D=1, I=64, H=128, T=32, B=1, dtype=F32, seed=BASE_SEED + 1),
    "C2": Config("C2", GRU, L=2, D=1, I=256, H=512, T=100, B=8, dtype=BF16, seed=BASE_SEED + 2,
                 h0_std=0.1),
    "C3": Config("C3", LSTM, L=4, D=1, I=1024, H=1024, T=128, B=1, dtype=BF16, seed=BASE_SEED + 3),
    "C4": Config("C4", LSTM, L=2, D=2, I=512, H=512, T=256, B=64, dtype=BF16, seed=BASE_SEED + 4,
                 len_min=64),
    "C5": Config("C5", LSTM, L=8, D=1, I=1024, H=1024, T=512, B=256, dtype=BF16,
                 seed=BASE_SEED + 5),
}


def paper_grid() -> List[Config]:
    """The paper's own model grid (Table 6): baseline <12 layers, batch 8, io 64, seq 96> and
    twelve one-parameter variants, unidirectional LSTM, fp32, io_size = input = hidden."""
    base = dict(L=12, B=8, H=64, T=96)
    variants = [dict()]
    variants += [dict(L=v) for v in (4, 8, 16)]
    variants += [dict(B=v) for v in (1, 2, 4, 16)]
    variants += [dict(H=v) for v in (32, 128)]
    variants += [dict(T=v) for v in (32, 64, 128)]
    out = []
    for i, v in enumerate(variants):
        p = {**base, **v}
        out.append(Config(f"P<{p['L']},{p['B']},{p['H']},{p['T']}>", LSTM, L=p["L"], D=1, I=p["H"],
                          H=p["H"], T=p["T"], B=p["B"], dtype=F32, seed=BASE_SEED + 100 + i))
    return out


@dataclass
class Workload:
    cfg: Config
    weights: List[np.ndarray]          # L*D*4 float32 arrays in order (l, d, {W_ih, W_hh, b_ih, b_hh})
    x: np.ndarray                      # [T, B, I] float32 (exactly representable in cfg.dtype)
    h0: Optional[np.ndarray]           # [L*D, B, H] float32 or None (zeros)
    c0: Optional[np.ndarray]           # [L*D, B, H] float32 or None (zeros)
    lengths: Optional[np.ndarray]      # [B] int32 or None (all T)
    meta: dict = field(default_factory=dict)

    def weight(self, l: int, d: int, which: int) -> np.ndarray:
        return self.weights[(l * self.cfg.D + d) * 4 + which]

    def take_batch(self, idx) -> "Workload":
        """The same workload restricted to the batch rows in idx (sequences are independent)."""
        idx = np.asarray(idx, dtype=np.int64)
        cfg = self.cfg.scaled(B=int(idx.size))
        return Workload(
            cfg=cfg,
            weights=self.weights,
            x=np.ascontiguousarray(self.x[:, idx, :]),
            h0=None if self.h0 is None else np.ascontiguousarray(self.h0[:, idx, :]),
            c0=None if self.c0 is None else np.ascontiguousarray(self.c0[:, idx, :]),
            lengths=None if self.lengths is None else np.ascontiguousarray(self.lengths[idx]),
            meta=dict(self.meta),
        )


def make_workload(cfg: Config, zero_pad_x: bool = True) -> Workload:
    rng = np.random.default_rng(cfg.seed)
    k = 1.0 / np.sqrt(cfg.H)
    weights: List[np.ndarray] = []
    for l in range(cfg.L):
        il = cfg.layer_input(l)
        for _d in range(cfg.D):
            for shape in ((cfg.G * cfg.H, il), (cfg.G * cfg.H, cfg.H), (cfg.G * cfg.H,),
                          (cfg.G * cfg.H,)):
                weights.append(round_to_storage(rng.uniform(-k, k, size=shape), cfg.dtype))
    x = round_to_storage(rng.standard_normal(size=(cfg.T, cfg.B, cfg.I)), cfg.dtype)
    h0 = None
    if cfg.h0_std > 0:
        h0 = (rng.standard_normal(size=(cfg.L * cfg.D, cfg.B, cfg.H)) * cfg.h0_std).astype(np.float32)
    c0 = None
    lengths = None
    if cfg.len_min is not None:
        lengths = rng.integers(cfg.len_min, cfg.T + 1, size=cfg.B).astype(np.int32)
        if zero_pad_x:
            for b in range(cfg.B):
                x[int(lengths[b]):, b, :] = 0.0
    return Workload(cfg, weights, x, h0, c0, lengths)
