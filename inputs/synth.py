"""Synthetic stand-ins for the LLaMA-3.2 weight matrices the paper compresses (Table 1 models).

Shapes are the linear layers of LLaMA-3.2-1B / 3B (PyTorch ``Linear.weight`` order, rows = out
features, y = W x).  Values are i.i.d. draws: fp32 ``0.02 * N(0,1)`` or ``0.02 * t_4``.
Activations are ``N(0,1)`` rounded to bf16 (round-to-nearest-even), handed out both as raw
bf16 bit patterns (uint16) and as the exactly equal fp32 values.

Seeds: weights ``1000 * config + matrix_index``; activations ``+ 500_000``.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np


@dataclass(frozen=True)
class MatrixSpec:
    config: int        # 1..5
    index: int         # position in the config's ordered matrix list
    name: str          # e.g. "L03.gate_proj"
    rows: int
    cols: int
    dist: str          # "normal" | "student_t4"

    @property
    def weight_seed(self) -> int:
        return 1000 * self.config + self.index

    @property
    def act_seed(self) -> int:
        return 1000 * self.config + self.index + 500_000


def _layer(hidden: int, kv: int, inter: int):
    return [
        ("q_proj", hidden, hidden),
        ("k_proj", kv, hidden),
        ("v_proj", kv, hidden),
        ("o_proj", hidden, hidden),
        ("gate_proj", inter, hidden),
        ("up_proj", inter, hidden),
        ("down_proj", hidden, inter),
    ]


_L1B = _layer(2048, 512, 8192)
_L3B = _layer(3072, 1024, 8192)

CONFIGS = {
    1: dict(desc="single 2048x2048", dist="normal", batches=(1,)),
    2: dict(desc="one LLaMA-3.2-1B layer", dist="normal", batches=(1,)),
    3: dict(desc="LLaMA-3.2-1B decode-step sweep", dist="normal", batches=(1,)),
    4: dict(desc="LLaMA-3.2-3B decode-step sweep", dist="normal", batches=(1, 8)),
    5: dict(desc="LLaMA-3.2-3B shapes, Student-t(4) weights", dist="student_t4", batches=(16,)),
}


def config_matrices(config: int) -> List[MatrixSpec]:
    """Ordered matrix list of one decode step for a config (per layer q,k,v,o,gate,up,down; lm_head last)."""
    dist = CONFIGS[config]["dist"]
    out: List[MatrixSpec] = []

    def add(name, r, c):
        out.append(MatrixSpec(config, len(out), name, r, c, dist))

    if config == 1:
        add("w", 2048, 2048)
    elif config == 2:
        for n, r, c in _L1B:
            add(n, r, c)
    elif config == 3:
        for layer in range(16):
            for n, r, c in _L1B:
                add(f"L{layer:02d}.{n}", r, c)
        add("lm_head", 128256, 2048)
    elif config in (4, 5):
        for layer in range(28):
            for n, r, c in _L3B:
                add(f"L{layer:02d}.{n}", r, c)
        add("lm_head", 128256, 3072)
    else:
        raise ValueError(f"unknown config {config}")
    return out


def make_weights(spec: MatrixSpec) -> np.ndarray:
    """fp32 [rows, cols] weights for one matrix, from its seed."""
    rng = np.random.Generator(np.random.PCG64(spec.weight_seed))
    n = spec.rows * spec.cols
    if spec.dist == "normal":
        w = rng.standard_normal(n, dtype=np.float32)
    elif spec.dist == "student_t4":
        w = rng.standard_t(4, n).astype(np.float32)
    else:
        raise ValueError(spec.dist)
    w *= np.float32(0.02)
    return w.reshape(spec.rows, spec.cols)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even); returns the uint16 bit patterns.  Finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_activations(spec: MatrixSpec, batch: int):
    """Returns (bits uint16 [batch, cols], values fp32 [batch, cols]) — the same numbers in two dtypes."""
    rng = np.random.Generator(np.random.PCG64(spec.act_seed))
    x = rng.standard_normal((batch, spec.cols), dtype=np.float32)
    bits = f32_to_bf16_bits(x)
    return bits, bf16_bits_to_f32(bits)


def small_case(rows: int, cols: int, seed: int, dist: str = "normal") -> MatrixSpec:
    """A free-form small matrix for parity tests (config number 0 keeps its seeds apart from 1..5)."""
    return MatrixSpec(0, seed, f"small{rows}x{cols}", rows, cols, dist)
