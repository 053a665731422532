"""Seeded synthetic inputs for the rotate-and-quantize path.

This module only *draws numbers*: it holds none of the method's arithmetic (no
Hadamard matrix, no quantizer, no packing).  Both the CPU oracle's tests and the
GPU path's tests/benchmark take their inputs from here, so the two sides see the
same bits.

The paper's real workloads are activations and KV caches of 7-8B LLMs on WikiText2
(paper section 5.1); neither models nor data are available, so each workload below
is a stand-in with the same shape and the structure the paper describes for LLM
activations (section 2.2: heavy tails, a few outlier channels, a few massive
tokens).

Rows are generated in independent blocks of ``BLOCK_ROWS`` rows, each from its own
PCG64 stream keyed by (seed, block index); the per-tensor structure (which
channels are outliers, which rows are massive) comes from a stream keyed by
(seed, STRUCT_KEY).  A sampled subset of a very large tensor can therefore be
regenerated without drawing the whole tensor.

bf16 tensors are returned as uint16 bit patterns (numpy has no bf16 type).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

BLOCK_ROWS = 256
STRUCT_KEY = 0x5EED5


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


@dataclass(frozen=True)
class Workload:
    """One synthetic tensor: ``rows`` token rows of width ``d`` rotated at order ``n``."""
    name: str
    rows: int
    d: int
    n: int
    dtype: str            # "bf16" | "f32"
    bits: tuple           # bit-widths the config is quantized at
    clip: float
    seed: int
    recipe: str           # "normal_outlier" | "student_t" | "swiglu" | "kv_k" | "kv_v"
    n_outlier_ch: int = 0
    outlier_scale: float = 1.0
    n_massive_rows: int = 0
    massive_scale: float = 1.0
    head_rows: int = 0    # kv only: rows per (batch, head) = sequence length

    def with_rows(self, rows: int) -> "Workload":
        """Same per-row distribution with a different number of rows."""
        return Workload(**{**self.__dict__, "rows": int(rows)})


# The five benchmark configurations (index = configuration number; 3 and 4 have two
# tensors each).  Values marked (*) are choices made where the configuration list is
# silent.
WORKLOADS = {
    "tiny": Workload("tiny", 64, 256, 256, "f32", (3,), 1.0, 0, "normal_outlier",
                     n_outlier_ch=4, outlier_scale=30.0),
    "llama_hidden": Workload("llama_hidden", 2048, 4096, 4096, "bf16", (4, 3), 0.9, 100,
                             "student_t", n_outlier_ch=8, outlier_scale=50.0,
                             n_massive_rows=2, massive_scale=500.0),
    "qwen_hidden": Workload("qwen_hidden", 4096, 3584, 3584, "bf16", (3,), 0.9, 200,
                            "student_t", n_outlier_ch=8, outlier_scale=50.0,
                            n_massive_rows=2, massive_scale=500.0),
    "ffn_down": Workload("ffn_down", 4096, 18944, 18944, "bf16", (3,), 0.9, 300, "swiglu"),
    "ffn_expand": Workload("ffn_expand", 4096, 3000, 3072, "bf16", (3,), 0.9, 301, "swiglu"),
    # K and V: [16 batch x 32 heads x 8192 seq x 128]; one row = one (batch, head, position)
    "kv_k": Workload("kv_k", 16 * 32 * 8192, 128, 128, "bf16", (3,), 0.9, 400, "kv_k",
                     n_outlier_ch=2, outlier_scale=10.0, head_rows=8192),
    "kv_v": Workload("kv_v", 16 * 32 * 8192, 128, 128, "bf16", (3,), 0.9, 401, "kv_v",
                     head_rows=8192),
    "calib": Workload("calib", 512, 4096, 4096, "bf16", (3,), 0.9, 402, "student_t",
                      n_outlier_ch=8, outlier_scale=50.0,
                      n_massive_rows=2, massive_scale=500.0),
}


def clip_grid(k: int = 32, lo: float = 0.5, hi: float = 1.0) -> np.ndarray:
    """The calibration grid: ``k`` clip ratios evenly spaced in [lo, hi], as float32."""
    return (lo + (hi - lo) * np.arange(k, dtype=np.float64) / (k - 1)).astype(np.float32)


def _structure(w: Workload):
    rng = np.random.default_rng([w.seed, STRUCT_KEY])
    ch = rows = None
    if w.recipe in ("normal_outlier", "student_t") and w.n_outlier_ch:
        ch = np.sort(rng.choice(w.d, w.n_outlier_ch, replace=False))
    if w.n_massive_rows:
        rows = np.sort(rng.choice(w.rows, min(w.n_massive_rows, w.rows), replace=False))
    if w.recipe == "kv_k":
        # outlier channels differ per (batch, head)
        n_heads = max(1, -(-w.rows // w.head_rows))        # a last, partial head counts too
        ch = np.stack([np.sort(rng.choice(w.d, w.n_outlier_ch, replace=False))
                       for _ in range(n_heads)])
    return ch, rows


def _block_f32(w: Workload, blk: int, ch, massive_rows) -> np.ndarray:
    r0 = blk * BLOCK_ROWS
    nr = min(BLOCK_ROWS, w.rows - r0)
    rng = np.random.default_rng([w.seed, blk])
    if w.recipe == "normal_outlier":
        x = rng.standard_normal((nr, w.d), dtype=np.float32)
        x[:, ch] *= np.float32(w.outlier_scale)
    elif w.recipe == "student_t":
        x = rng.standard_t(3.0, size=(nr, w.d)).astype(np.float32)
        x[:, ch] *= np.float32(w.outlier_scale)
    elif w.recipe == "swiglu":
        g = rng.standard_normal((nr, w.d), dtype=np.float32)
        u = rng.standard_normal((nr, w.d), dtype=np.float32)
        x = (g / (1.0 + np.exp(-g))) * u
    elif w.recipe == "kv_k":
        x = rng.standard_normal((nr, w.d), dtype=np.float32)
        heads = (r0 + np.arange(nr)) // w.head_rows
        for h in np.unique(heads):
            sel = heads == h
            x[np.ix_(sel, ch[h])] *= np.float32(w.outlier_scale)
    elif w.recipe == "kv_v":
        x = rng.standard_normal((nr, w.d), dtype=np.float32)
    else:
        raise ValueError(w.recipe)
    if massive_rows is not None:
        for r in massive_rows:
            if r0 <= r < r0 + nr:
                x[r - r0] *= np.float32(w.massive_scale)
    return x


def n_blocks(w: Workload) -> int:
    return (w.rows + BLOCK_ROWS - 1) // BLOCK_ROWS


def generate_blocks(w: Workload, blocks) -> np.ndarray:
    """Rows of the given blocks, concatenated; float32 for "f32", uint16 bits for "bf16"."""
    ch, mrows = _structure(w)
    out = []
    for b in blocks:
        x = _block_f32(w, int(b), ch, mrows)
        out.append(x if w.dtype == "f32" else f32_to_bf16_bits(x))
    return np.concatenate(out, axis=0)


def generate(w: Workload, out: Optional[np.ndarray] = None) -> np.ndarray:
    """The whole tensor [rows, d] (row-major, leading dimension d)."""
    dt = np.float32 if w.dtype == "f32" else np.uint16
    if out is None:
        out = np.empty((w.rows, w.d), dtype=dt)
    ch, mrows = _structure(w)
    for b in range(n_blocks(w)):
        x = _block_f32(w, b, ch, mrows)
        out[b * BLOCK_ROWS: b * BLOCK_ROWS + x.shape[0]] = x if w.dtype == "f32" else f32_to_bf16_bits(x)
    return out


def block_row_index(blocks, w: Workload) -> np.ndarray:
    """Global row numbers of the rows ``generate_blocks(w, blocks)`` returns."""
    idx = []
    for b in blocks:
        r0 = int(b) * BLOCK_ROWS
        idx.append(np.arange(r0, min(r0 + BLOCK_ROWS, w.rows)))
    return np.concatenate(idx)
