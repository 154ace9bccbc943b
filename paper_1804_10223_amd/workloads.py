"""Seeded synthetic workloads for the sparse persistent recurrent step.

This module only draws random inputs (sparsity patterns, weight values, input
projections, initial states).  It contains none of the method's arithmetic and
is the one module that the CPU oracle's tests and the HIP path's tests both
use, so that both see bit-identical inputs.

The shapes follow the paper's workloads (Section 5.1): pruned recurrent layers
of 1k-6k units at 70-99 % sparsity with an unstructured random pattern (the
paper's own timing runs use a random, unstructured nonzero pattern, Appendix
B.2), batch 1-8, tens to hundreds of timesteps.  The five named configurations
are the ones this repository is measured on.

Draw order per workload (one ``numpy.random.Generator(PCG64(seed))``):
  1. per-row nonzero counts (only for ``row_nnz="poisson"``),
  2. per-row column choice: ``rng.random(H)`` keys, the ``k`` smallest keys'
     indices, sorted ascending,
  3. all nonzero values: ``standard_normal(nnz, float32) / sqrt(k_row) * gain``,
     rounded once to binary16 (round-to-nearest-even, subnormals kept),
  4. ``x``: ``standard_normal((T, B, R), float32)`` (+1.0 on the forget block
     of an LSTM: the forget-gate bias folded into b' of Eq. 2),
  5. ``h0``: ``normal(0, h0_std)`` if ``h0_std > 0`` else absent (zeros),
  6. GRU only: ``b_hn``: ``normal(0, 0.5)`` of length H.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

CELL_RNN_RELU = "relu"
CELL_RNN_TANH = "tanh"
CELL_RNN_IDENTITY = "identity"
CELL_LSTM = "lstm"
CELL_GRU = "gru"
GATES = {CELL_LSTM: 4, CELL_GRU: 3}   # gate rows per hidden unit


@dataclass
class Workload:
    name: str
    cell: str                 # "relu" | "tanh" | "identity" | "lstm" | "gru"
    hidden: int               # H
    batch: int                # B
    steps: int                # T
    row_ptr: np.ndarray       # int32 [R+1], R = H (RNN), 4H (LSTM) or 3H (GRU)
    col_idx: np.ndarray       # int32 [nnz], strictly increasing inside a row
    val_bits: np.ndarray      # uint16 [nnz], IEEE binary16 bit patterns
    x: np.ndarray             # float32 [T, B, R]
    h0: Optional[np.ndarray]  # float32 [B, H] or None (zeros)
    c0: Optional[np.ndarray] = None  # float32 [B, H] or None (zeros); LSTM only
    b_hn: Optional[np.ndarray] = None  # float32 [H]; GRU only: recurrent bias of the candidate gate
    meta: dict = field(default_factory=dict)

    @property
    def rows(self) -> int:
        return self.hidden * GATES.get(self.cell, 1)

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1])


def draw_pattern(rng: np.random.Generator, rows: int, cols: int, counts: np.ndarray):
    """Uniform random column subsets, ``counts[r]`` distinct columns in row r, ascending."""
    counts = np.asarray(counts, dtype=np.int64)
    row_ptr = np.zeros(rows + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    col_idx = np.empty(int(row_ptr[-1]), dtype=np.int32)
    chunk = max(1, min(rows, (32 << 20) // max(cols, 1)))
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        keys = rng.random((r1 - r0, cols), dtype=np.float32)
        order = np.argsort(keys, axis=1, kind="stable")
        for r in range(r0, r1):
            k = int(counts[r])
            col_idx[row_ptr[r]:row_ptr[r + 1]] = np.sort(order[r - r0, :k])
    return row_ptr.astype(np.int32), col_idx


def make_workload(name: str, cell: str, hidden: int, batch: int, steps: int, density: float,
                  seed: int = 0, gain: float = 0.9, row_nnz: str = "fixed",
                  h0_std: float = 0.0, forget_bias: float = 1.0) -> Workload:
    rng = np.random.Generator(np.random.PCG64(seed))
    rows = hidden * GATES.get(cell, 1)
    k_mean = density * hidden
    if row_nnz == "fixed":
        counts = np.full(rows, int(round(k_mean)), dtype=np.int64)
    elif row_nnz == "poisson":
        counts = np.clip(rng.poisson(k_mean, size=rows), 0, hidden).astype(np.int64)
    else:
        raise ValueError(row_nnz)
    row_ptr, col_idx = draw_pattern(rng, rows, hidden, counts)
    nnz = int(row_ptr[-1])
    per_nnz_count = np.repeat(np.maximum(counts, 1), counts).astype(np.float32)
    vals = rng.standard_normal(nnz, dtype=np.float32) / np.sqrt(per_nnz_count) * np.float32(gain)
    val_bits = vals.astype(np.float16).view(np.uint16).copy()
    x = rng.standard_normal((steps, batch, rows), dtype=np.float32)
    if cell == CELL_LSTM and forget_bias != 0.0:
        x[:, :, hidden:2 * hidden] += np.float32(forget_bias)
    h0 = None
    if h0_std > 0.0:
        h0 = (rng.standard_normal((batch, hidden), dtype=np.float32) * np.float32(h0_std)).astype(np.float32)
    b_hn = None
    if cell == CELL_GRU:
        b_hn = (rng.standard_normal(hidden, dtype=np.float32) * np.float32(0.5)).astype(np.float32)
    return Workload(name=name, cell=cell, hidden=hidden, batch=batch, steps=steps,
                    row_ptr=row_ptr, col_idx=col_idx, val_bits=val_bits, x=x, h0=h0, c0=None, b_hn=b_hn,
                    meta=dict(density=density, seed=seed, gain=gain, row_nnz=row_nnz, h0_std=h0_std))


# The five measured configurations.
CONFIGS = {
    "cfg1": dict(cell=CELL_RNN_RELU, hidden=256, batch=1, steps=16, density=0.10, gain=0.9),
    "cfg2": dict(cell=CELL_RNN_RELU, hidden=1152, batch=4, steps=256, density=0.10, gain=0.9, h0_std=0.1),
    "cfg3": dict(cell=CELL_RNN_RELU, hidden=2304, batch=4, steps=256, density=0.30, gain=0.9),
    "cfg4": dict(cell=CELL_RNN_RELU, hidden=5760, batch=2, steps=128, density=0.10, gain=0.9, row_nnz="poisson"),
    "cfg5": dict(cell=CELL_LSTM, hidden=1024, batch=8, steps=128, density=0.20, gain=1.0),
}


def make_config(name: str, seed: int = 0, steps: Optional[int] = None) -> Workload:
    """One of the five measured configurations ("cfg1".."cfg5"); ``steps`` overrides T."""
    kw = dict(CONFIGS[name])
    if steps is not None:
        kw["steps"] = steps
    return make_workload(name, seed=seed, **kw)


@dataclass
class Projection:
    """Inputs of the step before the recurrence (Section 3.1): b' = W_in x + b for all timesteps."""
    rows: int                 # R: H, or 4H for an LSTM (gate blocks i | f | g | o)
    input_size: int           # I
    w_bits: np.ndarray        # uint16 [R, I], dense IEEE binary16 bit patterns
    bias: np.ndarray          # float32 [R]
    x_in: np.ndarray          # float32 [T, B, I]


def make_projection(rows: int, input_size: int, steps: int, batch: int, seed: int = 0, x_scale: float = 1.0,
                    forget_block: Optional[tuple] = None, forget_bias: float = 1.0) -> Projection:
    """Dense input weights N(0, 1/I) rounded once to binary16, bias N(0, 0.1^2) (+forget_bias on rows
    forget_block = (first, last)), inputs N(0, x_scale^2); drawn in that order from PCG64(seed)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    w = rng.standard_normal((rows, input_size), dtype=np.float32) / np.float32(np.sqrt(input_size))
    w_bits = w.astype(np.float16).view(np.uint16).copy()
    bias = (rng.standard_normal(rows, dtype=np.float32) * np.float32(0.1)).astype(np.float32)
    if forget_block is not None:
        bias[forget_block[0]:forget_block[1]] += np.float32(forget_bias)
    x_in = (rng.standard_normal((steps, batch, input_size), dtype=np.float32) * np.float32(x_scale)).astype(np.float32)
    return Projection(rows=rows, input_size=input_size, w_bits=w_bits, bias=bias, x_in=x_in)


def csr_from_dense(dense_fp16: np.ndarray):
    """CSR (row_ptr, col_idx, val_bits) of the nonzero pattern of a float16 matrix; stored zeros are dropped."""
    dense_fp16 = np.asarray(dense_fp16, dtype=np.float16)
    rows, _ = dense_fp16.shape
    bits = dense_fp16.view(np.uint16)
    mask = (bits & 0x7FFF) != 0
    counts = mask.sum(axis=1)
    row_ptr = np.zeros(rows + 1, dtype=np.int32)
    np.cumsum(counts, out=row_ptr[1:])
    r, c = np.nonzero(mask)
    return row_ptr, c.astype(np.int32), bits[r, c].astype(np.uint16)
