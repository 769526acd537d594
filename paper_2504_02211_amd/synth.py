"""Seeded synthetic inputs and fault-candidate streams for fault-tolerant attention.

This module holds no attention or checksum arithmetic.  It produces

* Q, K, V tensors of the five benchmark workloads as 16-bit patterns (fp16 or
  bf16) in ``[batch, heads, seq, head_dim]`` layout, the tensor shape the paper
  uses for every attention operand (Section 3.1), and
* deterministic streams of *candidate* soft errors (single bit flips in a named
  fp32 intermediate, the fault model of Section 2.2 and the "one bit flip per
  attention computation" injection of Section 4.3).

Both the CPU oracle's tests and the GPU library's tests draw from here so that
the two sides see identical bits.  Everything is numpy; nothing here imports the
oracle or the GPU binding.
"""
from __future__ import annotations

import dataclasses
from typing import Iterator, List, Optional, Tuple

import numpy as np

F16 = 0
BF16 = 1

# Injection stages: the fp32 intermediates a compute-unit fault can hit.
ST_S = 0       # raw score accumulator of GEMM I
ST_EXP = 1     # exp(S - m)
ST_ROWSUM = 2  # running row-sum l
ST_OACC = 3    # un-normalised output accumulator of GEMM II
STAGE_NAMES = ("S", "EXP", "ROWSUM", "OACC")

DATA_SEED_BASE = 0xF7A77000
FAULT_SEED_BASE = 0xF7A7F000


@dataclasses.dataclass(frozen=True)
class Workload:
    """One benchmark configuration (shape, value recipe, mask, fault recipe)."""
    cfg: int
    name: str
    batch: int
    heads: int
    seq: int
    head_dim: int
    dtype: int            # F16 | BF16
    causal: bool
    value_scale: float    # multiplier applied to Q, K and V before rounding
    k_outlier_frac: float  # fraction of K rows (per head) multiplied by 8
    faults_per_head: int
    fault_stages: Tuple[int, ...]   # stages a fault slot may use
    one_per_stage: bool   # slot k is pinned to fault_stages[k]
    bit_lo: int
    bit_hi: int           # inclusive

    @property
    def useful_flops(self) -> float:
        f = 4.0 * self.batch * self.heads * float(self.seq) ** 2 * self.head_dim
        return f / 2 if self.causal else f


WORKLOADS = {
    1: Workload(1, "tiny", 1, 1, 128, 64, F16, False, 1.0, 0.0, 8,
                (ST_S, ST_EXP, ST_ROWSUM, ST_OACC), False, 20, 30),
    2: Workload(2, "encoder", 16, 12, 512, 64, F16, False, 0.125, 0.0, 1,
                (ST_S, ST_EXP, ST_ROWSUM, ST_OACC), False, 20, 30),
    3: Workload(3, "decoder-causal", 8, 16, 2048, 64, BF16, True, 1.0, 0.0, 1,
                (ST_S, ST_OACC), False, 20, 30),
    4: Workload(4, "large-head-causal", 4, 32, 4096, 128, BF16, True, 1.0, 0.01, 4,
                (ST_S, ST_EXP, ST_ROWSUM, ST_OACC), True, 20, 30),
    5: Workload(5, "long-sequence", 1, 32, 16384, 128, BF16, True, 1.0, 0.0, 1,
                (ST_EXP, ST_ROWSUM), False, 23, 30),
}


# ----------------------------------------------------------------------------
# 16-bit encodings
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    u = b.astype(np.uint32) << 16
    return u.view(np.float32).astype(np.float64)


def to_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    """Round real values to the 16-bit storage type; returns uint16 patterns."""
    if dtype == F16:
        return np.ascontiguousarray(x.astype(np.float16)).view(np.uint16)
    return f32_to_bf16_bits(x.astype(np.float32))


def bits_to_f64(b: np.ndarray, dtype: int) -> np.ndarray:
    """Exact widening of 16-bit patterns to float64."""
    if dtype == F16:
        return np.ascontiguousarray(b).view(np.float16).astype(np.float64)
    return bf16_bits_to_f64(b)


# ----------------------------------------------------------------------------
# Tensors
# ----------------------------------------------------------------------------

def gen_qkv(shape: Tuple[int, int, int, int], dtype: int, seed: int,
            value_scale: float = 1.0, k_outlier_frac: float = 0.0,
            heads_subset: Optional[List[Tuple[int, int]]] = None):
    """Standard-normal Q, K, V rounded to ``dtype``; returns three uint16 arrays.

    Every (batch, head) pair has its own Philox stream keyed by (seed, b, h), so a
    subset of heads can be regenerated without producing the whole tensor
    (``heads_subset`` = list of (b, h); other heads are left zero).
    A fraction ``k_outlier_frac`` of K rows per head (floor(frac * seq) rows,
    chosen without replacement) is multiplied by 8 before rounding.
    """
    B, H, N, d = shape
    q = np.zeros(shape, np.uint16)
    k = np.zeros(shape, np.uint16)
    v = np.zeros(shape, np.uint16)
    pairs = heads_subset if heads_subset is not None else [(b, h) for b in range(B) for h in range(H)]
    for (b, h) in pairs:
        rng = np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, (b << 20) | h]))
        x = rng.standard_normal((3, N, d)) * value_scale
        n_out = int(np.floor(k_outlier_frac * N))
        if n_out > 0:
            rows = rng.choice(N, size=n_out, replace=False)
            x[1, rows, :] *= 8.0
        q[b, h] = to_bits(x[0], dtype)
        k[b, h] = to_bits(x[1], dtype)
        v[b, h] = to_bits(x[2], dtype)
    return q, k, v


def gen_workload(cfg: int, heads_subset: Optional[List[Tuple[int, int]]] = None):
    w = WORKLOADS[cfg]
    return gen_qkv((w.batch, w.heads, w.seq, w.head_dim), w.dtype, DATA_SEED_BASE + cfg,
                   w.value_scale, w.k_outlier_frac, heads_subset)


# ----------------------------------------------------------------------------
# Fault candidates
# ----------------------------------------------------------------------------
# A fault is the integer 7-tuple (b, h, stage, kv_tile, row, col, bit):
#   S, EXP : (row, col) = (query, key) position, kv_tile = col // block_n
#   ROWSUM : row; kv_tile = iteration after whose update l is flipped; col = 0
#   OACC   : row; col = feature index; kv_tile = iteration after whose update
#            the accumulator element is flipped
# bit is the bit of the fp32 encoding that is inverted.

FAULT_FIELDS = ("b", "h", "stage", "kv_tile", "row", "col", "bit")


def n_kv_tiles(row: int, seq: int, block_n: int, causal: bool) -> int:
    """Number of key tiles that hold at least one unmasked key for ``row``."""
    last_key = row if causal else seq - 1
    return last_key // block_n + 1


def candidate_stream(seed: int, b: int, h: int, slot: int, seq: int, head_dim: int,
                     block_n: int, causal: bool, stages: Tuple[int, ...],
                     bit_lo: int, bit_hi: int) -> Iterator[Tuple[int, ...]]:
    """Endless deterministic stream of candidate faults for one (b, h, slot)."""
    rng = np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, (b << 40) | (h << 20) | slot]))
    while True:
        stage = int(stages[int(rng.integers(len(stages)))])
        row = int(rng.integers(seq))
        bit = int(rng.integers(bit_lo, bit_hi + 1))
        nt = n_kv_tiles(row, seq, block_n, causal)
        if stage in (ST_S, ST_EXP):
            col = int(rng.integers(row + 1 if causal else seq))
            kv_tile = col // block_n
        elif stage == ST_ROWSUM:
            col = 0
            kv_tile = int(rng.integers(nt))
        else:
            col = int(rng.integers(head_dim))
            kv_tile = int(rng.integers(nt))
        yield (b, h, stage, kv_tile, row, col, bit)


def conflicts(f: Tuple[int, ...], accepted: List[Tuple[int, ...]]) -> bool:
    """Single-event-upset rule: at most one fault per detection/correction cycle.

    A cycle is one row of one key-tile iteration for the S and EXP stages, one
    row for ROWSUM, and one (row, stride-8 feature class) for OACC.
    """
    b, h, st, kt, row, col, _ = f
    for g in accepted:
        if g[0] != b or g[1] != h or g[4] != row:
            continue
        gst = g[2]
        if st in (ST_S, ST_EXP) and gst in (ST_S, ST_EXP) and g[3] == kt:
            return True
        if st == ST_ROWSUM and gst == ST_ROWSUM:
            return True
        if st == ST_OACC and gst == ST_OACC and (g[5] % 8) == (col % 8):
            return True
    return False


def workload_fault_slots(cfg: int):
    """Yields (b, h, slot, stages) for every fault slot of a workload."""
    w = WORKLOADS[cfg]
    for b in range(w.batch):
        for h in range(w.heads):
            for k in range(w.faults_per_head):
                stages = (w.fault_stages[k],) if w.one_per_stage else w.fault_stages
                yield b, h, k, stages


def faults_to_array(faults: List[Tuple[int, ...]]) -> np.ndarray:
    a = np.asarray(faults, dtype=np.int32).reshape(-1, 7)
    return np.ascontiguousarray(a)


# ----------------------------------------------------------------------------
# Linear layer (feed-forward / projection GEMM protected by the same tensor checksums)
# ----------------------------------------------------------------------------
# A fault of the linear layer is the integer triple (row, col, bit): bit `bit` of the fp32
# accumulator of Y[row, col] is inverted after the last accumulation step.

LINEAR_SEED_BASE = 0xF7A7A000


def gen_linear(m: int, n: int, k: int, seed: int, x_scale: float = 1.0, dtype: int = F16):
    """Activations X [m, k] ~ N(0, x_scale^2) and weights W [n, k] ~ N(0, 1/k) (so that the
    outputs are of order x_scale), rounded to ``dtype``; returns two uint16 arrays.  Rows are drawn
    from per-row-block Philox streams so that a slice can be regenerated on its own."""
    x = np.zeros((m, k), np.uint16)
    w = np.zeros((n, k), np.uint16)
    for which, arr, rows, sc in ((0, x, m, x_scale), (1, w, n, 1.0 / np.sqrt(k))):
        for r0 in range(0, rows, 1024):
            rng = np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, (which << 40) | r0]))
            nr = min(1024, rows - r0)
            arr[r0:r0 + nr] = to_bits(rng.standard_normal((nr, k)) * sc, dtype)
    return x, w


def linear_fault_stream(seed: int, slot: int, m: int, n: int, bit_lo: int, bit_hi: int) -> Iterator[Tuple[int, int, int]]:
    """Endless deterministic stream of candidate faults (row, col, bit) for one slot."""
    rng = np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, (7 << 40) | slot]))
    while True:
        yield int(rng.integers(m)), int(rng.integers(n)), int(rng.integers(bit_lo, bit_hi + 1))
