"""Seeded synthetic inputs for the ABFT-checked low-precision EmbeddingBag (arXiv 2103.00130,
Section III-C and Section V; shapes of Table I).

Input generation only: row-wise 8-bit quantized tables, index sets, offsets and per-sample
weights.  None of the operator's or the check's arithmetic lives here (no row sums, no
pooling, no comparison); the CPU oracle and the HIP path both read what this module draws.

Table I of the paper: 4,000,000 rows, 32 / 64 / 128 / 256 columns, average pooling size 100,
batch size 10, regular and weighted sum.  `TABLE1` names those; the other entries are smaller
cases for tests and a large batch that is bound by memory bandwidth instead of latency.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

EB_SEED_BASE = 210300130 + 50_000


@dataclass(frozen=True)
class EbWorkload:
    name: str
    rows: int       # rows of the embedding table
    d: int          # embedding dimension (columns)
    n_bags: int     # batch size: index sets pooled by one call
    pooling: int    # average number of rows per index set
    weighted: bool  # per-sample weights (weighted sum)
    regime: str     # value distribution of the table, see draw_table


TABLE1 = {d: EbWorkload(f"table1_rows4000000_d{d}_pool100_batch10", 4_000_000, d, 10, 100, False, "uniform")
          for d in (32, 64, 128, 256)}
# the same tables pooled for a large batch: the gather is then bound by memory bandwidth
LARGE_BATCH = {d: EbWorkload(f"rows4000000_d{d}_pool100_batch16384", 4_000_000, d, 16384, 100, False, "uniform")
               for d in (32, 64, 128, 256)}


def rng_for(tag: int, rep: int = 0, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(EB_SEED_BASE + 1000 * tag + rep + 7919 * stream))


def pack_nibbles(codes: np.ndarray) -> np.ndarray:
    """4-bit codes [rows, d] (values 0..15) as bytes [rows, d/2]: the even column in the low half."""
    return (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)


def draw_table(rng: np.random.Generator, rows: int, d: int, regime: str, bits: int = 8):
    """Row-wise quantized table: codes T, float32 scale[rows], float32 bias[rows]; row i stands for
    the real vector scale[i] * code[i, :] + bias[i].  bits = 8: T is uint8 [rows, d]; bits = 4: codes
    0..15 packed two per byte, T is uint8 [rows, d/2] (see pack_nibbles) and scales are 17 times larger
    so that the values cover the same range.

    regime "uniform": codes uniform on [0, 255], scale uniform on [0.005, 0.02), bias uniform on
        [-0.5, 0): values of mostly one sign, as after a ReLU-like training range.
    regime "gauss": every row quantizes d draws of N(0, 1) with its own min/max range (scale =
        (max - min) / 255, bias = min): values centred on zero.
    regime "integer": scale 1, bias 0 (the operator is then exact integer arithmetic).
    """
    top = (1 << bits) - 1
    if regime == "uniform":
        T = rng.integers(0, top + 1, size=(rows, d), dtype=np.uint8)
        scale = (rng.uniform(0.005, 0.02, size=rows) * (255 // top)).astype(np.float32)
        bias = rng.uniform(-0.5, 0.0, size=rows).astype(np.float32)
    elif regime == "gauss":
        x = rng.standard_normal(size=(rows, d)).astype(np.float32)
        lo, hi = x.min(axis=1), x.max(axis=1)
        scale = ((hi - lo) / np.float32(top)).astype(np.float32)
        scale[scale == 0] = np.float32(1)
        bias = lo.astype(np.float32)
        T = np.clip(np.rint((x - bias[:, None]) / scale[:, None]), 0, top).astype(np.uint8)
    elif regime == "integer":
        T = rng.integers(0, top + 1, size=(rows, d), dtype=np.uint8)
        scale = np.ones(rows, dtype=np.float32)
        bias = np.zeros(rows, dtype=np.float32)
    else:
        raise ValueError(regime)
    return (T if bits == 8 else pack_nibbles(T)), scale, bias


def draw_bags(rng: np.random.Generator, rows: int, n_bags: int, pooling: int, lengths: str = "spread"):
    """Index sets in the offsets form: indices[int64], offsets[int64, n_bags + 1]; bag b pools
    indices[offsets[b] : offsets[b + 1]].  Rows are drawn uniformly with repetition.

    lengths "fixed": every bag has `pooling` rows; "spread": uniform on [pooling/2, 3*pooling/2]
    (mean `pooling`); "ragged": geometric-like mix that includes empty and single-row bags.
    """
    if lengths == "fixed":
        n = np.full(n_bags, pooling, dtype=np.int64)
    elif lengths == "spread":
        n = rng.integers(pooling // 2, pooling + pooling // 2 + 1, size=n_bags, dtype=np.int64)
    elif lengths == "ragged":
        n = np.minimum(rng.geometric(1.0 / max(pooling, 1), size=n_bags) - 1, 8 * pooling).astype(np.int64)
        n[rng.random(n_bags) < 0.1] = 0
        n[rng.random(n_bags) < 0.1] = 1
    else:
        raise ValueError(lengths)
    offsets = np.zeros(n_bags + 1, dtype=np.int64)
    np.cumsum(n, out=offsets[1:])
    indices = rng.integers(0, rows, size=int(offsets[-1]), dtype=np.int64)
    return indices, offsets


def draw_weights(rng: np.random.Generator, n: int) -> np.ndarray:
    """Per-sample weights of the weighted sum: uniform on [0.25, 1.75), float32."""
    return rng.uniform(0.25, 1.75, size=n).astype(np.float32)


@dataclass
class EbInputs:
    wl: EbWorkload
    T: np.ndarray
    scale: np.ndarray
    bias: np.ndarray
    indices: np.ndarray
    offsets: np.ndarray
    weights: np.ndarray | None


def make_inputs(wl: EbWorkload, tag: int = 0, rep: int = 0, lengths: str = "spread") -> EbInputs:
    rng = rng_for(tag, rep)
    T, scale, bias = draw_table(rng, wl.rows, wl.d, wl.regime)
    indices, offsets = draw_bags(rng, wl.rows, wl.n_bags, wl.pooling, lengths)
    weights = draw_weights(rng, indices.size) if wl.weighted else None
    return EbInputs(wl, T, scale, bias, indices, offsets, weights)


def draw_table_flips(rng: np.random.Generator, indices: np.ndarray, d: int, n: int, bits: str, code_bits: int = 8):
    """Fault list of Section VI-B-2: single bit flips in table elements that the batch reads.
    Returns arrays (row, col, bit); the row is one of `indices` (uniform over positions), the
    column uniform, the bit uniform over the upper ("high") or lower ("low") half of the element's
    code_bits bits (8-bit codes: 4..7 and 0..3)."""
    half = code_bits // 2
    lo = {"high": half, "low": 0}[bits]
    pos = rng.integers(0, indices.size, size=n)
    return indices[pos].astype(np.int64), rng.integers(0, d, size=n, dtype=np.int32), \
        rng.integers(lo, lo + half, size=n, dtype=np.int32)
