"""Seeded synthetic workloads: shapes, operand distributions and fault lists.

This module draws numbers and nothing else: no sums, products, checksums or
comparisons of the method live here, so both the HIP path and the CPU checker
can be fed from it without sharing arithmetic.

The paper evaluates on uniformly random 8-bit operands (Section IV-C states the
assumption: A uniform unsigned 8-bit, B uniform signed 8-bit) over DLRM
fully-connected shapes, and simulates faults by inverting one random bit of one
random element of an input or of the 32-bit intermediate (Section VI-B).  The
five workloads below follow that recipe on DLRM-shaped (m, n, k).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 210300130


@dataclass(frozen=True)
class Workload:
    index: int
    name: str
    M: int
    N: int
    K: int
    zA: int = 128                 # zero point of the uint8 activations
    zC: int = 128                 # zero point of the uint8 output
    relu_like: bool = False       # 40 % zeros, rest uniform[1,255]
    requant: str = "none"         # "none" | "tensor" | "channel"
    n_flips: dict = field(default_factory=dict)   # target -> number of injections


WORKLOADS = (
    Workload(0, "m64_n256_k512", 64, 256, 512, n_flips={"C": 1000}),
    Workload(1, "dlrm_bottom_m256_n512_k1024", 256, 512, 1024, requant="tensor"),
    Workload(2, "tall_skinny_m16_n4096_k2048", 16, 4096, 2048,
             n_flips={"A": 10000, "B": 10000, "C": 10000}),
    Workload(3, "dlrm_top_m1024_n1024_k4096", 1024, 1024, 4096, zA=0, relu_like=True,
             requant="channel"),
    Workload(4, "dense_m4096_n4096_k4096", 4096, 4096, 4096, n_flips={"C": 100000}),
)


def seed_for(cfg: int, rep: int = 0) -> int:
    return BASE_SEED + 1000 * cfg + rep


def rng_for(cfg: int, rep: int = 0, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed_for(cfg, rep) + stream))


def draw_a(rng: np.random.Generator, M: int, K: int, relu_like: bool = False) -> np.ndarray:
    """uint8 activations: uniform[0,255], or 40 % zeros with the rest uniform[1,255]."""
    if not relu_like:
        return rng.integers(0, 256, size=(M, K), dtype=np.uint8)
    vals = rng.integers(1, 256, size=(M, K), dtype=np.uint8)
    zero = rng.random(size=(M, K)) < 0.4
    vals[zero] = 0
    return vals


def draw_b(rng: np.random.Generator, K: int, N: int) -> np.ndarray:
    """int8 weights, symmetric quantization: uniform[-127,127], K x N row-major."""
    return rng.integers(-127, 128, size=(K, N), dtype=np.int8)


def draw_mult(rng: np.random.Generator, N: int, kind: str) -> np.ndarray | None:
    """Requantization multiplier(s) alpha_A*alpha_B/alpha_C, log-uniform[1e-4, 1e-2]."""
    if kind == "none":
        return None
    n = 1 if kind == "tensor" else N
    return np.exp(rng.uniform(np.log(1e-4), np.log(1e-2), size=n)).astype(np.float32)


@dataclass
class Operands:
    wl: Workload
    A: np.ndarray
    B: np.ndarray
    mult: np.ndarray | None


def make_operands(cfg: int, rep: int = 0) -> Operands:
    wl = WORKLOADS[cfg]
    rng = rng_for(cfg, rep)
    A = draw_a(rng, wl.M, wl.K, wl.relu_like)
    B = draw_b(rng, wl.K, wl.N)
    mult = draw_mult(rng, wl.N, wl.requant)
    return Operands(wl, A, B, mult)


def draw_flips(cfg: int, target: str, n: int | None = None, rep: int = 0):
    """Fault list for one target: arrays (idx0, idx1, bit).

    target "A": (row i, column k, bit 0..7); "B": (row k, column j, bit 0..7);
    "C": (row r, column c, bit 0..31).  Element and bit are uniform.
    """
    wl = WORKLOADS[cfg]
    if n is None:
        n = wl.n_flips[target]
    stream = 500 + {"A": 0, "B": 1, "C": 2}[target]
    rng = rng_for(cfg, rep, stream)
    d0, d1, nb = {"A": (wl.M, wl.K, 8), "B": (wl.K, wl.N, 8), "C": (wl.M, wl.N, 32)}[target]
    i0 = rng.integers(0, d0, size=n, dtype=np.int32)
    i1 = rng.integers(0, d1, size=n, dtype=np.int32)
    bit = rng.integers(0, nb, size=n, dtype=np.int32)
    return i0, i1, bit


def draw_value_faults(cfg: int, target: str, n: int, rep: int = 0):
    """Fault list for the value-replacement model: arrays (idx0, idx1, new_value).

    target "B": (row k, column j, new int8 value, uniform over all 256 codes);
    "C": (row r, column c, new int32 value, uniform over all 2^32 codes).
    """
    wl = WORKLOADS[cfg]
    rng = rng_for(cfg, rep, 510 + {"B": 1, "C": 2}[target])
    d0, d1 = {"B": (wl.K, wl.N), "C": (wl.M, wl.N)}[target]
    i0 = rng.integers(0, d0, size=n, dtype=np.int32)
    i1 = rng.integers(0, d1, size=n, dtype=np.int32)
    if target == "B":
        new = rng.integers(-128, 128, size=n, dtype=np.int32)
    else:
        new = rng.integers(-2**31, 2**31, size=n, dtype=np.int64).astype(np.int32)
    return i0, i1, new


def draw_multibit_masks(cfg: int, target: str, n: int, n_bits: int, rep: int = 0):
    """Fault list for multi-bit upsets: arrays (idx0, idx1, xor_mask) with exactly n_bits
    distinct bits set in the mask (8-bit masks for "B", 32-bit for "C")."""
    wl = WORKLOADS[cfg]
    rng = rng_for(cfg, rep, 520 + {"B": 1, "C": 2}[target])
    d0, d1, width = {"B": (wl.K, wl.N, 8), "C": (wl.M, wl.N, 32)}[target]
    i0 = rng.integers(0, d0, size=n, dtype=np.int32)
    i1 = rng.integers(0, d1, size=n, dtype=np.int32)
    masks = np.zeros(n, dtype=np.uint32)
    for t in range(n):
        for b in rng.choice(width, size=n_bits, replace=False):
            masks[t] |= np.uint32(1) << np.uint32(b)
    return i0, i1, masks
