"""numpy front end of the EmbeddingBag CPU oracle (oracle/eb_oracle.c).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this module; the tests,
the smoke check and the benchmark's cpu_baseline leg do.  The functions marshal numpy
arrays into the plain-C loops that state the operator of arXiv 2103.00130 Section III-C
and its check (Section V, Eq. 4, Algorithm 2); `checked_eb` strings them together in the
order of Algorithm 2.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "eb_oracle.c")
_LIB = os.path.join(_HERE, "libeb_oracle.so")

_u8p = ctypes.POINTER(ctypes.c_uint8)
_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i64 = ctypes.c_int64
_int = ctypes.c_int
_dbl = ctypes.c_double

REL_BOUND = 1e-5  # Section V, "Round off error bound": the relative bound the paper chooses


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, no contraction of a*b+c into fused operations
    other than the fmaf calls the source writes out)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"],
                       check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.eb_oracle_rowsums.argtypes = [_u8p, _i64, _int, _int, _i32p]
        fwd = [_u8p, _i64, _int, _int, _f32p, _f32p, _i64p, _i64p, _i64, _f32p]
        L.eb_oracle_forward_f64.argtypes = fwd + [_f64p]
        L.eb_oracle_forward_f32.argtypes = fwd + [_f32p]
        L.eb_oracle_check.argtypes = [_f32p, _i64, _i64, _int, _f32p, _f32p, _i32p, _i64p, _i64p, _i64, _f32p, _dbl,
                                      _i32p, _f64p, _f64p]
        L.eb_oracle_campaign_table_flips.argtypes = [_u8p, _i64, _int, _int, _f32p, _f32p, _i32p, _i64p, _i64p, _i64, _f32p,
                                                     _dbl, _i64p, _i32p, _i32p, _i64, _i32p]
        for f in (L.eb_oracle_rowsums, L.eb_oracle_forward_f64, L.eb_oracle_forward_f32, L.eb_oracle_check,
                  L.eb_oracle_campaign_table_flips):
            f.restype = None
        _lib = L
    return _lib


def _p(a, t):
    return a.ctypes.data_as(t) if a is not None else None


def _table(T, bits=8):
    """The code table as bytes, and its number of columns d (4-bit codes lie two per byte)."""
    T = np.ascontiguousarray(T, dtype=np.uint8)
    assert T.ndim == 2 and bits in (4, 8)
    return T, T.shape[1] * 8 // bits


def _bags(indices, offsets):
    indices = np.ascontiguousarray(indices, dtype=np.int64)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    assert offsets.ndim == 1 and offsets.size >= 1 and offsets[0] >= 0 and offsets[-1] <= indices.size
    assert np.all(np.diff(offsets) >= 0)
    return indices, offsets


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def table_rowsums(T, bits: int = 8) -> np.ndarray:
    """C_T of Section V: 32-bit integer row sums of the code table."""
    T, d = _table(T, bits)
    out = np.empty(T.shape[0], dtype=np.int32)
    lib().eb_oracle_rowsums(_p(T, _u8p), T.shape[0], d, bits, _p(out, _i32p))
    return out


def forward(T, scale, bias, indices, offsets, weights=None, precision: str = "f32", bits: int = 8) -> np.ndarray:
    """The EmbeddingBag of Section III-C for a batch, in double ("f64", the definition) or in
    float in index order ("f32", the paper's precision)."""
    T, d = _table(T, bits)
    scale, bias, weights = _f32(scale), _f32(bias), _f32(weights)
    indices, offsets = _bags(indices, offsets)
    n_bags = offsets.size - 1
    if precision == "f64":
        R = np.empty((n_bags, d), dtype=np.float64)
        lib().eb_oracle_forward_f64(_p(T, _u8p), T.shape[0], d, bits, _p(scale, _f32p), _p(bias, _f32p),
                                    _p(indices, _i64p), _p(offsets, _i64p), n_bags, _p(weights, _f32p), _p(R, _f64p))
    elif precision == "f32":
        R = np.empty((n_bags, d), dtype=np.float32)
        lib().eb_oracle_forward_f32(_p(T, _u8p), T.shape[0], d, bits, _p(scale, _f32p), _p(bias, _f32p),
                                    _p(indices, _i64p), _p(offsets, _i64p), n_bags, _p(weights, _f32p), _p(R, _f32p))
    else:
        raise ValueError(precision)
    return R


@dataclass
class EbCheck:
    flags: np.ndarray   # int32 per bag: bit 0 Algorithm 2's err, bit 1 an index outside the table
    rsum: np.ndarray    # float64 per bag
    csum: np.ndarray    # float64 per bag
    robust: np.ndarray  # bool per bag: the comparison cannot depend on the order of the double sums


def check(R, rows, scale, bias, C_T, indices, offsets, weights=None, bound: float = REL_BOUND) -> EbCheck:
    """Algorithm 2 after the lookup: RSum, CSum (Eq. 4) and the comparison, for every bag.

    `robust[b]` is False where |RSum - CSum| lies so close to the bound that summing the same
    doubles in another order could flip the comparison (margin: the worst-case reordering
    error of a double sum over the terms involved); RSum itself is also formed with an
    exactly rounded sum (math.fsum) to measure that."""
    R = np.ascontiguousarray(R, dtype=np.float32)
    scale, bias, weights = _f32(scale), _f32(bias), _f32(weights)
    C_T = np.ascontiguousarray(C_T, dtype=np.int32)
    indices, offsets = _bags(indices, offsets)
    n_bags, d = R.shape
    flags = np.empty(n_bags, dtype=np.int32)
    rsum = np.empty(n_bags, dtype=np.float64)
    csum = np.empty(n_bags, dtype=np.float64)
    lib().eb_oracle_check(_p(R, _f32p), d, int(rows), d, _p(scale, _f32p), _p(bias, _f32p), _p(C_T, _i32p),
                          _p(indices, _i64p), _p(offsets, _i64p), n_bags, _p(weights, _f32p), float(bound),
                          _p(flags, _i32p), _p(rsum, _f64p), _p(csum, _f64p))
    robust = np.ones(n_bags, dtype=bool)
    eps = 2.0 ** -52
    for b in range(n_bags):
        row = R[b].astype(np.float64)
        if not np.all(np.isfinite(row)) or not math.isfinite(csum[b]):
            continue
        exact = math.fsum(row)
        slack = 2.0 * d * eps * float(np.abs(row).sum()) + abs(exact - rsum[b])
        gap = abs(abs(exact - csum[b]) - bound * max(abs(exact), abs(csum[b])))
        robust[b] = slack == 0.0 or gap > slack + bound * slack  # (all-zero rows sum to zero in any order)
    return EbCheck(flags, rsum, csum, robust)


@dataclass
class CheckedEb:
    R: np.ndarray
    C_T: np.ndarray
    flags: np.ndarray
    rsum: np.ndarray
    csum: np.ndarray
    robust: np.ndarray


def checked_eb(T, scale, bias, indices, offsets, weights=None, bound: float = REL_BOUND, C_T=None,
               bits: int = 8) -> CheckedEb:
    """Algorithm 2 end to end: lookup in float, RSum, CSum, comparison.  C_T may be given
    (row sums taken before a fault was planted in T); otherwise it is computed from T."""
    T, _ = _table(T, bits)
    if C_T is None:
        C_T = table_rowsums(T, bits)
    R = forward(T, scale, bias, indices, offsets, weights, "f32", bits)
    c = check(R, T.shape[0], scale, bias, C_T, indices, offsets, weights, bound)
    return CheckedEb(R, C_T, c.flags, c.rsum, c.csum, c.robust)


def campaign_table_flips(T, scale, bias, C_T, indices, offsets, weights, f_row, f_col, f_bit,
                         bound: float = REL_BOUND, bits: int = 8) -> np.ndarray:
    """Section VI-B-2: per planted single-bit flip in the table (after C_T), the flags of the
    whole batch.  Returns int32 [n_flips, n_bags]."""
    T, d = _table(T, bits)
    T = T.copy()
    scale, bias, weights = _f32(scale), _f32(bias), _f32(weights)
    C_T = np.ascontiguousarray(C_T, dtype=np.int32)
    indices, offsets = _bags(indices, offsets)
    f_row = np.ascontiguousarray(f_row, dtype=np.int64)
    f_col = np.ascontiguousarray(f_col, dtype=np.int32)
    f_bit = np.ascontiguousarray(f_bit, dtype=np.int32)
    n, n_bags = f_row.size, offsets.size - 1
    out = np.empty((n, n_bags), dtype=np.int32)
    lib().eb_oracle_campaign_table_flips(_p(T, _u8p), T.shape[0], d, bits, _p(scale, _f32p), _p(bias, _f32p),
                                         _p(C_T, _i32p), _p(indices, _i64p), _p(offsets, _i64p), n_bags,
                                         _p(weights, _f32p), float(bound), _p(f_row, _i64p), _p(f_col, _i32p),
                                         _p(f_bit, _i32p), n, _p(out, _i32p))
    return out


def roundoff_tolerance(T, scale, bias, indices, offsets, weights=None, bits: int = 8) -> np.ndarray:
    """Per bag, a bound on |R_f32[j] - R_f64[j]| for any column j and any order of summation:
    (m + 3) * 2^-24 * sum_i (|a_i| * (2^bits - 1) + |b_i|), m the bag's length (standard forward error
    bound of a length-m float sum, plus the roundings of w*alpha, w*beta and the final add)."""
    scale, bias, weights = _f32(scale), _f32(bias), _f32(weights)
    indices, offsets = _bags(indices, offsets)
    n_bags = offsets.size - 1
    tol = np.zeros(n_bags, dtype=np.float64)
    for b in range(n_bags):
        idx = indices[offsets[b]:offsets[b + 1]]
        ok = (idx >= 0) & (idx < len(scale))
        idx = idx[ok]
        w = np.ones(idx.size) if weights is None else weights[offsets[b]:offsets[b + 1]][ok].astype(np.float64)
        mag = float(np.sum(np.abs(w * scale[idx].astype(np.float64)) * float(2 ** bits - 1) + np.abs(w * bias[idx].astype(np.float64))))
        tol[b] = (idx.size + 3) * 2.0 ** -24 * mag
    return tol
