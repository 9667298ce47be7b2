"""numpy front end of the CPU oracle (oracle/abft_oracle.c).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this module;
the tests, the smoke check and the benchmark's cpu_baseline leg do.  Every
function here only marshals numpy arrays into the plain-C routines, which state
the method of arXiv 2103.00130 (Section IV, Algorithm 1; Section III, Eq. 1)
as loops.  `checked_gemm` strings them together in the order of Algorithm 1.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "abft_oracle.c")
_LIB = os.path.join(_HERE, "libabft_oracle.so")

_i8p = ctypes.POINTER(ctypes.c_int8)
_u8p = ctypes.POINTER(ctypes.c_uint8)
_i32p = ctypes.POINTER(ctypes.c_int32)
_u32p = ctypes.POINTER(ctypes.c_uint32)
_f32p = ctypes.POINTER(ctypes.c_float)
_i64 = ctypes.c_int64
_int = ctypes.c_int


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP over rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"],
            check=True,
        )
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.oracle_num_threads.restype = _int
        L.oracle_b_checksum.argtypes = [_i8p, _i64, _int, _int, _i32p]
        L.oracle_b_colsum.argtypes = [_i8p, _i64, _int, _int, _i32p]
        L.oracle_gemm_u8s8s32.argtypes = [_u8p, _i64, _i8p, _i64, _int, _int, _int, _i32p, _i64]
        L.oracle_row_checksum.argtypes = [_u8p, _i64, _i32p, _int, _int, _i32p]
        L.oracle_row_sums.argtypes = [_i32p, _i64, _int, _int, _i32p]
        L.oracle_compare.argtypes = [_i32p, _i32p, _int, _i32p]
        L.oracle_compare.restype = _int
        rq = [_i32p, _i64, _int, _int, _i32p, ctypes.c_int32, ctypes.c_int32, _f32p, _int, _i32p, _u8p, _i64]
        L.oracle_requantize_f64.argtypes = rq
        L.oracle_requantize_f32.argtypes = rq
        L.oracle_b_checksum_mod127.argtypes = [_i8p, _i64, _int, _int, _i8p]
        L.oracle_row_checksum_mod127.argtypes = [_u8p, _i64, _i8p, _int, _int, _i32p]
        L.oracle_compare_mod127.argtypes = [_i32p, _i64, _int, _int, _i32p, _i32p]
        L.oracle_compare_mod127.restype = _int
        L.oracle_campaign_c_flips.argtypes = [_i32p, _i64, _int, _i32p, _int, _i32p, _i32p, _i32p, _i32p, _i32p]
        L.oracle_campaign_b_flips.argtypes = [_u8p, _i64, _i8p, _i64, _i32p, _i64, _int, _int, _int, _i32p,
                                              _int, _i32p, _i32p, _i32p, _i32p, _i32p]
        L.oracle_campaign_b_flips_mod127.argtypes = [_u8p, _i64, _i8p, _i64, _i32p, _i64, _int, _int, _int, _i32p,
                                                     _int, _i32p, _i32p, _i32p, _i32p, _i32p]
        L.oracle_campaign_c_masks.argtypes = [_i32p, _i64, _int, _i32p, _int, _i32p, _i32p, _u32p, _i32p, _i32p]
        L.oracle_campaign_b_values.argtypes = [_u8p, _i64, _i8p, _i64, _i32p, _i64, _int, _int, _int, _i32p,
                                               _int, _i32p, _i32p, _i32p, _i32p, _i32p]
        L.oracle_campaign_a_flips.argtypes = [_u8p, _i64, _i8p, _i64, _i32p, _int, _int, _int,
                                              _i32p, _i32p, _i32p, _i32p, _i32p]
        L.oracle_a_colsum.argtypes = [_u8p, _i64, _int, _int, _i32p]
        L.oracle_col_checksum.argtypes = [_i32p, _i8p, _i64, _int, _int, _i32p]
        L.oracle_col_sums.argtypes = [_i32p, _i64, _int, _int, _i32p]
        L.oracle_locate_correct.argtypes = [_i32p, _i64, _int, _int, _i32p, _i32p, _i32p, _i32p, _i32p]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _c(a: np.ndarray, dtype) -> np.ndarray:
    a = np.asarray(a)
    if a.dtype != np.dtype(dtype):
        raise TypeError(f"expected {np.dtype(dtype)}, got {a.dtype}")
    if a.ndim == 2 and a.strides[1] != a.itemsize:
        a = np.ascontiguousarray(a)
    elif a.ndim == 1 and a.size and a.strides[0] != a.itemsize:
        a = np.ascontiguousarray(a)
    return a


def _ld(a: np.ndarray) -> int:
    return a.strides[0] // a.itemsize if a.shape[0] > 1 else max(a.shape[1], 1)


def _p(a: np.ndarray, t):
    return a.ctypes.data_as(t)


def b_checksum(B: np.ndarray) -> np.ndarray:
    """S_B = B e (Section IV), exact int32."""
    B = _c(B, np.int8)
    K, N = B.shape
    out = np.empty(K, np.int32)
    lib().oracle_b_checksum(_p(B, _i8p), _ld(B), K, N, _p(out, _i32p))
    return out


def b_colsum(B: np.ndarray) -> np.ndarray:
    """e^T B (Eq. 1), exact int32."""
    B = _c(B, np.int8)
    K, N = B.shape
    out = np.empty(N, np.int32)
    lib().oracle_b_colsum(_p(B, _i8p), _ld(B), K, N, _p(out, _i32p))
    return out


def gemm_u8s8s32(A: np.ndarray, B: np.ndarray) -> np.ndarray:
    """C_temp = A B with wrap-around int32 accumulation (Section III-B)."""
    A = _c(A, np.uint8)
    B = _c(B, np.int8)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    C = np.empty((M, N), np.int32)
    lib().oracle_gemm_u8s8s32(_p(A, _u8p), _ld(A), _p(B, _i8p), _ld(B), M, N, K, _p(C, _i32p), max(N, 1))
    return C


def row_checksum(A: np.ndarray, S_B: np.ndarray) -> np.ndarray:
    """chk = A S_B: the extra column of C_temp in Algorithm 1."""
    A = _c(A, np.uint8)
    S_B = _c(S_B, np.int32)
    M, K = A.shape
    assert S_B.shape == (K,)
    out = np.empty(M, np.int32)
    lib().oracle_row_checksum(_p(A, _u8p), _ld(A), _p(S_B, _i32p), M, K, _p(out, _i32p))
    return out


def row_sums(C: np.ndarray) -> np.ndarray:
    """tSum of Algorithm 1 for every row."""
    C = _c(C, np.int32)
    M, N = C.shape
    out = np.empty(M, np.int32)
    lib().oracle_row_sums(_p(C, _i32p), _ld(C), M, N, _p(out, _i32p))
    return out


def compare(rsum: np.ndarray, chk: np.ndarray):
    """Eq. 2b as an equality mod 2^32 -> (flags[M], errCount)."""
    rsum = _c(rsum, np.int32)
    chk = _c(chk, np.int32)
    flags = np.empty(rsum.shape[0], np.int32)
    n = lib().oracle_compare(_p(rsum, _i32p), _p(chk, _i32p), rsum.shape[0], _p(flags, _i32p))
    return flags, int(n)


def requantize(C, colsum, zA, zC, mult, bias=None, precision="f64") -> np.ndarray:
    """uint8 output of the requantization step; precision 'f64' or 'f32'."""
    C = _c(C, np.int32)
    colsum = _c(colsum, np.int32)
    mult = np.atleast_1d(np.asarray(mult, np.float32))
    M, N = C.shape
    per_channel = 0 if mult.size == 1 else 1
    if per_channel:
        assert mult.shape == (N,)
    bp = None
    if bias is not None:
        bias = _c(bias, np.int32)
        bp = _p(bias, _i32p)
    out = np.empty((M, N), np.uint8)
    fn = {"f64": lib().oracle_requantize_f64, "f32": lib().oracle_requantize_f32}[precision]
    fn(_p(C, _i32p), _ld(C), M, N, _p(colsum, _i32p), int(zA), int(zC), _p(mult, _f32p), per_channel, bp,
       _p(out, _u8p), max(N, 1))
    return out


@dataclass
class Checked:
    C: np.ndarray          # int32 [M,N], as returned (with any C fault in it)
    S_B: np.ndarray        # int32 [K]
    colsum: np.ndarray     # int32 [N]
    chk: np.ndarray        # int32 [M]
    rsum: np.ndarray       # int32 [M]
    flags: np.ndarray      # int32 [M]
    err_count: int


def checked_gemm(A, B, flips_a=(), flips_b=(), flips_c=()) -> Checked:
    """Algorithm 1 end to end with optional simulated faults (Section VI-B).

    Order of events: the checksum S_B and the column sums are taken from the
    clean B (the encode step, done once per weight); then faults in B
    ((k, j, bit), raw byte XOR, checksum left stale) and in A ((i, k, bit)) are
    applied; then the product, the checksum column A S_B, faults in the 32-bit
    intermediate ((r, c, xor_mask)), the row sums and the comparison.
    """
    A = np.array(_c(A, np.uint8), copy=True)
    B = np.array(_c(B, np.int8), copy=True)
    S_B = b_checksum(B)
    colsum = b_colsum(B)
    for (k, j, bit) in flips_b:
        B.view(np.uint8)[k, j] ^= np.uint8(1 << bit)
    for (i, k, bit) in flips_a:
        A[i, k] ^= np.uint8(1 << bit)
    C = gemm_u8s8s32(A, B)
    chk = row_checksum(A, S_B)
    for (r, c, mask) in flips_c:
        C.view(np.uint32)[r, c] ^= np.uint32(mask)
    rsum = row_sums(C)
    flags, n = compare(rsum, chk)
    return Checked(C, S_B, colsum, chk, rsum, flags, n)


# ---- Algorithm 1 as printed (modulus 127) ------------------------------------------

def b_checksum_mod127(B: np.ndarray) -> np.ndarray:
    B = _c(B, np.int8)
    K, N = B.shape
    out = np.empty(K, np.int8)
    lib().oracle_b_checksum_mod127(_p(B, _i8p), _ld(B), K, N, _p(out, _i8p))
    return out


def checked_gemm_mod127(A, B, flips_b=(), flips_c=(), flips_rowsum=()):
    """Algorithm 1 with its printed modulus -> (C, flags, errCount).  flips_rowsum: (k, bit 0..7) inverts
    one bit of the stored 8-bit entry rowSum[k] after it was computed (the paper assumes that column
    error-free, Section IV-C; this is the fault it excludes)."""
    A = _c(A, np.uint8)
    B = np.array(_c(B, np.int8), copy=True)
    M, K = A.shape
    rs = b_checksum_mod127(B)
    for (k, bit) in flips_rowsum:
        rs.view(np.uint8)[k] ^= np.uint8(1 << bit)
    for (k, j, bit) in flips_b:
        B.view(np.uint8)[k, j] ^= np.uint8(1 << bit)
    C = gemm_u8s8s32(A, B)
    chk = np.empty(M, np.int32)
    lib().oracle_row_checksum_mod127(_p(A, _u8p), _ld(A), _p(rs, _i8p), M, K, _p(chk, _i32p))
    for (r, c, mask) in flips_c:
        C.view(np.uint32)[r, c] ^= np.uint32(mask)
    flags = np.empty(M, np.int32)
    n = lib().oracle_compare_mod127(_p(C, _i32p), _ld(C), M, C.shape[1], _p(chk, _i32p), _p(flags, _i32p))
    return C, flags, int(n)


# ---- campaigns ------------------------------------------------------------------------

def _i32(a):
    return np.ascontiguousarray(np.asarray(a, np.int32))


def campaign_c_flips(C_clean, chk, rows, cols, bits):
    """Per injection: (flag of the hit row, value of the flipped element)."""
    C_clean = _c(C_clean, np.int32)
    chk = _c(chk, np.int32)
    rows, cols, bits = _i32(rows), _i32(cols), _i32(bits)
    n = rows.size
    flag = np.empty(n, np.int32)
    val = np.empty(n, np.int32)
    lib().oracle_campaign_c_flips(_p(C_clean, _i32p), _ld(C_clean), C_clean.shape[1], _p(chk, _i32p), n,
                                  _p(rows, _i32p), _p(cols, _i32p), _p(bits, _i32p), _p(flag, _i32p),
                                  _p(val, _i32p))
    return flag, val


def campaign_b_flips(A, B, C_clean, chk, ks, js, bits):
    """Per injection: (flags[M], recomputed column j of C [M])."""
    A = _c(A, np.uint8)
    B = _c(B, np.int8)
    C_clean = _c(C_clean, np.int32)
    chk = _c(chk, np.int32)
    ks, js, bits = _i32(ks), _i32(js), _i32(bits)
    M, K = A.shape
    N = B.shape[1]
    n = ks.size
    flags = np.empty((n, M), np.int32)
    col = np.empty((n, M), np.int32)
    lib().oracle_campaign_b_flips(_p(A, _u8p), _ld(A), _p(B, _i8p), _ld(B), _p(C_clean, _i32p), _ld(C_clean),
                                  M, N, K, _p(chk, _i32p), n, _p(ks, _i32p), _p(js, _i32p), _p(bits, _i32p),
                                  _p(flags, _i32p), _p(col, _i32p))
    return flags, col


def row_checksum_mod127(A, B) -> np.ndarray:
    """C_temp[i][n] of Algorithm 1 as printed: A times the 8-bit column rowSum = (B e) mod 127."""
    A = _c(A, np.uint8)
    rs = b_checksum_mod127(B)
    M, K = A.shape
    chk = np.empty(M, np.int32)
    lib().oracle_row_checksum_mod127(_p(A, _u8p), _ld(A), _p(rs, _i8p), M, K, _p(chk, _i32p))
    return chk


def campaign_b_flips_mod127(A, B, C_clean, chk127, ks, js, bits):
    """campaign_b_flips under the printed modulus: (flags[M], recomputed column j of C [M])."""
    A = _c(A, np.uint8)
    B = _c(B, np.int8)
    C_clean = _c(C_clean, np.int32)
    chk127 = _c(chk127, np.int32)
    ks, js, bits = _i32(ks), _i32(js), _i32(bits)
    M, K = A.shape
    N = B.shape[1]
    n = ks.size
    flags = np.empty((n, M), np.int32)
    col = np.empty((n, M), np.int32)
    lib().oracle_campaign_b_flips_mod127(_p(A, _u8p), _ld(A), _p(B, _i8p), _ld(B), _p(C_clean, _i32p), _ld(C_clean),
                                         M, N, K, _p(chk127, _i32p), n, _p(ks, _i32p), _p(js, _i32p), _p(bits, _i32p),
                                         _p(flags, _i32p), _p(col, _i32p))
    return flags, col


def campaign_c_masks(C_clean, chk, rows, cols, masks):
    """Per injection of an arbitrary XOR mask (multi-bit upset, or old ^ new for a value
    replacement): (flag of the hit row, value of the changed element)."""
    C_clean = _c(C_clean, np.int32)
    chk = _c(chk, np.int32)
    rows, cols = _i32(rows), _i32(cols)
    masks = np.ascontiguousarray(np.asarray(masks, np.uint32))
    n = rows.size
    flag = np.empty(n, np.int32)
    val = np.empty(n, np.int32)
    lib().oracle_campaign_c_masks(_p(C_clean, _i32p), _ld(C_clean), C_clean.shape[1], _p(chk, _i32p), n,
                                  _p(rows, _i32p), _p(cols, _i32p), _p(masks, _u32p), _p(flag, _i32p),
                                  _p(val, _i32p))
    return flag, val


def campaign_b_values(A, B, C_clean, chk, ks, js, new_vals):
    """Per replacement of B[k][j] by new_vals[t] after the checksum was taken:
    (flags[M], recomputed column j of C [M])."""
    A = _c(A, np.uint8)
    B = _c(B, np.int8)
    C_clean = _c(C_clean, np.int32)
    chk = _c(chk, np.int32)
    ks, js, new_vals = _i32(ks), _i32(js), _i32(new_vals)
    M, K = A.shape
    N = B.shape[1]
    n = ks.size
    flags = np.empty((n, M), np.int32)
    col = np.empty((n, M), np.int32)
    lib().oracle_campaign_b_values(_p(A, _u8p), _ld(A), _p(B, _i8p), _ld(B), _p(C_clean, _i32p), _ld(C_clean),
                                   M, N, K, _p(chk, _i32p), n, _p(ks, _i32p), _p(js, _i32p), _p(new_vals, _i32p),
                                   _p(flags, _i32p), _p(col, _i32p))
    return flags, col


def campaign_a_flips(A, B, S_B, is_, ks, bits, want_rows=False):
    """Per injection: flag of the hit row (and, if asked, the recomputed row of C)."""
    A = _c(A, np.uint8)
    B = _c(B, np.int8)
    S_B = _c(S_B, np.int32)
    is_, ks, bits = _i32(is_), _i32(ks), _i32(bits)
    K, N = B.shape
    n = is_.size
    flag = np.empty(n, np.int32)
    rows = np.empty((n, N), np.int32) if want_rows else None
    lib().oracle_campaign_a_flips(_p(A, _u8p), _ld(A), _p(B, _i8p), _ld(B), _p(S_B, _i32p), N, K, n,
                                  _p(is_, _i32p), _p(ks, _i32p), _p(bits, _i32p), _p(flag, _i32p),
                                  _p(rows, _i32p) if want_rows else None)
    return (flag, rows) if want_rows else flag


# ---- locating and correcting one faulty element (Section IV, Eq. 2a) --------------------

def a_colsum(A: np.ndarray) -> np.ndarray:
    """S_A[k] = sum_i A[i][k], the row appended to A (Section IV)."""
    A = _c(A, np.uint8)
    M, K = A.shape
    out = np.empty(K, np.int32)
    lib().oracle_a_colsum(_p(A, _u8p), _ld(A), M, K, _p(out, _i32p))
    return out


def col_checksum(S_A: np.ndarray, B: np.ndarray) -> np.ndarray:
    """The checksum row C'[m][:] = S_A B, computed on its own."""
    S_A = _c(S_A, np.int32)
    B = _c(B, np.int8)
    K, N = B.shape
    out = np.empty(N, np.int32)
    lib().oracle_col_checksum(_p(S_A, _i32p), _p(B, _i8p), _ld(B), K, N, _p(out, _i32p))
    return out


def col_sums(C: np.ndarray) -> np.ndarray:
    C = _c(C, np.int32)
    M, N = C.shape
    out = np.empty(N, np.int32)
    lib().oracle_col_sums(_p(C, _i32p), _ld(C), M, N, _p(out, _i32p))
    return out


@dataclass
class Located:
    C: np.ndarray           # C after the call (repaired in place when status == 1)
    status: int             # 0 nothing violated, 1 located and corrected, 2 not one element
    row: int
    col: int
    old_value: int
    new_value: int
    rows_violated: int
    cols_violated: int
    col_flags: np.ndarray


def locate_correct(A, B, C, row_flags, S_B=None) -> Located:
    """Eq. 2a on the stored C with the checksum row recomputed from A and the B in memory, then the
    decision and repair of Section IV.  A, B: the operands as they stand in memory; C, row_flags: what
    the checked product returned; S_B: the checksum column stored with the weight (when B was hit after
    it was encoded, pass the column of the clean B; default: computed from B)."""
    A = _c(A, np.uint8)
    B = _c(B, np.int8)
    C = np.array(_c(C, np.int32), copy=True)
    row_flags = _c(np.asarray(row_flags, np.int32), np.int32)
    M, N = C.shape
    col_chk = col_checksum(a_colsum(A), B)
    row_chk = row_checksum(A, b_checksum(B) if S_B is None else _c(S_B, np.int32))
    col_flags = np.empty(N, np.int32)
    out = np.zeros(8, np.int32)
    lib().oracle_locate_correct(_p(C, _i32p), _ld(C), M, N, _p(row_flags, _i32p), _p(row_chk, _i32p),
                                _p(col_chk, _i32p), _p(col_flags, _i32p), _p(out, _i32p))
    return Located(C, int(out[0]), int(out[1]), int(out[2]), int(out[3]), int(out[4]), int(out[5]), int(out[6]), col_flags)
