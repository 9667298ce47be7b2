"""Pins for the CPU oracle: it is checked against things that are not itself.

 - brute force in Python arbitrary-precision integers on tiny, extreme inputs;
 - an independent library routine (BLAS float64 matmul, exact below 2^53);
 - closed forms for constant operands, including forced 32-bit wrap-around;
 - the invariants the paper states (Table II: clean runs never flag, every flip
   in the 32-bit intermediate is caught; Section IV-C-3: A is not covered);
 - the closed form for a flip in B (Section IV-C-1 with the modulus replaced);
 - exact rational arithmetic for the requantization step;
 - the paper's printed figures for its own modulus 127 (tests/golden).
"""
import itertools
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2103_00130_amd import workloads as wlmod

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
MASK = (1 << 32) - 1


def to_i32(v: int) -> int:
    v &= MASK
    return v - (1 << 32) if v >= (1 << 31) else v


def brute(A, B):
    """C, S_B, colsum, chk, rsum as Python ints reduced mod 2^32."""
    M, K = len(A), len(A[0])
    N = len(B[0])
    C = [[to_i32(sum(int(A[i][k]) * int(B[k][j]) for k in range(K))) for j in range(N)] for i in range(M)]
    S = [sum(int(B[k][j]) for j in range(N)) for k in range(K)]
    cs = [sum(int(B[k][j]) for k in range(K)) for j in range(N)]
    chk = [to_i32(sum(int(A[i][k]) * S[k] for k in range(K))) for i in range(M)]
    rsum = [to_i32(sum(C[i][j] for j in range(N))) for i in range(M)]
    return C, S, cs, chk, rsum


A_EXT = [0, 1, 127, 128, 255]
B_EXT = [-128, -127, -1, 0, 127]


@pytest.mark.parametrize("M,N,K", list(itertools.product([1, 2, 3, 5], repeat=3)))
def test_bruteforce_tiny_extremes(oracle, M, N, K):
    rng = np.random.default_rng(1000 * M + 100 * N + K)
    for _ in range(4):
        A = rng.choice(A_EXT, size=(M, K)).astype(np.uint8)
        B = rng.choice(B_EXT, size=(K, N)).astype(np.int8)
        C, S, cs, chk, rsum = brute(A.tolist(), B.tolist())
        r = oracle.checked_gemm(A, B)
        assert r.C.tolist() == C
        assert r.S_B.tolist() == S
        assert r.colsum.tolist() == cs
        assert r.chk.tolist() == chk
        assert r.rsum.tolist() == rsum
        assert r.flags.tolist() == [0] * M and r.err_count == 0


def test_bruteforce_nonsymmetric_operands(oracle):
    # a transposed operand or a swapped index would survive symmetric inputs
    A = np.array([[1, 2, 3], [4, 5, 6]], np.uint8)
    B = np.array([[1, -2, 3, -4], [5, 6, -7, 8], [-9, 10, 11, 12]], np.int8)
    r = oracle.checked_gemm(A, B)
    assert r.C.tolist() == [[-16, 40, 22, 48], [-25, 82, 43, 96]]
    assert r.S_B.tolist() == [-2, 12, 24]
    assert r.colsum.tolist() == [-3, 14, 7, 16]
    assert r.chk.tolist() == [94, 196] and r.rsum.tolist() == [94, 196]


@pytest.mark.parametrize("cfg", [0, 1, 2, 3])
def test_against_blas_float64(oracle, cfg):
    ops = wlmod.make_operands(cfg)
    A, B = ops.A, ops.B
    # every partial sum is below 255*128*4096 < 2^53: float64 BLAS is exact
    ref = (A.astype(np.float64) @ B.astype(np.float64)).astype(np.int64)
    C = oracle.gemm_u8s8s32(A, B)
    assert np.array_equal(C.astype(np.int64), ref)
    S = oracle.b_checksum(B)
    assert np.array_equal(S.astype(np.int64), B.astype(np.int64).sum(axis=1))
    assert np.array_equal(oracle.b_colsum(B).astype(np.int64), B.astype(np.int64).sum(axis=0))
    chk = oracle.row_checksum(A, S)
    chk_ref = (A.astype(np.float64) @ S.astype(np.float64)).astype(np.int64)  # < 2^53
    assert np.array_equal(chk.astype(np.uint32), (chk_ref & MASK).astype(np.uint32))
    rs = oracle.row_sums(C)
    assert np.array_equal(rs.astype(np.uint32), (ref.sum(axis=1) & MASK).astype(np.uint32))


def test_against_blas_float64_cfg4_sampled_rows(oracle):
    ops = wlmod.make_operands(4)
    rows = np.random.default_rng(7).choice(ops.wl.M, size=48, replace=False)
    A = np.ascontiguousarray(ops.A[rows])
    ref = (A.astype(np.float64) @ ops.B.astype(np.float64)).astype(np.int64)
    assert np.array_equal(oracle.gemm_u8s8s32(A, ops.B).astype(np.int64), ref)


@pytest.mark.parametrize("a,b,M,N,K", [(3, -5, 4, 6, 7), (255, 127, 2, 3, 70000), (255, -128, 3, 2, 70000),
                                       (255, 127, 2, 40, 4096), (200, -100, 1, 1, 1)])
def test_closed_form_constant_operands(oracle, a, b, M, N, K):
    # A == a, B == b: C == K a b, S_B == N b, colsum == K b, chk == rsum == K a N b (mod 2^32);
    # (255,127,70000) drives one entry past 2^31, (.., N=40, K=4096) wraps the row sum only.
    A = np.full((M, K), a, np.uint8)
    B = np.full((K, N), b, np.int8)
    r = oracle.checked_gemm(A, B)
    assert (r.C == to_i32(K * a * b)).all()
    assert (r.S_B == N * b).all() and (r.colsum == K * b).all()
    assert (r.chk == to_i32(K * a * N * b)).all() and (r.rsum == to_i32(K * a * N * b)).all()
    assert r.err_count == 0
    if (a, b, K) == (255, 127, 70000):
        assert K * a * b > 2**31 - 1 and r.C[0, 0] == K * a * b - 2**32


@pytest.mark.parametrize("cfg", [0, 1, 2])
def test_clean_runs_never_flag(oracle, cfg):
    # Table II, column "no error": 0 detected.  Eq. 2b holds identically mod 2^32.
    wl = wlmod.WORKLOADS[cfg]
    M, N, K = min(wl.M, 32), min(wl.N, 256), min(wl.K, 256)
    for rep in range(40):
        rng = wlmod.rng_for(cfg, rep)
        A = wlmod.draw_a(rng, M, K, relu_like=(rep % 2 == 1))
        B = rng.integers(-128, 128, size=(K, N), dtype=np.int8)
        r = oracle.checked_gemm(A, B)
        assert r.err_count == 0 and not r.flags.any()
        assert np.array_equal(r.rsum, r.chk)


def test_c_flip_always_flags_exactly_its_row(oracle):
    # Section IV-C-2 / Table II "error in C": the row sum moves by +-2^b, never 0 mod 2^32.
    rng = wlmod.rng_for(0, 3)
    A = wlmod.draw_a(rng, 6, 40)
    B = wlmod.draw_b(rng, 40, 9)
    for (r_, c_) in [(0, 0), (5, 8), (2, 3)]:
        for bit in range(32):
            res = oracle.checked_gemm(A, B, flips_c=[(r_, c_, 1 << bit)])
            want = np.zeros(6, np.int32)
            want[r_] = 1
            assert res.flags.tolist() == want.tolist() and res.err_count == 1
            clean = oracle.gemm_u8s8s32(A, B)
            assert (res.C.view(np.uint32)[r_, c_] ^ clean.view(np.uint32)[r_, c_]) == (1 << bit)
            diff = res.C != clean
            assert diff.sum() == 1 and diff[r_, c_]


def test_b_flip_flags_rows_with_nonzero_activation(oracle):
    # Section IV-C-1 with modulus 2^32: the row sum of row p moves by d*A[p][k], |d| = 2^b <= 128,
    # so row p is flagged iff A[p][k] != 0, and C is corrupted in exactly those rows.
    rng = wlmod.rng_for(3, 1)
    M, N, K = 24, 17, 33
    A = wlmod.draw_a(rng, M, K, relu_like=True)
    B = rng.integers(-128, 128, size=(K, N), dtype=np.int8)
    clean = oracle.gemm_u8s8s32(A, B)
    for t in range(60):
        k, j, bit = int(rng.integers(K)), int(rng.integers(N)), int(rng.integers(8))
        res = oracle.checked_gemm(A, B, flips_b=[(k, j, bit)])
        want = (A[:, k] != 0).astype(np.int32)
        assert res.flags.tolist() == want.tolist()
        corrupted_rows = (res.C != clean).any(axis=1)
        assert corrupted_rows.tolist() == (want == 1).tolist()
        assert ((res.C != clean).sum(axis=0) > 0).nonzero()[0].tolist() in ([j], [])


def test_a_flip_is_never_flagged(oracle):
    # Section IV-C-3: only B is encoded; C and the checksum column see the same A.
    rng = wlmod.rng_for(2, 1)
    A = wlmod.draw_a(rng, 8, 50)
    B = wlmod.draw_b(rng, 50, 12)
    clean = oracle.gemm_u8s8s32(A, B)
    for t in range(40):
        i, k, bit = int(rng.integers(8)), int(rng.integers(50)), int(rng.integers(8))
        res = oracle.checked_gemm(A, B, flips_a=[(i, k, bit)])
        assert res.err_count == 0
        changed = (res.C != clean).any(axis=1).nonzero()[0].tolist()
        assert changed in ([i], [])     # [] only if B[k,:] == 0


def exact_requant(t: int, mult: np.float32, zC: int) -> int:
    """round-half-even of the exact rational t*mult, plus zC, clamped to [0,255]."""
    q = Fraction(t) * Fraction(float(mult))
    fl = q.numerator // q.denominator
    rem = q - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return min(255, max(0, fl + zC))


def test_requant_ties_saturation_and_rational(oracle):
    colsum = np.array([0, 0, 0, 0, 0, 0, 0], np.int32)
    C = np.array([[1, 3, 5, -1, -3, 1000, -1000]], np.int32)
    # mult = 0.5: products .5, 1.5, 2.5, -.5, -1.5 are exact ties -> 0, 2, 2, -0, -2
    for prec in ("f64", "f32"):
        out = oracle.requantize(C, colsum, 0, 10, np.float32(0.5), precision=prec)
        assert out.tolist() == [[10, 12, 12, 10, 8, 255, 0]]
    # zero-point correction and bias: t = C - zA*colsum + bias
    colsum = np.array([2, -3], np.int32)
    C2 = np.array([[100, 100]], np.int32)
    out = oracle.requantize(C2, colsum, 128, 0, np.array([1.0, 1.0], np.float32), bias=np.array([0, 1], np.int32))
    assert out.tolist() == [[0, 255]]           # 100-256 = -156 -> 0 ; 100+384+1 = 485 -> 255
    out = oracle.requantize(C2, colsum, 10, 0, np.array([1.0, 0.5], np.float32), bias=np.array([0, 1], np.int32))
    assert out.tolist() == [[80, 66]]           # 100-20 = 80 ; (100+30+1)*0.5 = 65.5 -> 66 (even)
    rng = np.random.default_rng(11)
    t = rng.integers(-2**31, 2**31, size=(3, 200), dtype=np.int64).astype(np.int32)
    t[0, :100] = rng.integers(-40000, 40000, size=100)
    mult = np.exp(rng.uniform(np.log(1e-4), np.log(1e-2), size=200)).astype(np.float32)
    zero = np.zeros(200, np.int32)
    got = oracle.requantize(t, zero, 0, 128, mult, precision="f64")
    for i in range(3):
        for j in range(200):
            assert got[i, j] == exact_requant(int(t[i, j]), mult[j], 128)


@pytest.mark.parametrize("cfg", [1, 3])
def test_requant_f32_within_one_code_of_f64(oracle, cfg):
    ops = wlmod.make_operands(cfg)
    wl = ops.wl
    A, B = ops.A[:64], ops.B
    C = oracle.gemm_u8s8s32(A, B)
    cs = oracle.b_colsum(B)
    q64 = oracle.requantize(C, cs, wl.zA, wl.zC, ops.mult, precision="f64").astype(np.int32)
    q32 = oracle.requantize(C, cs, wl.zA, wl.zC, ops.mult, precision="f32").astype(np.int32)
    assert np.abs(q64 - q32).max() <= 1
    assert (q64 != q32).mean() < 1e-3
    assert q64.min() == 0 and q64.max() == 255          # both clamp ends are exercised
    assert ((q64 > 0) & (q64 < 255)).mean() > 0.02


def test_campaign_helpers_match_full_recomputation(oracle):
    rng = wlmod.rng_for(0, 9)
    M, N, K = 7, 19, 23
    A = wlmod.draw_a(rng, M, K, relu_like=True)
    B = wlmod.draw_b(rng, K, N)
    base = oracle.checked_gemm(A, B)
    n = 50
    r_, c_, b_ = rng.integers(M, size=n), rng.integers(N, size=n), rng.integers(32, size=n)
    flag, val = oracle.campaign_c_flips(base.C, base.chk, r_, c_, b_)
    k_, j_, b8 = rng.integers(K, size=n), rng.integers(N, size=n), rng.integers(8, size=n)
    bflags, bcol = oracle.campaign_b_flips(A, B, base.C, base.chk, k_, j_, b8)
    i_, ka, ba = rng.integers(M, size=n), rng.integers(K, size=n), rng.integers(8, size=n)
    aflag, arow = oracle.campaign_a_flips(A, B, base.S_B, i_, ka, ba, want_rows=True)
    for t in range(n):
        full = oracle.checked_gemm(A, B, flips_c=[(int(r_[t]), int(c_[t]), 1 << int(b_[t]))])
        assert flag[t] == full.flags[r_[t]] and full.err_count == flag[t]
        assert val[t] == full.C[r_[t], c_[t]]
        full = oracle.checked_gemm(A, B, flips_b=[(int(k_[t]), int(j_[t]), int(b8[t]))])
        assert bflags[t].tolist() == full.flags.tolist()
        assert bcol[t].tolist() == full.C[:, j_[t]].tolist()
        full = oracle.checked_gemm(A, B, flips_a=[(int(i_[t]), int(ka[t]), int(ba[t]))])
        assert aflag[t] == full.flags[i_[t]] == 0
        assert arow[t].tolist() == full.C[i_[t]].tolist()


def test_mod127_b_campaign_helper(oracle):
    """The modulus-127 B-fault helper against full recomputation and against the closed form of
    Section IV-C-1: the row sum moves by A[p][k]*d with d = +-2^b, which 127 divides only when it
    divides A[p][k], i.e. for A[p][k] in {0, 127, 254}."""
    rng = wlmod.rng_for(0, 13)
    M, N, K = 9, 15, 20
    A = wlmod.draw_a(rng, M, K)
    A[0, :], A[1, :], A[2, :] = 127, 254, 0
    B = wlmod.draw_b(rng, K, N)
    clean = oracle.gemm_u8s8s32(A, B)
    chk127 = oracle.row_checksum_mod127(A, B)
    n = 40
    k_, j_, b_ = rng.integers(K, size=n), rng.integers(N, size=n), rng.integers(8, size=n)
    flags, col = oracle.campaign_b_flips_mod127(A, B, clean, chk127, k_, j_, b_)
    for t in range(n):
        Cw, fw, nw = oracle.checked_gemm_mod127(A, B, flips_b=[(int(k_[t]), int(j_[t]), int(b_[t]))])
        assert flags[t].tolist() == fw.tolist() and col[t].tolist() == Cw[:, j_[t]].tolist()
        assert flags[t].tolist() == [int(A[p, k_[t]] % 127 != 0) for p in range(M)]


def test_value_and_multibit_campaign_helpers(oracle):
    """The value-replacement and multi-bit helpers against full recomputation, and the closed
    forms that hold at modulus 2^32: any change of a C element moves its row sum; a change of
    B[k][j] by d (0 < |d| <= 255) moves row p by A[p][k]*d, which is 0 only when A[p][k] is."""
    rng = wlmod.rng_for(0, 11)
    M, N, K = 6, 17, 21
    A = wlmod.draw_a(rng, M, K, relu_like=True)
    B = wlmod.draw_b(rng, K, N)
    base = oracle.checked_gemm(A, B)
    n = 60
    r_, c_ = rng.integers(M, size=n), rng.integers(N, size=n)
    new_c = rng.integers(-2**31, 2**31, size=n, dtype=np.int64).astype(np.int32)
    masks = (base.C[r_, c_].view(np.uint32) ^ new_c.view(np.uint32)).astype(np.uint32)
    flag, val = oracle.campaign_c_masks(base.C, base.chk, r_, c_, masks)
    assert val.tolist() == new_c.tolist()
    assert flag.tolist() == (masks != 0).astype(np.int32).tolist()
    k_, j_ = rng.integers(K, size=n), rng.integers(N, size=n)
    new_b = rng.integers(-128, 128, size=n, dtype=np.int32)
    bflags, bcol = oracle.campaign_b_values(A, B, base.C, base.chk, k_, j_, new_b)
    for t in range(n):
        full = oracle.checked_gemm(A, B, flips_c=[(int(r_[t]), int(c_[t]), int(masks[t]))])
        assert flag[t] == full.flags[r_[t]] == full.err_count and val[t] == full.C[r_[t], c_[t]]
        diff = (int(B[k_[t], j_[t]]) & 0xFF) ^ (int(new_b[t]) & 0xFF)
        full = oracle.checked_gemm(A, B, flips_b=[(int(k_[t]), int(j_[t]), bit) for bit in range(8) if diff >> bit & 1])
        assert bflags[t].tolist() == full.flags.tolist()
        assert bcol[t].tolist() == full.C[:, j_[t]].tolist()
        changed = int(new_b[t]) != int(B[k_[t], j_[t]])
        assert bflags[t].tolist() == [int(changed and A[p, k_[t]] != 0) for p in range(M)]


# ---- Algorithm 1 with the printed modulus ------------------------------------------------

def golden():
    with open(os.path.join(GOLDEN, "paper_detection_figures.json")) as f:
        return json.load(f)


def test_mod127_clean_and_c_flips(oracle):
    g = golden()
    rng = wlmod.rng_for(1, 5)
    A = wlmod.draw_a(rng, 5, 64)
    B = rng.integers(-128, 128, size=(64, 11), dtype=np.int8)   # negative row sums included
    rs = oracle.b_checksum_mod127(B)
    assert rs.min() >= 0 and rs.max() <= 126
    assert np.array_equal(rs.astype(np.int64), B.astype(np.int64).sum(axis=1) % 127)
    _, flags, n = oracle.checked_gemm_mod127(A, B)
    assert n == g["clean_false_positives"] == 0
    hits = 0
    for bit in range(32):
        _, flags, n = oracle.checked_gemm_mod127(A, B, flips_c=[(3, 7, 1 << bit)])
        hits += int(flags.tolist() == [0, 0, 0, 1, 0])
    assert 100.0 * hits / 32 == g["mod127_c_flip_detection_percent"]


def test_mod127_b_flip_miss_set_is_the_papers(oracle):
    # Exhaustive: activation value a in 0..255 in row a of A, one flipped bit of B;
    # the row misses exactly for a in {0, 127, 254}: 3 of 256 (Section IV-C-1).
    g = golden()
    K, N = 4, 5
    A = np.zeros((256, K), np.uint8)
    A[:, 2] = np.arange(256, dtype=np.uint8)
    A[:, 0] = 9
    rng = np.random.default_rng(5)
    B = rng.integers(-127, 128, size=(K, N), dtype=np.int8)
    missed = 0
    for bit in range(8):
        _, flags, _ = oracle.checked_gemm_mod127(A, B, flips_b=[(2, 1, bit)])
        silent = np.nonzero(flags == 0)[0].tolist()
        assert silent == g["mod127_b_flip_silent_activation_values"]
        missed += len(silent)
    num, den = g["mod127_b_flip_row_miss_probability"]
    assert Fraction(missed, 8 * 256) == Fraction(num, den)
    assert round(100 * (1 - num / den), 2) == g["mod127_b_flip_detection_lower_bound_percent"]
    # the same flips under the 2^32 check: only a == 0 is silent (and there C is not corrupted)
    for bit in range(8):
        res = oracle.checked_gemm(A, B, flips_b=[(2, 1, bit)])
        assert np.nonzero(res.flags == 0)[0].tolist() == [0]


def test_overhead_model_identity():
    # Section IV-A-1: (kn + 2mk + mn) / (2mnk) == 1/(2m) + 1/n + 1/(2k)
    for wl in wlmod.WORKLOADS:
        m, n, k = wl.M, wl.N, wl.K
        assert Fraction(k * n + 2 * m * k + m * n, 2 * m * n * k) == \
            Fraction(1, 2 * m) + Fraction(1, n) + Fraction(1, 2 * k)


def test_mod127_rowsum_entry_flip_closed_form(oracle):
    """A fault in the stored 8-bit checksum entry rowSum[k] (the case Section IV-C excludes): the checksum
    product of row p moves by A[p][k] * delta, so row p is flagged iff that is not a multiple of 127."""
    rng = np.random.default_rng(77)
    M, N, K = 40, 9, 12
    A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
    A[0, 5], A[1, 5], A[2, 5] = 0, 127, 254
    B = rng.integers(-127, 128, size=(K, N), dtype=np.int8)
    rs = oracle.b_checksum_mod127(B).astype(np.int64)
    for bit in range(8):
        new = np.array([rs[5]], np.int64).astype(np.uint8) ^ np.uint8(1 << bit)
        delta = int(new.view(np.int8)[0]) - int(rs[5])
        _, flags, n = oracle.checked_gemm_mod127(A, B, flips_rowsum=[(5, bit)])
        want = ((A[:, 5].astype(np.int64) * delta) % 127 != 0).astype(np.int32)
        assert np.array_equal(flags, want) and n == int(want.sum())
        assert flags[0] == 0 and flags[1] == 0 and flags[2] == 0


# ---- locating and correcting one faulty element (Section IV, Eq. 2a) ------------------------

def test_column_checksum_row_against_bigint_and_matmul(oracle):
    """S_A and the checksum row S_A B: Python integers on tiny extreme inputs, float64 matmul (exact below
    2^53) on a workload-sized case, and Eq. 2a itself: every column of a clean product sums to its entry."""
    for (M, N, K) in [(1, 1, 1), (2, 3, 4), (5, 2, 3)]:
        for a_val in (0, 255):
            for b_val in (-128, 127):
                A = np.full((M, K), a_val, np.uint8)
                B = np.full((K, N), b_val, np.int8)
                A[0, 0] = 7
                B[0, N - 1] = -3
                S_A = oracle.a_colsum(A)
                want_S = [sum(int(A[i, k]) for i in range(M)) for k in range(K)]
                assert S_A.tolist() == want_S
                chk = oracle.col_checksum(S_A, B)
                want = [sum(want_S[k] * int(B[k, j]) for k in range(K)) for j in range(N)]
                assert [int(v) for v in chk] == [((w + 2**31) % 2**32) - 2**31 for w in want]
    rng = np.random.default_rng(11)
    A = rng.integers(0, 256, size=(256, 1024), dtype=np.uint8)
    B = rng.integers(-128, 128, size=(1024, 300), dtype=np.int8)
    S_A = oracle.a_colsum(A)
    assert np.array_equal(S_A, A.astype(np.int64).sum(axis=0).astype(np.int32))
    exact = (S_A.astype(np.float64) @ B.astype(np.float64)).astype(np.int64)
    chk = oracle.col_checksum(S_A, B)
    assert np.array_equal(chk, (exact & 0xFFFFFFFF).astype(np.uint32).view(np.int32))
    C = oracle.gemm_u8s8s32(A, B)
    assert np.array_equal(oracle.col_sums(C), chk)                       # Eq. 2a on a clean product
    assert np.array_equal(oracle.col_sums(C), C.astype(np.int64).sum(axis=0).astype(np.uint64).astype(np.uint32).view(np.int32))


def test_column_checksum_closed_form_with_wrap(oracle):
    """Constant operands: S_A = M a, checksum row = K M a b, forced past 2^31."""
    M, N, K, a, b = 3000, 3, 40, 255, 127
    A = np.full((M, K), a, np.uint8)
    B = np.full((K, N), b, np.int8)
    assert K * M * a * b > 2**31
    chk = oracle.col_checksum(oracle.a_colsum(A), B)
    want = ((K * M * a * b + 2**31) % 2**32) - 2**31
    assert chk.tolist() == [want] * N


def test_single_c_fault_is_located_and_restored_for_every_bit(oracle):
    rng = np.random.default_rng(12)
    M, N, K = 23, 17, 40
    A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
    B = rng.integers(-128, 128, size=(K, N), dtype=np.int8)
    clean = oracle.checked_gemm(A, B)
    got = oracle.locate_correct(A, B, clean.C, clean.flags)
    assert got.status == 0 and got.rows_violated == 0 and got.cols_violated == 0 and np.array_equal(got.C, clean.C)
    for bit in range(32):
        r, c = int(rng.integers(M)), int(rng.integers(N))
        bad = oracle.checked_gemm(A, B, flips_c=[(r, c, 1 << bit)])
        assert bad.err_count == 1 and bad.flags[r] == 1
        got = oracle.locate_correct(A, B, bad.C, bad.flags)
        assert (got.status, got.row, got.col) == (1, r, c)
        assert got.old_value == int(bad.C[r, c]) and got.new_value == int(clean.C[r, c])
        assert np.array_equal(got.C, clean.C)
        want_cols = np.zeros(N, np.int32)
        want_cols[c] = 1
        assert np.array_equal(got.col_flags, want_cols)
    # an arbitrary replacement value (second fault model of Section IV-C) is repaired just the same
    bad = oracle.checked_gemm(A, B, flips_c=[(5, 6, 0xDEADBEEF)])
    got = oracle.locate_correct(A, B, bad.C, bad.flags)
    assert got.status == 1 and np.array_equal(got.C, clean.C)


def test_patterns_that_are_not_one_element_are_left_alone(oracle):
    rng = np.random.default_rng(13)
    M, N, K = 20, 30, 25
    A = rng.integers(1, 256, size=(M, K), dtype=np.uint8)
    B = rng.integers(-127, 128, size=(K, N), dtype=np.int8)
    clean = oracle.checked_gemm(A, B)
    # two faults: distinct rows and columns / same row / same column
    for flips, rows, cols in (([(1, 2, 1 << 5), (7, 9, 1 << 20)], 2, 2), ([(4, 2, 1), (4, 9, 1 << 31)], 1, 2),
                              ([(4, 3, 1 << 8), (11, 3, 1 << 9)], 2, 1)):
        bad = oracle.checked_gemm(A, B, flips_c=flips)
        got = oracle.locate_correct(A, B, bad.C, bad.flags)
        assert got.status == 2 and (got.rows_violated, got.cols_violated) == (rows, cols)
        assert np.array_equal(got.C, bad.C) and got.row == -1 and got.col == -1
    # a fault in B after it was encoded corrupts a whole column of C consistently with the B in memory:
    # rows violate Eq. 2b, no column violates Eq. 2a, nothing is "corrected"
    bad = oracle.checked_gemm(A, B, flips_b=[(3, 8, 6)])
    assert bad.err_count == M
    B_bad = B.copy()
    B_bad.view(np.uint8)[3, 8] ^= np.uint8(1 << 6)
    got = oracle.locate_correct(A, B_bad, bad.C, bad.flags, S_B=clean.S_B)
    assert got.status == 2 and got.rows_violated == M and got.cols_violated == 0 and np.array_equal(got.C, bad.C)
    # ... even when only one row shows it (all other rows have a zero at that k)
    A1 = A.copy()
    A1[:, 3] = 0
    A1[6, 3] = 9
    bad = oracle.checked_gemm(A1, B, flips_b=[(3, 8, 6)])
    assert bad.err_count == 1
    got = oracle.locate_correct(A1, B_bad, bad.C, bad.flags, S_B=oracle.b_checksum(B))
    assert got.status == 2 and (got.rows_violated, got.cols_violated) == (1, 0) and np.array_equal(got.C, bad.C)
    # one column violated, no row flagged (a stale verdict): not an element either
    C2 = clean.C.copy()
    C2[2, 2] ^= 4
    got = oracle.locate_correct(A, B, C2, clean.flags)
    assert got.status == 2 and (got.rows_violated, got.cols_violated) == (0, 1) and np.array_equal(got.C, C2)


def test_the_two_correction_formulas_agree_or_nothing_is_written(oracle):
    """One row and one column violated, but by different elements' worth: the column formula and the row formula
    give different values, and C is left as it is."""
    rng = np.random.default_rng(14)
    M, N, K = 9, 8, 16
    A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
    B = rng.integers(-128, 128, size=(K, N), dtype=np.int8)
    clean = oracle.checked_gemm(A, B)
    C2 = clean.C.copy()
    C2[3, 5] += 100
    flags = np.zeros(M, np.int32)
    flags[7] = 1                      # verdicts that name another row than the one the column points at
    got = oracle.locate_correct(A, B, C2, flags)
    assert got.status == 2 and (got.rows_violated, got.cols_violated) == (1, 1) and np.array_equal(got.C, C2)
