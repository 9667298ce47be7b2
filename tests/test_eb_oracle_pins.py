"""Pins for the EmbeddingBag oracle (oracle/eb_oracle.*): each test fixes it to something
other than itself - exact rational arithmetic on tiny inputs, the identity the check rests
on (arXiv 2103.00130 Section V, Eq. 4), an independent library routine, integer special
cases, and the closed-form detection threshold of Algorithm 2."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import eb_oracle as eb
from paper_2103_00130_amd import eb_workloads as w


def tiny(seed, rows=7, d=5, n_bags=4, weighted=False, regime="uniform"):
    rng = np.random.default_rng(seed)
    T, scale, bias = w.draw_table(rng, rows, d, regime)
    lens = rng.integers(0, 5, size=n_bags)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    indices = rng.integers(0, rows, size=int(offsets[-1]), dtype=np.int64)
    weights = w.draw_weights(rng, indices.size) if weighted else None
    return T, scale, bias, indices, offsets, weights


def exact_rows(T, scale, bias, indices, offsets, weights):
    """Section III-C in exact rational arithmetic (float inputs are exact rationals)."""
    out = []
    for b in range(offsets.size - 1):
        row = [Fraction(0)] * T.shape[1]
        for p in range(offsets[b], offsets[b + 1]):
            i = int(indices[p])
            wi = Fraction(float(weights[p])) if weights is not None else Fraction(1)
            for j in range(T.shape[1]):
                row[j] += wi * (Fraction(float(scale[i])) * int(T[i, j]) + Fraction(float(bias[i])))
        out.append(row)
    return out


@pytest.mark.parametrize("weighted", [False, True])
def test_forward_against_exact_rational_arithmetic(weighted):
    for seed in range(5):
        T, scale, bias, indices, offsets, weights = tiny(seed, weighted=weighted)
        exact = exact_rows(T, scale, bias, indices, offsets, weights)
        R64 = eb.forward(T, scale, bias, indices, offsets, weights, "f64")
        R32 = eb.forward(T, scale, bias, indices, offsets, weights, "f32")
        tol = eb.roundoff_tolerance(T, scale, bias, indices, offsets, weights)
        for b, row in enumerate(exact):
            for j, x in enumerate(row):
                assert abs(float(x) - R64[b, j]) <= 1e-13 * max(1.0, abs(float(x)))
                assert abs(float(x) - float(R32[b, j])) <= tol[b] + 1e-30


def test_eq4_identity_in_exact_arithmetic():
    """Eq. 4: sum_j R[j] == sum_{i in I} (alpha_i * C_T[i] + d * beta_i), exactly, with C_T the
    oracle's row sums.  A dropped factor d, a wrong row sum or a swapped scale/bias fails."""
    for seed in range(5):
        T, scale, bias, indices, offsets, _ = tiny(seed + 10, rows=9, d=6)
        C_T = eb.table_rowsums(T)
        assert np.array_equal(C_T, T.astype(np.int64).sum(axis=1))
        exact = exact_rows(T, scale, bias, indices, offsets, None)
        d = T.shape[1]
        for b, row in enumerate(exact):
            rhs = sum((Fraction(float(scale[int(i)])) * int(C_T[int(i)]) + d * Fraction(float(bias[int(i)]))
                       for i in indices[offsets[b]:offsets[b + 1]]), Fraction(0))
            assert sum(row, Fraction(0)) == rhs


@pytest.mark.parametrize("weighted", [False, True])
def test_forward_against_library_embedding_bag(weighted):
    """The dequantized table pooled by torch's embedding_bag (an independent implementation
    of the operator the paper's footnote points to), in double."""
    rng = np.random.default_rng(3)
    T, scale, bias = w.draw_table(rng, 300, 24, "gauss")
    indices, offsets = w.draw_bags(rng, 300, 40, 9, "ragged")
    weights = w.draw_weights(rng, indices.size) if weighted else None
    table = torch.from_numpy(scale.astype(np.float64)[:, None] * T.astype(np.float64) + bias.astype(np.float64)[:, None])
    ref = torch.nn.functional.embedding_bag(
        torch.from_numpy(indices), table, torch.from_numpy(offsets[:-1].copy()), mode="sum",
        per_sample_weights=None if weights is None else torch.from_numpy(weights.astype(np.float64))).numpy()
    R64 = eb.forward(T, scale, bias, indices, offsets, weights, "f64")
    assert np.allclose(R64, ref, rtol=1e-12, atol=1e-12)
    assert np.any(np.diff(offsets) == 0) and np.all(R64[np.diff(offsets) == 0] == 0)  # empty bags pool to zero
    R32 = eb.forward(T, scale, bias, indices, offsets, weights, "f32")
    tol = eb.roundoff_tolerance(T, scale, bias, indices, offsets, weights)
    assert np.all(np.abs(R32.astype(np.float64) - ref) <= tol[:, None] + 1e-30)


def test_integer_table_is_exact_integer_pooling():
    """scale 1, bias 0: R is the integer column sum of the pooled rows, exact in float."""
    rng = np.random.default_rng(5)
    T, scale, bias = w.draw_table(rng, 500, 32, "integer")
    indices, offsets = w.draw_bags(rng, 500, 20, 50, "spread")
    R = eb.forward(T, scale, bias, indices, offsets, None, "f32")
    for b in range(20):
        assert np.array_equal(R[b].astype(np.int64), T[indices[offsets[b]:offsets[b + 1]]].astype(np.int64).sum(axis=0))
    out = eb.checked_eb(T, scale, bias, indices, offsets)
    assert np.array_equal(out.rsum, out.csum) and not out.flags.any()  # both sides are the same integer


def test_f32_order_is_the_stated_one():
    """Float result retyped with numpy scalars for one bag: per column fma in index order,
    biases summed apart and added last (the product alpha*code is exact in double, so one
    rounding of the double sum to float is the fused operation unless the addends are more
    than 2^21 apart, which these inputs exclude)."""
    rng = np.random.default_rng(8)
    T, scale, bias = w.draw_table(rng, 50, 8, "uniform")
    indices = rng.integers(0, 50, size=30, dtype=np.int64)
    offsets = np.array([0, 30], dtype=np.int64)
    weights = w.draw_weights(rng, 30)
    R = eb.forward(T, scale, bias, indices, offsets, weights, "f32")[0]
    acc = np.zeros(8, dtype=np.float32)
    bsum = np.float32(0)
    for p, i in enumerate(indices):
        a, c = np.float32(weights[p] * scale[i]), np.float32(weights[p] * bias[i])
        acc = (np.float64(a) * T[i].astype(np.float64) + acc.astype(np.float64)).astype(np.float32)
        bsum = np.float32(bsum + c)
    assert np.array_equal(R, (acc + bsum).astype(np.float32))


def test_algorithm2_threshold_closed_form():
    """Integer table, one bag: every quantity is an exact integer, so Algorithm 2's verdict on
    a planted error of size e in R is known in closed form: flagged iff e > bound * max(RSum + e, CSum)."""
    rng = np.random.default_rng(9)
    T, scale, bias = w.draw_table(rng, 200, 64, "integer")
    indices = rng.integers(0, 200, size=100, dtype=np.int64)
    offsets = np.array([0, 100], dtype=np.int64)
    C_T = eb.table_rowsums(T)
    R = eb.forward(T, scale, bias, indices, offsets, None, "f32")
    csum = int(C_T[indices].astype(np.int64).sum())
    assert int(R.astype(np.int64).sum()) == csum
    for e in (0, 1, 2, 4, 8, 16, 32, 64, 128):
        Rb = R.copy()
        Rb[0, 17] += e
        c = eb.check(Rb, 200, scale, bias, C_T, indices, offsets, None, 1e-5)
        assert c.rsum[0] == csum + e and c.csum[0] == csum
        assert int(c.flags[0]) == int(e > 1e-5 * (csum + e)), (e, csum)
    # csum is about 100*64*127.5 = 816000: the bound 1e-5 passes errors up to 8, catches 16 and above
    assert 800000 < csum < 832000
    # NaN and Inf in R are reported
    for bad in (np.nan, np.inf):
        Rb = R.copy()
        Rb[0, 3] = bad
        assert eb.check(Rb, 200, scale, bias, C_T, indices, offsets, None, 1e-5).flags[0] == 1


def test_table_flip_campaign_matches_the_threshold():
    """Section VI-B-2 on an integer table: a flip of bit k in a pooled element changes RSum by
    2^k times the number of times the row is pooled, CSum not at all; detection is then decided
    by the closed form above.  High bits (4..7) are all caught, low bits 0..2 all missed."""
    rng = np.random.default_rng(11)
    T, scale, bias = w.draw_table(rng, 400, 64, "integer")
    indices, offsets = w.draw_bags(rng, 400, 6, 100, "fixed")
    C_T = eb.table_rowsums(T)
    for bits, lo in (("high", 4), ("low", 0)):
        f_row, f_col, f_bit = w.draw_table_flips(rng, indices, 64, 40, bits)
        assert f_bit.min() >= lo and f_bit.max() < lo + 4
        flags = eb.campaign_table_flips(T, scale, bias, C_T, indices, offsets, None, f_row, f_col, f_bit)
        for t in range(40):
            for b in range(6):
                idx = indices[offsets[b]:offsets[b + 1]]
                mult = int((idx == f_row[t]).sum())
                csum = int(C_T[idx].astype(np.int64).sum())
                delta = mult * (1 << int(f_bit[t])) * (1 if not (T[f_row[t], f_col[t]] >> f_bit[t]) & 1 else -1)
                assert int(flags[t, b]) == int(abs(delta) > 1e-5 * max(csum + delta, csum)), (t, b)
        detected = flags.any(axis=1)
        if bits == "high":
            assert detected.all()
        else:
            assert not detected[f_bit <= 2].any()


def test_invalid_indices_are_skipped_and_reported():
    T, scale, bias, _, _, _ = tiny(1)
    indices = np.array([0, 99, 3, -1, 2], dtype=np.int64)
    offsets = np.array([0, 2, 3, 5], dtype=np.int64)
    out = eb.checked_eb(T, scale, bias, indices, offsets)
    ref = eb.checked_eb(T, scale, bias, np.array([0, 3, 2], dtype=np.int64), np.array([0, 1, 2, 3], dtype=np.int64))
    assert np.array_equal(out.R, ref.R)
    assert out.flags.tolist() == [2, 0, 2] and ref.flags.tolist() == [0, 0, 0]


def test_clean_runs_and_robust_band():
    """Clean lookups in the regime of mostly positive values: |RSum - CSum| is round-off only,
    orders of magnitude under the bound, and every verdict is robust to the order of the sums."""
    wl = w.EbWorkload("t", 5000, 64, 64, 100, True, "uniform")
    x = w.make_inputs(wl, tag=1)
    out = eb.checked_eb(x.T, x.scale, x.bias, x.indices, x.offsets, x.weights)
    assert not out.flags.any() and out.robust.all()
    assert np.all(np.abs(out.rsum - out.csum) < 1e-6 * np.abs(out.csum))


# ---- 4-bit tables (two codes per byte) ---------------------------------------------------------

def unpack(Tp):
    out = np.empty((Tp.shape[0], Tp.shape[1] * 2), dtype=np.uint8)
    out[:, 0::2] = Tp & 15
    out[:, 1::2] = Tp >> 4
    return out


def test_int4_equals_the_8bit_oracle_on_unpacked_codes():
    """A 4-bit table is the 8-bit table of its unpacked codes: row sums, both precisions of the
    lookup, Algorithm 2 and the flip campaign must agree (the 8-bit path is pinned above), and the
    unpacking itself is pinned by hand-written bytes."""
    Tp = np.array([[0x21, 0xF0], [0x0A, 0x37]], dtype=np.uint8)
    assert unpack(Tp).tolist() == [[1, 2, 0, 15], [10, 0, 7, 3]]
    assert eb.table_rowsums(Tp, bits=4).tolist() == [18, 20]
    for seed, weighted in ((1, False), (2, True)):
        rng = np.random.default_rng(seed)
        Tp, scale, bias = w.draw_table(rng, 300, 64, "uniform", bits=4)
        assert Tp.shape == (300, 32)
        T8 = unpack(Tp)
        assert T8.max() == 15
        indices, offsets = w.draw_bags(rng, 300, 30, 20, "ragged")
        weights = w.draw_weights(rng, indices.size) if weighted else None
        assert np.array_equal(eb.table_rowsums(Tp, bits=4), eb.table_rowsums(T8))
        for prec in ("f32", "f64"):
            assert np.array_equal(eb.forward(Tp, scale, bias, indices, offsets, weights, prec, bits=4),
                                  eb.forward(T8, scale, bias, indices, offsets, weights, prec))
        a, c = eb.checked_eb(Tp, scale, bias, indices, offsets, weights, bits=4), eb.checked_eb(T8, scale, bias, indices, offsets, weights)
        assert np.array_equal(a.flags, c.flags) and np.array_equal(a.csum, c.csum) and np.array_equal(a.rsum, c.rsum)
        f_row, f_col, f_bit = w.draw_table_flips(rng, indices, 64, 30, "high", code_bits=4)
        assert f_bit.min() >= 2 and f_bit.max() <= 3
        C_T = eb.table_rowsums(T8)
        assert np.array_equal(eb.campaign_table_flips(Tp, scale, bias, C_T, indices, offsets, weights, f_row, f_col, f_bit, bits=4),
                              eb.campaign_table_flips(T8, scale, bias, C_T, indices, offsets, weights, f_row, f_col, f_bit))


def test_int4_flip_changes_the_named_element_only():
    rng = np.random.default_rng(4)
    Tp, scale, bias = w.draw_table(rng, 50, 32, "integer", bits=4)
    indices = np.arange(50, dtype=np.int64)
    offsets = np.array([0, 50], dtype=np.int64)
    C_T = eb.table_rowsums(Tp, bits=4)
    base = eb.forward(Tp, scale, bias, indices, offsets, None, "f32", bits=4)[0]
    for row, col, bit in ((3, 0, 0), (3, 1, 3), (49, 31, 2), (10, 16, 1)):
        T2 = Tp.copy()
        T2[row, col // 2] ^= np.uint8(1 << (bit + 4 * (col & 1)))
        got = eb.forward(T2, scale, bias, indices, offsets, None, "f32", bits=4)[0]
        diff = got - base
        assert abs(diff[col]) == (1 << bit) and np.count_nonzero(diff) == 1
        flags = eb.campaign_table_flips(Tp, scale, bias, C_T, indices, offsets, None, [row], [col], [bit], bits=4)
        # RSum is about 50*32*7.5 = 12000: the bound 1e-5 is 0.12, every flip is caught
        assert flags[0, 0] == 1


def test_paper_figures_fixture():
    """What the paper prints for the EmbeddingBag check (tests/golden/paper_eb_figures.json): the bound
    the oracle defaults to, the shapes the workloads module names, and the overhead model, which must
    be the ratio of the two operation counts it is derived from."""
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_eb_figures.json")))
    assert eb.REL_BOUND == g["relative_bound"]
    t1 = g["table1"]
    assert sorted(w.TABLE1) == t1["columns"]
    for d, wl in w.TABLE1.items():
        assert (wl.rows, wl.d, wl.pooling, wl.n_bags) == (t1["rows"], d, t1["average_pooling"], t1["batch"])
    for m, d in ((100, 32), (100, 256), (7, 64)):
        env = {"m": Fraction(m), "d": Fraction(d), "p": Fraction(8)}
        assert eval(g["ops_extra"], {}, env) / eval(g["ops_without_abft"], {}, env) == eval(g["overhead_fraction"], {}, env)
        # the row sum is one 32-bit word per row of p*d bits
        assert eval(g["rowsum_memory_fraction"], {}, env) == Fraction(32, 8 * d)
    hi, lo, fp = (Fraction(*g["table3_detected"][k]) for k in ("high_bits", "low_bits", "no_error"))
    assert hi > lo > fp
