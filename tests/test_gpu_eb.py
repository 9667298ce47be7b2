"""GPU parity of the ABFT-checked EmbeddingBag (include/abft_eb.h) against the CPU oracle
(oracle/eb_oracle.*), through the C ABI.

Bar: R is compared element by element with the operator's definition evaluated in double
(Section III-C) within the derived binary32 round-off tolerance - that is the parity claim; the
table's row sums and the batch kernel's CSum are bit-exact; RSum agrees to double rounding (the
kernels add the same doubles in a tree, the oracle in sequence); the flags are equal wherever the
oracle says the comparison cannot depend on that order, which the tests require to be everywhere
for their seeds.  On top of that R is checked bit for bit against a binary32 evaluation in the
kernels' documented order: a reproducibility check, not the oracle."""
import numpy as np
import pytest
import torch

from oracle import eb_oracle as eb
from paper_2103_00130_amd import eb_workloads as w

pytestmark = pytest.mark.gpu

VARIANTS = {"auto": 0, "batch": 0x100, "group": 0x200}


@pytest.fixture(scope="module")
def b():
    from paper_2103_00130_amd import binding
    assert torch.cuda.is_available()
    return binding


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


class GpuTable:
    def __init__(self, b, T, scale, bias, aligned=False, bits=8):
        self.b = b
        self.Tp = b.abft_eb_pack_rowsum(dev(T), dev(scale), dev(bias), (b.ABFT_EB_PACK_LINE_ALIGNED if aligned else 0) |
                                        (b.ABFT_EB_PACK_INT4 if bits == 4 else 0))
        torch.cuda.synchronize()

    def rowsums(self):
        out = torch.empty(self.Tp.rows, dtype=torch.int32, device="cuda")
        self.b.abft_eb_table_get_rowsums(self.Tp, out)
        return out.cpu().numpy()

    def run(self, indices, offsets, weights=None, variant="auto", check=True, bound=1e-5, ldr=None):
        b, d = self.b, self.Tp.d
        n_bags = offsets.size - 1
        ldr = d if ldr is None else ldr
        Rbuf = torch.full((max(n_bags, 1), ldr), -7.0, dtype=torch.float32, device="cuda")
        R = Rbuf[:, :d]
        flags = torch.full((max(n_bags, 1),), -1, dtype=torch.int32, device="cuda")
        rsum = torch.full((max(n_bags, 1),), -1.0, dtype=torch.float64, device="cuda")
        csum = torch.full((max(n_bags, 1),), -1.0, dtype=torch.float64, device="cuda")
        b.abft_eb_u8_checked(self.Tp, dev(indices) if indices.size else torch.empty(0, dtype=torch.int64, device="cuda"),
                             dev(offsets), R[:n_bags] if n_bags else R[:0], flags, dev(weights), rsum, csum, bound,
                             VARIANTS[variant] | (0 if check else b.ABFT_EB_NOCHECK))
        torch.cuda.synchronize()
        return {"R": R[:n_bags].cpu().numpy(), "flags": flags[:n_bags].cpu().numpy(), "rsum": rsum[:n_bags].cpu().numpy(),
                "csum": csum[:n_bags].cpu().numpy(), "pad": Rbuf[:, d:].cpu().numpy()}


def same_bits(x, y):
    return np.array_equal(np.ascontiguousarray(x).view(np.uint32), np.ascontiguousarray(y).view(np.uint32))


def compare(out, ref, T, scale, bias, indices, offsets, weights, bits=8, csum_in_index_order=False):
    """THE PARITY BAR for R: element by element against the operator's definition evaluated in double
    (Section III-C: R = sum_i (alpha_i * eb_i + beta_i * e_d), `forward(..., "f64")`), within the
    round-off bound of a binary32 evaluation of that sum that roundoff_tolerance() derives.
    Row sums, flags: equal to the oracle's.  CSum: its terms are exact to one rounding on both sides; the
    batch kernel adds them in index order like the oracle (bit for bit), the group kernel adds them lanes
    in parallel, which moves the sum by at most m * 2^-53 * sum|term| (|term| <= d * (|scale| * code_max +
    |bias|): the magnitude roundoff_tolerance() is built on).  RSum: a binary64 sum of d binary32 values in
    the kernel's own order.
    After the parity checks, one REPRODUCIBILITY check that is not the oracle: R bit for bit against the
    binary32 evaluation in the one order the kernels document (one fused multiply-add per pooled row in
    index order, biases summed apart) - it pins that order from run to run and between the two kernels."""
    tol = eb.roundoff_tolerance(T, scale, bias, indices, offsets, weights, bits)
    R64 = eb.forward(T, scale, bias, indices, offsets, weights, "f64", bits)
    ok = np.isfinite(R64)
    assert np.array_equal(np.isfinite(out["R"]), ok)
    assert np.all(np.abs(out["R"].astype(np.float64) - R64)[ok] <= (tol[:, None] + np.zeros_like(R64))[ok] + 1e-30), \
        "R differs from the definition (double) by more than the binary32 round-off bound"
    if csum_in_index_order:
        assert np.array_equal(out["csum"].view(np.uint64), ref.csum.view(np.uint64)), "CSum differs"
    else:
        d = out["R"].shape[1]
        fin_c = np.isfinite(ref.csum)
        assert np.array_equal(np.isfinite(out["csum"]), fin_c)
        assert np.all(np.abs(out["csum"] - ref.csum)[fin_c] <= (tol * d * 2.0 ** -29)[fin_c]), "CSum differs"
    fin = np.isfinite(ref.rsum)
    assert np.allclose(out["rsum"][fin], ref.rsum[fin], rtol=1e-13, atol=0)
    assert ref.robust.all(), "seed gives a comparison that depends on summation order; pick another"
    assert np.array_equal(out["flags"], ref.flags)
    # reproducibility of the documented evaluation order (not the parity bar)
    assert same_bits(out["R"], ref.R), "R is not reproducible against the binary32 evaluation in the documented order"


@pytest.mark.parametrize("d", [16, 32, 64, 128, 256, 512])
@pytest.mark.parametrize("variant", ["batch", "group"])
def test_eb_matches_oracle(b, d, variant):
    for weighted, regime, lengths in ((False, "uniform", "spread"), (True, "gauss", "ragged"), (False, "integer", "ragged")):
        rng = w.rng_for(100 + d, 0, int(weighted))
        T, scale, bias = w.draw_table(rng, 3000, d, regime)
        indices, offsets = w.draw_bags(rng, 3000, 150, 40, lengths)
        # one lookup long enough to span several staging chunks of the group kernel at every d
        extra = rng.integers(0, 3000, size=1300, dtype=np.int64)
        indices = np.concatenate([indices, extra])
        offsets = np.concatenate([offsets, [indices.size]]).astype(np.int64)
        weights = w.draw_weights(rng, indices.size) if weighted else None
        aligned = regime == "gauss"     # one of the three passes runs on line-aligned records
        g = GpuTable(b, T, scale, bias, aligned)
        stride = {16: 32, 32: 64, 64: 128}.get(d, d + 16) if aligned else d + 16
        assert b.abft_eb_table_dims(g.Tp) == (3000, d, stride, 8)
        assert np.array_equal(g.rowsums(), eb.table_rowsums(T))
        ref = eb.checked_eb(T, scale, bias, indices, offsets, weights)
        out = g.run(indices, offsets, weights, variant)
        compare(out, ref, T, scale, bias, indices, offsets, weights, csum_in_index_order=variant == "batch")
        if regime != "gauss":
            assert not out["flags"].any()


def test_variants_agree_and_nocheck_is_the_same_lookup(b):
    rng = w.rng_for(7)
    T, scale, bias = w.draw_table(rng, 5000, 64, "gauss")
    indices, offsets = w.draw_bags(rng, 5000, 700, 30, "ragged")
    weights = w.draw_weights(rng, indices.size)
    g = GpuTable(b, T, scale, bias)
    outs = [g.run(indices, offsets, weights, v, check=c, ldr=72) for v in ("batch", "group") for c in (True, False)]
    for o in outs[1:]:
        assert same_bits(o["R"], outs[0]["R"])
        assert np.all(o["pad"] == -7.0)          # columns past d are not written
    assert np.array_equal(outs[0]["flags"], outs[2]["flags"])
    assert not outs[1]["flags"].any() and not outs[3]["flags"].any()   # no check: only bad indices are reported
    assert np.all(outs[1]["rsum"] == -1.0)                              # and the diagnostics are left alone


def test_bad_indices_empty_batches_and_clamped_offsets(b):
    rng = w.rng_for(8)
    T, scale, bias = w.draw_table(rng, 100, 32, "uniform")
    g = GpuTable(b, T, scale, bias)
    indices = np.array([5, 100, 7, -3, 9, 2**40, 11, 12], dtype=np.int64)
    offsets = np.array([0, 2, 2, 5, 8], dtype=np.int64)
    ref = eb.checked_eb(T, scale, bias, indices, offsets)
    assert ref.flags.tolist() == [2, 0, 2, 2]
    for v in ("batch", "group"):
        out = g.run(indices, offsets, None, v)
        assert same_bits(out["R"], ref.R) and np.array_equal(out["flags"], ref.flags)
        assert np.all(out["R"][1] == 0.0)
        nc = g.run(indices, offsets, None, v, check=False)
        assert nc["flags"].tolist() == [2, 0, 2, 2]
        # offsets beyond the index array are clamped: the last lookup pools what exists
        wild = np.array([0, 2, 2, 5, 1000], dtype=np.int64)
        out = g.run(indices, wild, None, v)
        assert same_bits(out["R"], ref.R)
        # no lookups at all
        empty = g.run(np.zeros(0, dtype=np.int64), np.zeros(1, dtype=np.int64), None, v)
        assert empty["R"].shape == (0, 32)
        # only empty lookups
        out = g.run(np.zeros(0, dtype=np.int64), np.zeros(6, dtype=np.int64), None, v)
        assert np.all(out["R"] == 0.0) and not out["flags"].any()
    with pytest.raises(b.AbftError):
        R = torch.empty((4, 32), dtype=torch.float32, device="cuda")
        b.abft_eb_u8_checked(g.Tp, dev(indices), dev(offsets), R, None)    # flags are required when checking
    with pytest.raises(b.AbftError):
        R = torch.empty((4, 33), dtype=torch.float32, device="cuda")[:, :32]  # ldr not a multiple of 4
        b.abft_eb_u8_checked(g.Tp, dev(indices), dev(offsets), R, torch.empty(4, dtype=torch.int32, device="cuda"))


def test_non_finite_parameters_are_reported(b):
    rng = w.rng_for(9)
    T, scale, bias = w.draw_table(rng, 200, 64, "uniform")
    scale[17] = np.inf
    bias[23] = np.nan
    indices, offsets = w.draw_bags(rng, 200, 40, 20, "fixed")
    indices[5], indices[45] = 17, 23      # lookups 0 and 2
    g = GpuTable(b, T, scale, bias)
    ref = eb.checked_eb(T, scale, bias, indices, offsets)
    assert ref.flags[0] == 1 and ref.flags[2] == 1
    for v in ("batch", "group"):
        out = g.run(indices, offsets, None, v)
        assert np.array_equal(out["flags"], ref.flags)
        assert np.array_equal(np.isnan(out["R"]), np.isnan(ref.R))
        ok = ~np.isnan(ref.R)
        assert np.array_equal(out["R"][ok], ref.R[ok])


def test_zero_bound_and_threshold_on_integer_table(b):
    """Integer table: RSum and CSum are the same integer, so even bound 0 passes a clean lookup;
    a planted flip is caught or passed exactly as the closed form says."""
    rng = w.rng_for(10)
    T, scale, bias = w.draw_table(rng, 400, 64, "integer")
    indices, offsets = w.draw_bags(rng, 400, 6, 100, "fixed")
    g = GpuTable(b, T, scale, bias)
    C_T = eb.table_rowsums(T)
    for v in ("batch", "group"):
        assert not g.run(indices, offsets, None, v, bound=0.0)["flags"].any()
    bag0 = indices[offsets[0]:offsets[1]]
    row, col = int(next(i for i in bag0 if (bag0 == i).sum() == 1)), 5   # pooled exactly once by lookup 0
    for bit in range(8):
        b.abft_eb_table_flip_bit(g.Tp, row, col, bit)
        T2 = T.copy()
        T2[row, col] ^= np.uint8(1 << bit)
        ref = eb.checked_eb(T2, scale, bias, indices, offsets, C_T=C_T)
        for v in ("batch", "group"):
            out = g.run(indices, offsets, None, v)
            assert same_bits(out["R"], ref.R) and np.array_equal(out["flags"], ref.flags)
            assert out["flags"][0] == int(bit >= 4)     # CSum is about 816000: 1e-5 of it lies between 8 and 16
        b.abft_eb_table_flip_bit(g.Tp, row, col, bit)
    assert np.array_equal(g.rowsums(), C_T)
    assert not g.run(indices, offsets, None, "group")["flags"].any()


@pytest.mark.parametrize("regime", ["uniform", "gauss"])
def test_table_flip_campaign_matches_oracle(b, regime):
    """Section VI-B-2 at reduced size: 100 flips in the upper and 100 in the lower four bits of
    pooled table elements, one per launch, plus clean launches; every flag vector equals the oracle's."""
    wl = w.EbWorkload("campaign", 20000, 64, 10, 100, False, regime)
    x = w.make_inputs(wl, tag=20)
    g = GpuTable(b, x.T, x.scale, x.bias, aligned=(regime == "gauss"))
    C_T = eb.table_rowsums(x.T)
    clean = eb.checked_eb(x.T, x.scale, x.bias, x.indices, x.offsets)
    assert clean.robust.all()
    assert np.array_equal(g.run(x.indices, x.offsets, None, "auto")["flags"], clean.flags)
    rates = {}
    for bits in ("high", "low"):
        rng = w.rng_for(20, 0, 1 + (bits == "low"))
        f_row, f_col, f_bit = w.draw_table_flips(rng, x.indices, 64, 100, bits)
        want = eb.campaign_table_flips(x.T, x.scale, x.bias, C_T, x.indices, x.offsets, None, f_row, f_col, f_bit)
        got = np.empty_like(want)
        for t in range(100):
            b.abft_eb_table_flip_bit(g.Tp, f_row[t], f_col[t], f_bit[t])
            got[t] = g.run(x.indices, x.offsets, None, "auto")["flags"]
            b.abft_eb_table_flip_bit(g.Tp, f_row[t], f_col[t], f_bit[t])
        assert np.array_equal(got, want)
        rates[bits] = float((got != 0).any(axis=1).mean())
    print(f"\n[eb campaign, {regime}] detected: high bits {rates['high']:.0%}, low bits {rates['low']:.0%}, "
          f"false positives {float((clean.flags != 0).mean()):.0%}")
    assert rates["high"] >= rates["low"]
    assert np.array_equal(g.rowsums(), C_T)


@pytest.mark.parametrize("d", [64, 256])
def test_table1_shapes_full_size(b, d):
    """The benchmark's own configurations: 4,000,000 rows, pooling 100, batch 10 (Table I) and
    the large batch of 16384 lookups, weighted and not, in the variant the library picks."""
    x = w.make_inputs(w.TABLE1[d], tag=30 + d)
    g = GpuTable(b, x.T, x.scale, x.bias)
    C_T = eb.table_rowsums(x.T)
    sample = np.concatenate([np.arange(0, 4_000_000, 40_009), x.indices[:200]])
    assert np.array_equal(g.rowsums()[sample], C_T[sample])
    ref = eb.checked_eb(x.T, x.scale, x.bias, x.indices, x.offsets, C_T=C_T)
    compare(g.run(x.indices, x.offsets), ref, x.T, x.scale, x.bias, x.indices, x.offsets, None)
    rng = w.rng_for(30 + d, 1)
    indices, offsets = w.draw_bags(rng, 4_000_000, 16384 if d == 64 else 4096, 100, "spread")
    weights = w.draw_weights(rng, indices.size)
    for wts in (None, weights):
        ref = eb.checked_eb(x.T, x.scale, x.bias, indices, offsets, wts, C_T=C_T)
        compare(g.run(indices, offsets, wts), ref, x.T, x.scale, x.bias, indices, offsets, wts)


@pytest.mark.parametrize("d", [32, 64, 128, 256, 512, 1024])
@pytest.mark.parametrize("variant", ["batch", "group"])
def test_int4_tables_match_oracle(b, d, variant):
    """4-bit codes, two per byte: same bar as the 8-bit tables, plus flips of each of the four bits of
    codes in even and odd columns."""
    for weighted, regime, lengths, aligned in ((False, "uniform", "spread", False), (True, "gauss", "ragged", True)):
        rng = w.rng_for(200 + d, 0, int(weighted))
        T, scale, bias = w.draw_table(rng, 2000, d, regime, bits=4)
        assert T.shape == (2000, d // 2)
        indices, offsets = w.draw_bags(rng, 2000, 100, 40, lengths)
        extra = rng.integers(0, 2000, size=1300, dtype=np.int64)
        indices = np.concatenate([indices, extra])
        offsets = np.concatenate([offsets, [indices.size]]).astype(np.int64)
        weights = w.draw_weights(rng, indices.size) if weighted else None
        g = GpuTable(b, T, scale, bias, aligned, bits=4)
        stride = {16: 32, 32: 64, 64: 128}.get(d // 2, d // 2 + 16) if aligned else d // 2 + 16
        assert b.abft_eb_table_dims(g.Tp) == (2000, d, stride, 4)
        C_T = eb.table_rowsums(T, bits=4)
        assert np.array_equal(g.rowsums(), C_T)
        ref = eb.checked_eb(T, scale, bias, indices, offsets, weights, bits=4)
        compare(g.run(indices, offsets, weights, variant), ref, T, scale, bias, indices, offsets, weights, bits=4,
                csum_in_index_order=variant == "batch")
        for col, bit in ((0, 0), (1, 3), (d - 1, 2), (d // 2, 1)):
            row = int(indices[offsets[-2] + 5])
            b.abft_eb_table_flip_bit(g.Tp, row, col, bit)
            T2 = T.copy()
            T2[row, col // 2] ^= np.uint8(1 << (bit + 4 * (col & 1)))
            ref = eb.checked_eb(T2, scale, bias, indices, offsets, weights, C_T=C_T, bits=4)
            out = g.run(indices, offsets, weights, variant)
            assert same_bits(out["R"], ref.R)
            assert np.array_equal(out["flags"][ref.robust], ref.flags[ref.robust])
            b.abft_eb_table_flip_bit(g.Tp, row, col, bit)
        with pytest.raises(b.AbftError):
            b.abft_eb_table_flip_bit(g.Tp, 0, 0, 4)     # a 4-bit code has bits 0..3


def test_large_batch_takes_the_batch_kernel_by_itself(b):
    """70000 short lookups at d = 32: the library picks the batch kernel (lookups alone fill the chip);
    same bar as everywhere."""
    rng = w.rng_for(40)
    T, scale, bias = w.draw_table(rng, 50000, 32, "uniform")
    indices, offsets = w.draw_bags(rng, 50000, 70000, 6, "spread")
    weights = w.draw_weights(rng, indices.size)
    g = GpuTable(b, T, scale, bias)
    ref = eb.checked_eb(T, scale, bias, indices, offsets, weights)
    out = g.run(indices, offsets, weights, "auto")
    compare(out, ref, T, scale, bias, indices, offsets, weights, csum_in_index_order=True)   # (only the batch kernel does)
    assert same_bits(g.run(indices, offsets, weights, "group")["R"], out["R"])


def test_table_beyond_4_gib(b):
    """Record offsets that do not fit 32 bits: a table of 17,000,000 records of 272 bytes (4.6 GB) built
    on the device; the rows a batch pools are brought back and the oracle runs on that compacted table."""
    rows, d = 17_000_000, 256
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    T = torch.randint(0, 256, (rows, d), dtype=torch.uint8, device="cuda", generator=gen)
    scale = torch.rand(rows, device="cuda", generator=gen) * 0.015 + 0.005
    bias = -0.5 * torch.rand(rows, device="cuda", generator=gen)
    Tp = b.abft_eb_pack_rowsum(T, scale, bias)
    torch.cuda.synchronize()
    assert b.abft_eb_table_dims(Tp)[2] * rows > 2 ** 32
    rng = w.rng_for(41)
    indices, offsets = w.draw_bags(rng, rows, 300, 40, "spread")
    indices[:50] = rows - 1 - np.arange(50)              # the far end of the table
    uniq, inv = np.unique(indices, return_inverse=True)
    sel = torch.from_numpy(uniq).cuda()
    T_small, scale_small, bias_small = T[sel].cpu().numpy(), scale[sel].cpu().numpy(), bias[sel].cpu().numpy()
    del T
    ref = eb.checked_eb(T_small, scale_small, bias_small, inv.astype(np.int64), offsets)
    rowsums = torch.empty(rows, dtype=torch.int32, device="cuda")
    b.abft_eb_table_get_rowsums(Tp, rowsums)
    assert np.array_equal(rowsums[sel].cpu().numpy(), ref.C_T)
    for variant in ("group", "batch"):
        R = torch.empty((300, d), dtype=torch.float32, device="cuda")
        flags = torch.empty(300, dtype=torch.int32, device="cuda")
        b.abft_eb_u8_checked(Tp, dev(indices), dev(offsets), R, flags, flags=VARIANTS[variant])
        torch.cuda.synchronize()
        assert same_bits(R.cpu().numpy(), ref.R) and np.array_equal(flags.cpu().numpy(), ref.flags)
    # a planted fault at the far end is seen
    b.abft_eb_table_flip_bit(Tp, rows - 1, 255, 7)
    b.abft_eb_u8_checked(Tp, dev(indices), dev(offsets), R, flags)
    torch.cuda.synchronize()
    assert flags[0].item() == 1
    Tp.destroy()
