"""Seeded fault-injection campaigns (the protocol of Section VI-B of the paper: one random
bit of one random element, in the 32-bit intermediate, in B after its checksum was taken,
or in A), run on the GPU through the C ABI and compared run by run with the CPU oracle.

Expected by construction of the check (equality mod 2^32):
  C flips: always detected, exactly the row that was hit   (paper, Table II: 2800/2800)
  B flips: row p flagged iff A[p][k] != 0, i.e. detected whenever C is corrupted
  A flips: never flagged (A is not encoded, Section IV-C-3)
"""
import sys

import numpy as np
import pytest

from paper_2103_00130_amd import workloads as wlmod

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def binding():
    import torch
    assert torch.cuda.is_available()
    from paper_2103_00130_amd import binding as b
    return b


class Rig:
    def __init__(self, b, cfg):
        import torch
        self.torch, self.b = torch, b
        self.ops = wlmod.make_operands(cfg)
        wl = self.wl = self.ops.wl
        self.A = torch.from_numpy(self.ops.A).cuda()
        self.Bp = b.abft_pack_b_checksum(torch.from_numpy(self.ops.B).cuda())
        self.C = torch.empty((wl.M, wl.N), dtype=torch.int32, device="cuda")
        self.ws = b.Workspace(wl.M, self.Bp)

    def run(self, flags_row, cnt_slot, inj=None):
        self.b.abft_gemm_u8s8s32_checked(self.A, self.Bp, self.C, flags_row, cnt_slot, inj=inj,
                                         n_inj=0 if inj is None else inj.numel() // 3, workspace=self.ws.tensor)


def c_flip_campaign(b, oracle, cfg, n, ref, batch_after=None, batch=64):
    """n single-bit flips in C accumulators.  The first `batch_after` (all, if None) run one
    per launch; the rest are grouped `batch` per launch with distinct rows."""
    import torch
    rig = Rig(b, cfg)
    wl = rig.wl
    r, c, bit = wlmod.draw_flips(cfg, "C", n)
    want_flag, want_val = oracle.campaign_c_flips(ref.C, ref.chk, r, c, bit)
    assert want_flag.all(), "oracle: a single bit flip in C always moves the row sum"
    n_single = n if batch_after is None else min(n, batch_after)
    inj_all = torch.from_numpy(np.stack([r, c, (np.uint32(1) << bit.astype(np.uint32)).view(np.int32)], axis=1)
                               .astype(np.int32)).cuda().contiguous()
    flags = torch.empty((n_single, wl.M), dtype=torch.int32, device="cuda")
    cnt = torch.empty(n_single, dtype=torch.int32, device="cuda")
    vals = torch.empty(n_single, dtype=torch.int32, device="cuda")
    for t in range(n_single):
        rig.run(flags[t], cnt[t:t + 1], inj=inj_all[t])
        vals[t:t + 1].copy_(rig.C[int(r[t]), int(c[t]):int(c[t]) + 1])
    torch.cuda.synchronize()
    expect = torch.zeros((n_single, wl.M), dtype=torch.int32, device="cuda")
    expect[torch.arange(n_single, device="cuda"), torch.from_numpy(r[:n_single]).cuda().long()] = \
        torch.from_numpy(want_flag[:n_single]).cuda()
    assert torch.equal(flags, expect), "flag vectors differ from the oracle's verdicts"
    assert np.array_equal(cnt.cpu().numpy(), want_flag[:n_single])
    assert np.array_equal(vals.cpu().numpy(), want_val[:n_single]), "returned C does not carry the flipped value"
    detected = int(cnt.sum().item())
    # batched remainder: distinct rows per launch, so every verdict is still attributable
    t = n_single
    launches = 0
    while t < n:
        rows_seen, group = set(), []
        while t < n and len(group) < batch and int(r[t]) not in rows_seen:
            rows_seen.add(int(r[t]))
            group.append(t)
            t += 1
        g = torch.tensor(group, device="cuda")
        fl = torch.empty(wl.M, dtype=torch.int32, device="cuda")
        ct = torch.empty(1, dtype=torch.int32, device="cuda")
        rig.run(fl, ct, inj=inj_all[g].contiguous())
        exp = torch.zeros(wl.M, dtype=torch.int32, device="cuda")
        exp[torch.from_numpy(r[group]).cuda().long()] = 1
        assert torch.equal(fl, exp) and int(ct.item()) == len(group)
        got = rig.C[torch.from_numpy(r[group]).cuda().long(), torch.from_numpy(c[group]).cuda().long()]
        assert np.array_equal(got.cpu().numpy(), want_val[group])
        detected += len(group)
        launches += 1
    # the workspace is clean and a fault-free run after the campaign raises nothing
    fl = torch.empty(wl.M, dtype=torch.int32, device="cuda")
    ct = torch.empty(1, dtype=torch.int32, device="cuda")
    rig.run(fl, ct)
    assert int(ct.item()) == 0 and not fl.any().item()
    assert np.array_equal(rig.C.cpu().numpy(), ref.C)
    say(f"  workload {cfg}: C flips detected {detected}/{n} = {100.0 * detected / n:.2f} %  "
        f"({n_single} single-fault launches, {launches} batched launches), false positives 0")
    return detected


def test_campaign_workload0_c_flips(binding, oracle):
    say("campaign: workload 0, 1000 C flips")
    ops = wlmod.make_operands(0)
    ref = oracle.checked_gemm(ops.A, ops.B)
    assert c_flip_campaign(binding, oracle, 0, 1000, ref) == 1000


def test_campaign_workload4_c_flips(binding, oracle):
    say("campaign: workload 4, 100000 C flips (2000 one per launch, the rest batched by 64 distinct rows)")
    ops = wlmod.make_operands(4)
    ref = oracle.checked_gemm(ops.A, ops.B)
    assert c_flip_campaign(binding, oracle, 4, 100000, ref, batch_after=2000) == 100000


def test_campaign_workload2_a_b_c_flips(binding, oracle):
    import torch
    b = binding
    cfg = 2
    ops = wlmod.make_operands(cfg)
    wl = ops.wl
    ref = oracle.checked_gemm(ops.A, ops.B)
    say("campaign: workload 2, 10000 C flips")
    assert c_flip_campaign(b, oracle, cfg, 10000, ref) == 10000

    rig = Rig(b, cfg)
    # ---- B flips, after the checksum was taken -------------------------------------------
    say("campaign: workload 2, 10000 B flips")
    n = wl.n_flips["B"]
    k, j, bit = wlmod.draw_flips(cfg, "B", n)
    want_flags, want_col = oracle.campaign_b_flips(ops.A, ops.B, ref.C, ref.chk, k, j, bit)
    assert np.array_equal(want_flags, (ops.A[:, k].T != 0).astype(np.int32)), "closed form: row p flags iff A[p][k] != 0"
    flags = torch.empty((n, wl.M), dtype=torch.int32, device="cuda")
    cnt = torch.empty(n, dtype=torch.int32, device="cuda")
    cols = torch.empty((n, wl.M), dtype=torch.int32, device="cuda")
    for t in range(n):
        b.abft_packed_b_flip_bit(rig.Bp, int(k[t]), int(j[t]), int(bit[t]))
        rig.run(flags[t], cnt[t:t + 1])
        b.abft_packed_b_flip_bit(rig.Bp, int(k[t]), int(j[t]), int(bit[t]))
        cols[t].copy_(rig.C[:, int(j[t])])
    torch.cuda.synchronize()
    assert np.array_equal(flags.cpu().numpy(), want_flags)
    assert np.array_equal(cnt.cpu().numpy(), want_flags.sum(axis=1))
    assert np.array_equal(cols.cpu().numpy(), want_col), "corrupted column of C differs from the oracle"
    corrupted = (want_col != ref.C[:, j].T).any(axis=1)
    detected = want_flags.any(axis=1)
    assert np.array_equal(corrupted, detected), "a B flip is flagged exactly when it corrupts C"
    say(f"  B flips: C corrupted in {int(corrupted.sum())}/{n} runs, detected {int(detected.sum())} "
        f"= {100.0 * detected.sum() / max(1, corrupted.sum()):.2f} % of corrupting flips")

    # ---- A flips ---------------------------------------------------------------------------
    say("campaign: workload 2, 10000 A flips")
    n = wl.n_flips["A"]
    i, k, bit = wlmod.draw_flips(cfg, "A", n)
    want = oracle.campaign_a_flips(ops.A, ops.B, ref.S_B, i, k, bit)
    assert not want.any(), "oracle: A is not covered"
    cnt = torch.empty(n, dtype=torch.int32, device="cuda")
    fl = torch.empty(wl.M, dtype=torch.int32, device="cuda")
    n_rows_checked = 200
    _, want_rows = oracle.campaign_a_flips(ops.A, ops.B, ref.S_B, i[:n_rows_checked], k[:n_rows_checked],
                                           bit[:n_rows_checked], want_rows=True)
    got_rows = torch.empty((n_rows_checked, wl.N), dtype=torch.int32, device="cuda")
    for t in range(n):
        rig.A[int(i[t]), int(k[t])] ^= (1 << int(bit[t]))
        rig.run(fl, cnt[t:t + 1])
        rig.A[int(i[t]), int(k[t])] ^= (1 << int(bit[t]))
        if t < n_rows_checked:
            got_rows[t].copy_(rig.C[int(i[t])])
    torch.cuda.synchronize()
    assert int(cnt.sum().item()) == 0
    assert np.array_equal(got_rows.cpu().numpy(), want_rows)
    assert np.array_equal(rig.A.cpu().numpy(), ops.A)
    say(f"  A flips: detected 0/{n} (silent by design: only B is encoded)")


def test_value_replacement_and_multibit_faults(binding, oracle):
    """The second fault model of Section IV-C (an element takes an arbitrary wrong value) and
    multi-bit upsets, workload 2.  At modulus 2^32: a changed C element is always detected; a
    changed B element is flagged in exactly the rows it corrupts."""
    import torch
    b = binding
    cfg = 2
    ops = wlmod.make_operands(cfg)
    wl = ops.wl
    ref = oracle.checked_gemm(ops.A, ops.B)
    rig = Rig(b, cfg)
    fl = torch.empty(wl.M, dtype=torch.int32, device="cuda")
    ct = torch.empty(1, dtype=torch.int32, device="cuda")

    def c_campaign(name, r, c, masks):
        n = len(r)
        want_flag, want_val = oracle.campaign_c_masks(ref.C, ref.chk, r, c, masks)
        assert np.array_equal(want_flag, (masks != 0).astype(np.int32))
        flags = torch.empty((n, wl.M), dtype=torch.int32, device="cuda")
        cnt = torch.empty(n, dtype=torch.int32, device="cuda")
        vals = torch.empty(n, dtype=torch.int32, device="cuda")
        inj = torch.from_numpy(np.stack([r, c, masks.view(np.int32)], axis=1).astype(np.int32)).cuda().contiguous()
        for t in range(n):
            rig.run(flags[t], cnt[t:t + 1], inj=inj[t])
            vals[t:t + 1].copy_(rig.C[int(r[t]), int(c[t]):int(c[t]) + 1])
        torch.cuda.synchronize()
        expect = np.zeros((n, wl.M), np.int32)
        expect[np.arange(n), r] = want_flag
        assert np.array_equal(flags.cpu().numpy(), expect)
        assert np.array_equal(cnt.cpu().numpy(), want_flag)
        assert np.array_equal(vals.cpu().numpy(), want_val)
        say(f"  {name}: detected {int(want_flag.sum())}/{int((masks != 0).sum())} changed elements")

    def b_campaign(name, k, j, new):
        n = len(k)
        want_flags, want_col = oracle.campaign_b_values(ops.A, ops.B, ref.C, ref.chk, k, j, new)
        flags = torch.empty((n, wl.M), dtype=torch.int32, device="cuda")
        cols = torch.empty((n, wl.M), dtype=torch.int32, device="cuda")
        for t in range(n):
            diff = (int(ops.B[k[t], j[t]]) & 0xFF) ^ (int(new[t]) & 0xFF)
            bits = [bit for bit in range(8) if diff >> bit & 1]
            for bit in bits:
                b.abft_packed_b_flip_bit(rig.Bp, int(k[t]), int(j[t]), bit)
            rig.run(flags[t], ct)
            for bit in bits:
                b.abft_packed_b_flip_bit(rig.Bp, int(k[t]), int(j[t]), bit)
            cols[t].copy_(rig.C[:, int(j[t])])
        torch.cuda.synchronize()
        assert np.array_equal(flags.cpu().numpy(), want_flags)
        assert np.array_equal(cols.cpu().numpy(), want_col)
        corrupted = (want_col != ref.C[:, j].T).any(axis=1)
        detected = want_flags.any(axis=1)
        assert np.array_equal(corrupted, detected)
        say(f"  {name}: C corrupted in {int(corrupted.sum())}/{n} runs, detected {int(detected.sum())}")

    n = 2000
    say("campaign: workload 2, value replacement in C")
    r, c, new = wlmod.draw_value_faults(cfg, "C", n)
    c_campaign("C value replacement", r, c, (ref.C[r, c].view(np.uint32) ^ new.view(np.uint32)).astype(np.uint32))
    for nb in (2, 3):
        say(f"campaign: workload 2, {nb}-bit upsets in C")
        r, c, masks = wlmod.draw_multibit_masks(cfg, "C", n, nb)
        c_campaign(f"C {nb}-bit upsets", r, c, masks)
    say("campaign: workload 2, value replacement in B")
    k, j, new = wlmod.draw_value_faults(cfg, "B", n)
    b_campaign("B value replacement", k, j, new)
    say("campaign: workload 2, 2-bit upsets in B")
    k, j, masks = wlmod.draw_multibit_masks(cfg, "B", n, 2)
    new = ((ops.B[k, j].astype(np.int32) & 0xFF) ^ masks.astype(np.int32)).astype(np.uint8).view(np.int8).astype(np.int32)
    b_campaign("B 2-bit upsets", k, j, new)
    rig.run(fl, ct)
    torch.cuda.synchronize()
    assert int(ct.item()) == 0 and not fl.any().item() and np.array_equal(rig.C.cpu().numpy(), ref.C)


def test_campaign_mod127_b_flips(binding, oracle):
    """Algorithm 1 as printed (ABFT_MOD127), workload 2, 10000 bit flips in B after the checksum
    was taken (the protocol behind Table II): run by run the flags of the oracle, and the miss
    rate per corrupted row that Section IV-C-1 predicts (operand values 127 and 254 out of the 255
    that corrupt)."""
    import torch
    b = binding
    cfg = 2
    ops = wlmod.make_operands(cfg)
    wl = ops.wl
    clean = oracle.gemm_u8s8s32(ops.A, ops.B)
    chk127 = oracle.row_checksum_mod127(ops.A, ops.B)
    n = wl.n_flips["B"]
    k, j, bit = wlmod.draw_flips(cfg, "B", n)
    say(f"campaign: workload 2, {n} B flips, modulus 127")
    want_flags, want_col = oracle.campaign_b_flips_mod127(ops.A, ops.B, clean, chk127, k, j, bit)
    rig = Rig(b, cfg)
    flags = torch.empty((n, wl.M), dtype=torch.int32, device="cuda")
    cnt = torch.empty(n, dtype=torch.int32, device="cuda")
    cols = torch.empty((n, wl.M), dtype=torch.int32, device="cuda")
    for t in range(n):
        b.abft_packed_b_flip_bit(rig.Bp, int(k[t]), int(j[t]), int(bit[t]))
        b.abft_gemm_u8s8s32_checked(rig.A, rig.Bp, rig.C, flags[t], cnt[t:t + 1], flags=b.ABFT_MOD127,
                                    workspace=rig.ws.tensor)
        b.abft_packed_b_flip_bit(rig.Bp, int(k[t]), int(j[t]), int(bit[t]))
        cols[t].copy_(rig.C[:, int(j[t])])
    torch.cuda.synchronize()
    assert np.array_equal(flags.cpu().numpy(), want_flags)
    assert np.array_equal(cnt.cpu().numpy(), want_flags.sum(axis=1))
    assert np.array_equal(cols.cpu().numpy(), want_col)
    corrupted_rows = want_col != clean[:, j].T
    missed_rows = corrupted_rows & (want_flags == 0)
    runs_corrupted = corrupted_rows.any(axis=1)
    runs_detected = want_flags.any(axis=1)
    assert not (runs_detected & ~runs_corrupted).any()
    rate = missed_rows.sum() / corrupted_rows.sum()
    say(f"  modulus 127: C corrupted in {int(runs_corrupted.sum())}/{n} runs, detected {int(runs_detected.sum())} "
        f"({100.0 * runs_detected.sum() / runs_corrupted.sum():.2f} %); corrupted rows missed "
        f"{int(missed_rows.sum())}/{int(corrupted_rows.sum())} = {100 * rate:.3f} % (predicted 2/255 = 0.784 %)")
    assert abs(rate - 2 / 255) < 0.002
