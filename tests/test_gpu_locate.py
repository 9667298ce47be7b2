"""GPU parity of abft_locate_correct (Section IV: the column check of Eq. 2a and the repair of one located
element) against the CPU oracle's locate_correct, through the C ABI.  Everything is integer: C after the call,
the column verdicts, the report and the row verdicts must match bit for bit."""
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
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2103_00130_amd import binding as b
    return b


@pytest.fixture(scope="module")
def gpu_util():
    import gpu_util
    return gpu_util


def operands(M, N, K, seed, relu_like=False):
    rng = np.random.Generator(np.random.PCG64(seed))
    return wlmod.draw_a(rng, M, K, relu_like), rng.integers(-128, 128, size=(K, N), dtype=np.int8)


class Rig:
    """Checked GEMM followed by abft_locate_correct on the same device buffers."""

    def __init__(self, b, gpu_util, A, B, requant=None, a_dev=None):
        import torch
        self.b, self.torch = b, torch
        self.run = gpu_util.GpuRun(b, B)
        self.A = gpu_util.dev(A) if a_dev is None else a_dev
        M, N = A.shape[0], B.shape[1]
        self.C = torch.empty((M, N), dtype=torch.int32, device="cuda")
        self.flags = torch.empty(M, dtype=torch.int32, device="cuda")
        self.cnt = torch.empty(1, dtype=torch.int32, device="cuda")
        self.colf = torch.full((N,), -1, dtype=torch.int32, device="cuda")
        self.ws = b.Workspace(M, self.run.Bp)
        self.rq = self.Cq = None
        self.keep = []
        if requant is not None:
            zA, zC, mult = requant
            m = gpu_util.dev(np.atleast_1d(mult).astype(np.float32))
            self.keep.append(m)
            self.rq = b.make_requant(zA, zC, m)
            self.Cq = torch.empty((M, N), dtype=torch.uint8, device="cuda")

    def gemm(self, injections=()):
        b = self.b
        inj = b.make_injections(list(injections)) if len(injections) else None
        b.abft_gemm_u8s8s32_checked(self.A, self.run.Bp, self.C, self.flags, self.cnt, rq=self.rq, Cq=self.Cq, inj=inj,
                                    n_inj=len(injections), workspace=self.ws.tensor)

    def locate(self):
        rep = self.b.abft_locate_correct(self.A, self.run.Bp, self.C, self.flags, self.cnt, rq=self.rq, Cq=self.Cq,
                                         col_flags=self.colf)
        self.torch.cuda.synchronize()
        return rep.cpu().numpy()

    def check(self, want, want_flags_after, want_count_after):
        rep = self.locate()
        assert (int(rep[0]), int(rep[1]), int(rep[2])) == (want.status, want.row, want.col)
        assert (int(rep[5]), int(rep[6])) == (want.rows_violated, want.cols_violated)
        if want.status == 1:
            assert (int(rep[3]), int(rep[4])) == (want.old_value, want.new_value)
        assert np.array_equal(self.C.cpu().numpy(), want.C), "C after the call differs from the oracle's"
        assert np.array_equal(self.colf.cpu().numpy(), want.col_flags)
        assert np.array_equal(self.flags.cpu().numpy(), want_flags_after)
        assert int(self.cnt.item()) == want_count_after


@pytest.mark.parametrize("M,N,K", [(150, 290, 144), (16, 4096, 2048), (300, 520, 200), (1, 1, 1), (70, 300, 130), (513, 257, 65)])
def test_single_fault_is_located_and_repaired(binding, gpu_util, oracle, M, N, K):
    say(f"locate/correct {M}x{N}x{K}")
    A, B = operands(M, N, K, 7 * M + N + K, relu_like=(M % 2 == 0))
    rig = Rig(binding, gpu_util, A, B)
    clean = oracle.checked_gemm(A, B)
    rig.gemm()
    rig.check(oracle.locate_correct(A, B, clean.C, clean.flags), clean.flags, 0)      # nothing to do
    rng = np.random.default_rng(M + N)
    for bit in [0, 1, 7, 8, 15, 16, 24, 30, 31]:
        r, c = int(rng.integers(M)), int(rng.integers(N))
        bad = oracle.checked_gemm(A, B, flips_c=[(r, c, 1 << bit)])
        rig.gemm([(r, c, 1 << bit)])
        assert int(rig.cnt.item()) == 1
        want = oracle.locate_correct(A, B, bad.C, bad.flags)
        assert want.status == 1 and np.array_equal(want.C, clean.C)
        rig.check(want, np.zeros(M, np.int32), 0)
    # the corner elements and an arbitrary replacement value
    for (r, c, mask) in [(0, 0, 0xFFFFFFFF), (M - 1, N - 1, 0x80000001)]:
        bad = oracle.checked_gemm(A, B, flips_c=[(r, c, mask)])
        rig.gemm([(r, c, mask)])
        rig.check(oracle.locate_correct(A, B, bad.C, bad.flags), np.zeros(M, np.int32), 0)


def test_requantized_output_is_repaired_too(binding, gpu_util, oracle):
    M, N, K = 140, 270, 608
    A, B = operands(M, N, K, 99)
    mult = wlmod.draw_mult(np.random.default_rng(3), N, "channel")
    rig = Rig(binding, gpu_util, A, B, requant=(128, 128, mult))
    clean = oracle.checked_gemm(A, B)
    q_clean = oracle.requantize(clean.C, clean.colsum, 128, 128, mult, precision="f32")
    inj = [(77, 200, 1 << 30)]
    bad = oracle.checked_gemm(A, B, flips_c=inj)
    rig.gemm(inj)
    q_bad = rig.Cq.cpu().numpy()
    assert q_bad[77, 200] != q_clean[77, 200] or True      # (the clamp may hide the fault in the 8-bit value)
    rig.check(oracle.locate_correct(A, B, bad.C, bad.flags), np.zeros(M, np.int32), 0)
    assert np.array_equal(rig.Cq.cpu().numpy(), q_clean)


def test_patterns_that_are_not_one_element(binding, gpu_util, oracle):
    M, N, K = 200, 300, 272
    say("locate/correct: patterns that are not one element")
    A, B = operands(M, N, K, 5)
    A[A == 0] = 1
    rig = Rig(binding, gpu_util, A, B)
    clean = oracle.checked_gemm(A, B)
    for flips in ([(1, 2, 1 << 5), (70, 9, 1 << 20)], [(4, 2, 1), (4, 299, 1 << 31)], [(4, 3, 1 << 8), (199, 3, 1 << 9)]):
        bad = oracle.checked_gemm(A, B, flips_c=flips)
        rig.gemm(flips)
        want = oracle.locate_correct(A, B, bad.C, bad.flags)
        assert want.status == 2
        rig.check(want, bad.flags, bad.err_count)
    # a fault in B after it was encoded: rows flagged, no column violated, nothing rewritten
    k, j, bit = 100, 8, 6
    bad = oracle.checked_gemm(A, B, flips_b=[(k, j, bit)])
    B_bad = B.copy()
    B_bad.view(np.uint8)[k, j] ^= np.uint8(1 << bit)
    binding.abft_packed_b_flip_bit(rig.run.Bp, k, j, bit)
    rig.gemm()
    want = oracle.locate_correct(A, B_bad, bad.C, bad.flags, S_B=clean.S_B)
    assert want.status == 2 and want.cols_violated == 0 and want.rows_violated == M
    rig.check(want, bad.flags, bad.err_count)
    binding.abft_packed_b_flip_bit(rig.run.Bp, k, j, bit)
    # a stored C_temp that was hit after the launch, with verdicts that name another row: the two formulas disagree
    rig.gemm([(7, 5, 1 << 12)])
    rig.C[7, 5] ^= (1 << 12)            # back to the clean value ...
    rig.C[30, 5] += 1000                # ... and another element of the same column is changed in memory
    C_now = rig.C.cpu().numpy()
    flags = np.zeros(M, np.int32)
    flags[7] = 1
    want = oracle.locate_correct(A, B, C_now, flags)
    assert want.status == 2 and (want.rows_violated, want.cols_violated) == (1, 1)
    rig.check(want, flags, 1)


def test_unaligned_a_and_long_tall_shapes(binding, gpu_util, oracle):
    import torch
    M, N, K = 90, 130, 77               # K not a multiple of 16, A at an odd address with an odd pitch
    A, B = operands(M, N, K, 31)
    buf = torch.zeros(M * 83 + 1, dtype=torch.uint8, device="cuda")
    a_dev = buf[1:].view(M, 83)[:, :K]
    a_dev.copy_(torch.from_numpy(A))
    rig = Rig(binding, gpu_util, A, B, a_dev=a_dev)
    clean = oracle.checked_gemm(A, B)
    bad = oracle.checked_gemm(A, B, flips_c=[(89, 129, 1 << 17)])
    rig.gemm([(89, 129, 1 << 17)])
    want = oracle.locate_correct(A, B, bad.C, bad.flags)
    assert want.status == 1 and np.array_equal(want.C, clean.C)
    rig.check(want, np.zeros(M, np.int32), 0)
    M, N, K = 70000, 64, 64
    A, B = operands(M, N, K, 32)
    rig = Rig(binding, gpu_util, A, B)
    bad = oracle.checked_gemm(A, B, flips_c=[(69999, 0, 1 << 3)])
    rig.gemm([(69999, 0, 1 << 3)])
    rig.check(oracle.locate_correct(A, B, bad.C, bad.flags), np.zeros(M, np.int32), 0)


def test_dense_workload_full_size(binding, gpu_util, oracle):
    ops = wlmod.make_operands(4)
    wl = ops.wl
    say(f"locate/correct on {wl.name}")
    rig = Rig(binding, gpu_util, ops.A, ops.B)
    clean = oracle.checked_gemm(ops.A, ops.B)
    inj = [(3000, 123, 1 << 21)]
    rig.gemm(inj)
    C_bad = clean.C.copy()
    C_bad.view(np.uint32)[3000, 123] ^= np.uint32(1 << 21)
    flags = np.zeros(wl.M, np.int32)
    flags[3000] = 1
    want = oracle.locate_correct(ops.A, ops.B, C_bad, flags)
    assert want.status == 1 and np.array_equal(want.C, clean.C)
    rig.check(want, np.zeros(wl.M, np.int32), 0)


def test_bad_arguments(binding, gpu_util):
    import torch
    A, B = operands(16, 32, 64, 1)
    rig = Rig(binding, gpu_util, A, B)
    rig.gemm()
    small = torch.empty(8, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.AbftError):
        binding.abft_locate_correct(rig.A, rig.run.Bp, rig.C, rig.flags, scratch=small)
    assert binding.abft_locate_scratch_bytes(rig.run.Bp) == (128 + 2 * 256) * 4
