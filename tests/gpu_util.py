"""Helpers for the GPU parity tests: upload seeded operands, call the C ABI through the
binding, bring results back as numpy.  No arithmetic of the method happens here."""
from __future__ import annotations

import numpy as np
import torch

VARIANTS = {"auto": 0, "tile256": 0x100, "tile128": 0x200, "tile64": 0x300, "smallm": 0x400,
            "tile256w2x4": 0x500, "tile256w4x2": 0x600}


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


class GpuRun:
    """One packed weight plus reusable output buffers."""

    def __init__(self, binding, B: np.ndarray, transposed: bool = False):
        self.b = binding
        self.B_dev = dev(B.T if transposed else B)
        self.Bp = binding.abft_pack_b_checksum(self.B_dev, b_is_transposed=transposed)
        self.K, self.N = self.Bp.K, self.Bp.N

    def _zero_ints(self, M, numel):
        base = 64 + max(2 * ((M + 63) // 64 * 64), 2 * (32 * 64 + 64))
        if numel <= base:
            return numel
        tiles = ((M + 63) // 64) * ((self.N + 63) // 64)
        return base + (tiles + 63) // 64 * 64

    def checksum(self) -> np.ndarray:
        out = torch.empty(self.K, dtype=torch.int32, device="cuda")
        self.b.abft_packed_b_get_checksum(self.Bp, out)
        return out.cpu().numpy()

    def colsum(self) -> np.ndarray:
        out = torch.empty(self.N, dtype=torch.int32, device="cuda")
        self.b.abft_packed_b_get_col_offsets(self.Bp, out)
        return out.cpu().numpy()

    def gemm(self, A, variant="auto", check=True, injections=(), requant=None, want_c=True, ws=None, mod127=False,
             accumulate_from=None, want_count=True):
        """A: numpy uint8 [M,K] or a device tensor.  requant = (zA, zC, mult_np, bias_np|None).
        Returns dict with C, flags, err_count, Cq (numpy; None where not produced)."""
        b = self.b
        A_dev = dev(A) if isinstance(A, np.ndarray) else A
        M = A_dev.shape[0]
        C = torch.full((M, self.N), -7, dtype=torch.int32, device="cuda") if want_c else None
        flags = torch.full((M,), -1, dtype=torch.int32, device="cuda")
        # accumulate_from = n: errCount is a counter that starts at n and is added to (ABFT_ERRCOUNT_ACCUMULATE)
        cnt = torch.full((1,), -1 if accumulate_from is None else accumulate_from, dtype=torch.int32, device="cuda")
        if ws is None:
            ws = b.Workspace(M, self.Bp)
        rq = Cq = None
        keep = []
        if requant is not None:
            zA, zC, mult, bias = requant
            mult_d = dev(np.atleast_1d(mult).astype(np.float32))
            bias_d = None if bias is None else dev(bias.astype(np.int32))
            keep += [mult_d, bias_d]
            rq = b.make_requant(zA, zC, mult_d, bias_d)
            Cq = torch.full((M, self.N), 7, dtype=torch.uint8, device="cuda")
        inj = b.make_injections(list(injections)) if len(injections) else None
        fl = VARIANTS[variant] | (b.ABFT_CHECK if check else b.ABFT_NOCHECK) | (b.ABFT_MOD127 if mod127 else 0)
        if accumulate_from is not None:
            fl |= b.ABFT_ERRCOUNT_ACCUMULATE
        b.abft_gemm_u8s8s32_checked(A_dev, self.Bp, C, flags, cnt if want_count else None, rq=rq, Cq=Cq, inj=inj, n_inj=len(injections),
                                    flags=fl, workspace=ws.tensor)
        torch.cuda.synchronize()
        return {
            "C": None if C is None else C.cpu().numpy(),
            "flags": flags.cpu().numpy(),
            "err_count": int(cnt.item()),
            "Cq": None if Cq is None else Cq.cpu().numpy(),
            # the words every call must leave at zero: row and counting words, and (when the workspace also has room for
            # the partial tiles of a K split across workgroups, whose contents are irrelevant) the tile tickets behind them
            "ws": ws.tensor.cpu().numpy()[: self._zero_ints(M, ws.tensor.numel())],
        }
