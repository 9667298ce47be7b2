"""ctypes binding of libabftgemm.so: same names as include/abft_gemm.h and include/abft_eb.h.

Argument marshalling only.  torch tensors supply device memory and the current
stream; every step of the method runs in the HIP kernels behind the C ABI.
Importing this module fails loudly when the library has not been built
(`python -m paper_2103_00130_amd.build`): there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# ABFT_LIBRARY: path of another build of the same library (the diagnostic build with in-kernel clock traces)
LIB_PATH = os.environ.get("ABFT_LIBRARY") or os.path.join(_HERE, "libabftgemm.so")

ABFT_OK, ABFT_EINVAL, ABFT_EUNSUPPORTED, ABFT_EHIP = 0, -1, -2, -3
ABFT_CHECK, ABFT_NOCHECK, ABFT_MOD127, ABFT_ERRCOUNT_ACCUMULATE = 0, 1, 2, 4
ABFT_VARIANT_TILE256, ABFT_VARIANT_TILE128, ABFT_VARIANT_TILE64, ABFT_VARIANT_SMALLM = 0x100, 0x200, 0x300, 0x400

EXPORTS = (
    "abft_pack_b_checksum", "abft_packed_b_dims", "abft_packed_b_get_checksum", "abft_packed_b_get_checksum_mod127",
    "abft_packed_b_get_col_offsets",
    "abft_packed_b_flip_bit", "abft_packed_b_flip_checksum_bit", "abft_packed_b_flip_checksum_bit_mod127",
    "abft_packed_b_destroy",
    "abft_gemm_workspace_bytes", "abft_workspace_init", "abft_gemm_u8s8s32_checked", "abft_gemm_u8s8s32_checked_static",
    "abft_requantize_u8",
    "abft_verify_rows", "abft_row_checksum", "abft_recover_scratch_bytes", "abft_recompute_flagged_rows",
    "abft_recompute_flagged_rows_async",
    "abft_locate_scratch_bytes", "abft_locate_correct", "abft_calib_copy", "abft_clock_probe", "abft_mfma_peak_probe", "abft_clock_trace", "abft_last_error",
)
ABFT_LOCATE_CLEAN, ABFT_LOCATE_CORRECTED, ABFT_LOCATE_NOT_ONE_ELEMENT = 0, 1, 2
EXPORTS_EB = (
    "abft_eb_pack_rowsum", "abft_eb_table_dims", "abft_eb_table_get_rowsums", "abft_eb_table_flip_bit",
    "abft_eb_table_destroy", "abft_eb_u8_checked",
)
ABFT_EB_CHECK, ABFT_EB_NOCHECK = 0, 1
ABFT_EB_VARIANT_BATCH, ABFT_EB_VARIANT_GROUP = 0x100, 0x200
ABFT_EB_ERR, ABFT_EB_BAD_INDEX = 1, 2
ABFT_EB_PACK_COMPACT, ABFT_EB_PACK_LINE_ALIGNED, ABFT_EB_PACK_INT4 = 0, 1, 2


class abft_requant_t(ctypes.Structure):
    _fields_ = [("zA", ctypes.c_int32), ("zC", ctypes.c_int32), ("mult", ctypes.c_void_p),
                ("per_channel", ctypes.c_int32), ("bias", ctypes.c_void_p)]


class abft_inject_t(ctypes.Structure):
    _fields_ = [("row", ctypes.c_int32), ("col", ctypes.c_int32), ("xor_mask", ctypes.c_uint32)]


class AbftError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libabftgemm error {code}: {msg}")
        self.code = code


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2103_00130_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, u32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint32, ctypes.c_size_t
    L.abft_last_error.restype = ctypes.c_char_p
    L.abft_pack_b_checksum.argtypes = [vp, i64, i32, i32, i32, vp, ctypes.POINTER(vp)]
    L.abft_packed_b_dims.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    L.abft_packed_b_get_checksum.argtypes = [vp, vp, vp]
    L.abft_packed_b_get_checksum_mod127.argtypes = [vp, vp, vp]
    L.abft_packed_b_get_col_offsets.argtypes = [vp, vp, vp]
    L.abft_packed_b_flip_bit.argtypes = [vp, i32, i32, i32, vp]
    L.abft_packed_b_flip_checksum_bit.argtypes = [vp, i32, i32, vp]
    L.abft_packed_b_flip_checksum_bit_mod127.argtypes = [vp, i32, i32, vp]
    L.abft_packed_b_destroy.argtypes = [vp]
    L.abft_packed_b_destroy.restype = None
    L.abft_gemm_workspace_bytes.argtypes = [i32, vp]
    L.abft_gemm_workspace_bytes.restype = sz
    L.abft_workspace_init.argtypes = [vp, sz, vp]
    L.abft_gemm_u8s8s32_checked.argtypes = [vp, i64, i32, vp, vp, i64, vp, vp, ctypes.POINTER(abft_requant_t), vp, i64,
                                            vp, i32, u32, vp, sz, vp]
    L.abft_gemm_u8s8s32_checked_static.argtypes = [vp, i64, i32, vp, vp, i64, vp, vp, ctypes.POINTER(abft_requant_t), vp, i64,
                                                   vp, i32, u32, vp]
    L.abft_requantize_u8.argtypes = [vp, i64, i32, i32, vp, ctypes.POINTER(abft_requant_t), vp, i64, vp]
    L.abft_verify_rows.argtypes = [vp, i64, i32, i32, vp, vp, vp, vp]
    L.abft_row_checksum.argtypes = [vp, i64, i32, vp, vp, vp]
    L.abft_calib_copy.argtypes = [vp, vp, sz, vp]
    L.abft_clock_probe.argtypes = [vp, i32, vp]
    L.abft_mfma_peak_probe.argtypes = [vp, i32, vp]
    L.abft_clock_trace.argtypes = [vp]
    L.abft_recover_scratch_bytes.argtypes = [i32, i32, vp]
    L.abft_recover_scratch_bytes.restype = sz
    L.abft_recompute_flagged_rows.argtypes = [vp, i64, i32, vp, vp, i64, vp, vp, ctypes.POINTER(abft_requant_t), vp, i64,
                                              i32, vp, sz, vp, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    L.abft_recompute_flagged_rows_async.argtypes = [vp, i64, i32, vp, vp, i64, vp, vp, ctypes.POINTER(abft_requant_t), vp, i64,
                                                    i32, vp, sz, vp, vp]
    L.abft_locate_scratch_bytes.argtypes = [vp]
    L.abft_locate_scratch_bytes.restype = sz
    L.abft_locate_correct.argtypes = [vp, i64, i32, vp, vp, i64, vp, vp, ctypes.POINTER(abft_requant_t), vp, i64, vp, vp, vp, sz, vp]
    L.abft_eb_pack_rowsum.argtypes = [vp, i64, vp, vp, i64, i32, u32, vp, ctypes.POINTER(vp)]
    L.abft_eb_table_dims.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i32)]
    L.abft_eb_table_get_rowsums.argtypes = [vp, vp, vp]
    L.abft_eb_table_flip_bit.argtypes = [vp, i64, i32, i32, vp]
    L.abft_eb_table_destroy.argtypes = [vp]
    L.abft_eb_table_destroy.restype = None
    L.abft_eb_u8_checked.argtypes = [vp, vp, i64, vp, i64, vp, vp, i64, vp, vp, vp, ctypes.c_double, u32, vp]
    return L


lib = _load()


def _check(rc: int):
    if rc != ABFT_OK:
        raise AbftError(rc, lib.abft_last_error().decode())


def _stream(stream=None) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _ptr(t, dtype, name):
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _ld(t, name):
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{name} must be 2-D with unit column stride")
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


class PackedB:
    """Owner of an abft_packed_b handle."""

    def __init__(self, handle: int, K: int, N: int):
        self.handle, self.K, self.N = handle, K, N

    def destroy(self):
        if self.handle:
            torch.cuda.synchronize()
            lib.abft_packed_b_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def abft_pack_b_checksum(B: torch.Tensor, b_is_transposed: bool = False, stream=None) -> PackedB:
    """B: int8 device tensor, K x N (or N x K when b_is_transposed)."""
    ptr = _ptr(B, torch.int8, "B")
    ldb = _ld(B, "B")
    K, N = (B.shape[1], B.shape[0]) if b_is_transposed else (B.shape[0], B.shape[1])
    out = ctypes.c_void_p()
    _check(lib.abft_pack_b_checksum(ptr, ldb, K, N, int(b_is_transposed), _stream(stream), ctypes.byref(out)))
    return PackedB(out.value, K, N)


def abft_packed_b_dims(Bp: PackedB):
    k, n = ctypes.c_int(), ctypes.c_int()
    _check(lib.abft_packed_b_dims(Bp.handle, ctypes.byref(k), ctypes.byref(n)))
    return k.value, n.value


def abft_packed_b_get_checksum(Bp: PackedB, S_B: torch.Tensor, stream=None):
    assert S_B.numel() >= Bp.K
    _check(lib.abft_packed_b_get_checksum(Bp.handle, _ptr(S_B, torch.int32, "S_B"), _stream(stream)))


def abft_packed_b_get_checksum_mod127(Bp: PackedB, row_sum: torch.Tensor, stream=None):
    assert row_sum.numel() >= Bp.K
    _check(lib.abft_packed_b_get_checksum_mod127(Bp.handle, _ptr(row_sum, torch.int32, "row_sum"), _stream(stream)))


def abft_packed_b_get_col_offsets(Bp: PackedB, colsum: torch.Tensor, stream=None):
    assert colsum.numel() >= Bp.N
    _check(lib.abft_packed_b_get_col_offsets(Bp.handle, _ptr(colsum, torch.int32, "colsum"), _stream(stream)))


def abft_packed_b_flip_bit(Bp: PackedB, k: int, j: int, bit: int, stream=None):
    _check(lib.abft_packed_b_flip_bit(Bp.handle, int(k), int(j), int(bit), _stream(stream)))


def abft_packed_b_flip_checksum_bit(Bp: PackedB, k: int, bit: int, stream=None):
    _check(lib.abft_packed_b_flip_checksum_bit(Bp.handle, int(k), int(bit), _stream(stream)))


def abft_packed_b_flip_checksum_bit_mod127(Bp: PackedB, k: int, bit: int, stream=None):
    _check(lib.abft_packed_b_flip_checksum_bit_mod127(Bp.handle, int(k), int(bit), _stream(stream)))


def abft_gemm_workspace_bytes(M: int, Bp: PackedB) -> int:
    return int(lib.abft_gemm_workspace_bytes(int(M), Bp.handle))


def abft_workspace_init(workspace: torch.Tensor, stream=None):
    _check(lib.abft_workspace_init(workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(stream)))


def make_requant(zA: int, zC: int, mult: torch.Tensor, bias: torch.Tensor | None = None) -> abft_requant_t:
    """Host struct holding device pointers; keep `mult`/`bias` alive while it is in use."""
    return abft_requant_t(int(zA), int(zC), _ptr(mult, torch.float32, "mult"), int(mult.numel() > 1),
                          _ptr(bias, torch.int32, "bias"))


def make_injections(entries, device="cuda") -> torch.Tensor:
    """[(row, col, xor_mask), ...] -> device tensor laid out as abft_inject_t[n]."""
    import numpy as np
    arr = np.zeros((len(entries), 3), dtype=np.uint32)
    for t, (r, c, m) in enumerate(entries):
        arr[t] = (r, c, m)
    return torch.from_numpy(arr.view(np.int32)).to(device)


def abft_gemm_u8s8s32_checked(A, Bp: PackedB, C, row_flags, err_count, rq=None, Cq=None, inj=None, n_inj=0,
                              flags=ABFT_CHECK, workspace=None, stream=None):
    M = A.shape[0]
    if A.shape[1] != Bp.K:
        raise ValueError(f"A is {tuple(A.shape)}, packed B has K={Bp.K}")
    for t, nm in ((C, "C"), (Cq, "Cq")):
        if t is not None and tuple(t.shape) != (M, Bp.N):
            raise ValueError(f"{nm} must be {M}x{Bp.N}")
    if row_flags is not None and row_flags.numel() < M:
        raise ValueError("row_flags shorter than M")
    if inj is not None and inj.numel() < 3 * n_inj:
        raise ValueError("injection tensor shorter than n_inj entries")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.abft_gemm_u8s8s32_checked(
        _ptr(A, torch.uint8, "A"), _ld(A, "A"), M, Bp.handle,
        _ptr(C, torch.int32, "C"), 0 if C is None else _ld(C, "C"),
        _ptr(row_flags, torch.int32, "row_flags"), _ptr(err_count, torch.int32, "err_count"),
        None if rq is None else ctypes.byref(rq), _ptr(Cq, torch.uint8, "Cq"), 0 if Cq is None else _ld(Cq, "Cq"),
        _ptr(inj, torch.int32, "inj"), int(n_inj), int(flags),
        None if workspace is None else workspace.data_ptr(), ws_bytes, _stream(stream)))


ABFT_STATIC_WS_MAX_M = 131072


def abft_gemm_u8s8s32_checked_static(A, Bp: PackedB, C, row_flags, err_count, rq=None, Cq=None, inj=None, n_inj=0,
                                     flags=ABFT_CHECK, stream=None):
    """The checked GEMM on the library's built-in workspace (no allocation, no workspace argument)."""
    M = A.shape[0]
    if A.shape[1] != Bp.K:
        raise ValueError(f"A is {tuple(A.shape)}, packed B has K={Bp.K}")
    for t, nm in ((C, "C"), (Cq, "Cq")):
        if t is not None and tuple(t.shape) != (M, Bp.N):
            raise ValueError(f"{nm} must be {M}x{Bp.N}")
    if row_flags is not None and row_flags.numel() < M:
        raise ValueError("row_flags shorter than M")
    if inj is not None and inj.numel() < 3 * n_inj:
        raise ValueError("injection tensor shorter than n_inj entries")
    _check(lib.abft_gemm_u8s8s32_checked_static(
        _ptr(A, torch.uint8, "A"), _ld(A, "A"), M, Bp.handle,
        _ptr(C, torch.int32, "C"), 0 if C is None else _ld(C, "C"),
        _ptr(row_flags, torch.int32, "row_flags"), _ptr(err_count, torch.int32, "err_count"),
        None if rq is None else ctypes.byref(rq), _ptr(Cq, torch.uint8, "Cq"), 0 if Cq is None else _ld(Cq, "Cq"),
        _ptr(inj, torch.int32, "inj"), int(n_inj), int(flags), _stream(stream)))


def abft_requantize_u8(C, Bp: PackedB, rq: abft_requant_t, Cq, stream=None):
    M, N = C.shape
    _check(lib.abft_requantize_u8(_ptr(C, torch.int32, "C"), _ld(C, "C"), M, N, Bp.handle, ctypes.byref(rq),
                                  _ptr(Cq, torch.uint8, "Cq"), _ld(Cq, "Cq"), _stream(stream)))


def abft_verify_rows(C, row_chk, row_flags, err_count=None, stream=None):
    M, N = C.shape
    _check(lib.abft_verify_rows(_ptr(C, torch.int32, "C"), _ld(C, "C"), M, N, _ptr(row_chk, torch.int32, "row_chk"),
                                _ptr(row_flags, torch.int32, "row_flags"), _ptr(err_count, torch.int32, "err_count"),
                                _stream(stream)))


def abft_row_checksum(A, Bp: PackedB, row_chk, stream=None):
    _check(lib.abft_row_checksum(_ptr(A, torch.uint8, "A"), _ld(A, "A"), A.shape[0], Bp.handle,
                                 _ptr(row_chk, torch.int32, "row_chk"), _stream(stream)))


def abft_recover_scratch_bytes(M: int, max_rows_per_pass: int, Bp: PackedB) -> int:
    return int(lib.abft_recover_scratch_bytes(M, max_rows_per_pass, Bp.handle))


def abft_recompute_flagged_rows(A, Bp: PackedB, C, row_flags, err_count=None, rq=None, Cq=None, max_rows_per_pass=256,
                                scratch=None, stream=None):
    """Recomputes the flagged rows in place (synchronises the stream).  Returns
    (rows found flagged, rows still flagged after the recomputation)."""
    M = A.shape[0]
    if scratch is None:
        scratch = torch.empty(abft_recover_scratch_bytes(M, max_rows_per_pass, Bp), dtype=torch.uint8, device=A.device)
    before, after = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib.abft_recompute_flagged_rows(
        _ptr(A, torch.uint8, "A"), _ld(A, "A"), M, Bp.handle,
        _ptr(C, torch.int32, "C"), _ld(C, "C") if C is not None else 0,
        _ptr(row_flags, torch.int32, "row_flags"), _ptr(err_count, torch.int32, "err_count"),
        ctypes.byref(rq) if rq is not None else None, _ptr(Cq, torch.uint8, "Cq"), _ld(Cq, "Cq") if Cq is not None else 0,
        max_rows_per_pass, scratch.data_ptr(), scratch.numel(), _stream(stream), ctypes.byref(before), ctypes.byref(after)))
    return before.value, after.value


def abft_recompute_flagged_rows_async(A, Bp: PackedB, C, row_flags, err_count=None, rq=None, Cq=None, max_rows=64,
                                      scratch=None, status=None, stream=None):
    """Recomputes up to max_rows flagged rows in place without synchronising; returns the device tensor
    `status` (rows found flagged, rows still flagged)."""
    M = A.shape[0]
    if scratch is None:
        scratch = torch.empty(abft_recover_scratch_bytes(M, max_rows, Bp), dtype=torch.uint8, device=A.device)
    if status is None:
        status = torch.empty(2, dtype=torch.int32, device=A.device)
    _check(lib.abft_recompute_flagged_rows_async(
        _ptr(A, torch.uint8, "A"), _ld(A, "A"), M, Bp.handle,
        _ptr(C, torch.int32, "C"), _ld(C, "C") if C is not None else 0,
        _ptr(row_flags, torch.int32, "row_flags"), _ptr(err_count, torch.int32, "err_count"),
        ctypes.byref(rq) if rq is not None else None, _ptr(Cq, torch.uint8, "Cq"), _ld(Cq, "Cq") if Cq is not None else 0,
        max_rows, scratch.data_ptr(), scratch.numel(), _ptr(status, torch.int32, "status"), _stream(stream)))
    return status


def abft_locate_scratch_bytes(Bp: PackedB) -> int:
    return int(lib.abft_locate_scratch_bytes(Bp.handle))


def abft_locate_correct(A, Bp: PackedB, C, row_flags, err_count=None, rq=None, Cq=None, col_flags=None, report=None,
                        scratch=None, stream=None):
    """Eq. 2a column check + repair of a single located element, in place, asynchronously.  Returns the device
    tensor holding the abft_locate_t report (8 int32: status, row, col, old, new, rows flagged, columns violated, -)."""
    M = A.shape[0]
    if scratch is None:
        scratch = torch.empty(abft_locate_scratch_bytes(Bp), dtype=torch.uint8, device=A.device)
    if report is None:
        report = torch.empty(8, dtype=torch.int32, device=A.device)
    if col_flags is not None and col_flags.numel() < Bp.N:
        raise ValueError("col_flags shorter than N")
    _check(lib.abft_locate_correct(
        _ptr(A, torch.uint8, "A"), _ld(A, "A"), M, Bp.handle, _ptr(C, torch.int32, "C"), _ld(C, "C"),
        _ptr(row_flags, torch.int32, "row_flags"), _ptr(err_count, torch.int32, "err_count"),
        ctypes.byref(rq) if rq is not None else None, _ptr(Cq, torch.uint8, "Cq"), _ld(Cq, "Cq") if Cq is not None else 0,
        _ptr(col_flags, torch.int32, "col_flags"), _ptr(report, torch.int32, "report"),
        scratch.data_ptr(), scratch.numel() * scratch.element_size(), _stream(stream)))
    return report


def abft_calib_copy(src, dst, stream=None):
    if src.numel() * src.element_size() != dst.numel() * dst.element_size():
        raise ValueError("abft_calib_copy: src and dst differ in size")
    if not (src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()):
        raise ValueError("abft_calib_copy: contiguous device tensors expected")
    _check(lib.abft_calib_copy(src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size(), _stream(stream)))


def abft_clock_probe(out: torch.Tensor, microseconds: int, stream=None):
    """out: int64 device tensor of 4 (wall ticks at 100 MHz and shader cycles, start and end)."""
    if out.dtype != torch.int64 or out.numel() < 4 or not out.is_cuda:
        raise ValueError("abft_clock_probe: out must be an int64 device tensor of at least 4 entries")
    _check(lib.abft_clock_probe(out.data_ptr(), int(microseconds), _stream(stream)))


def abft_mfma_peak_probe(out: torch.Tensor, iters: int, stream=None):
    """out: int64 device tensor of 4 * 256 (shader cycles, wall ticks before; the same after; per workgroup)."""
    if out.dtype != torch.int64 or out.numel() < 4 * 256 or not out.is_cuda:
        raise ValueError("abft_mfma_peak_probe: out must be an int64 device tensor of at least 1024 entries")
    _check(lib.abft_mfma_peak_probe(out.data_ptr(), int(iters), _stream(stream)))


def abft_clock_trace(buf: torch.Tensor | None):
    """Diagnostic library only: buf int64 device tensor, 6 entries per workgroup of the largest grid; None = off."""
    _check(lib.abft_clock_trace(None if buf is None else buf.data_ptr()))


class Workspace:
    """A zero-initialised workspace tensor sized for (M, Bp)."""

    def __init__(self, M: int, Bp: PackedB, device="cuda"):
        self.tensor = torch.empty(abft_gemm_workspace_bytes(M, Bp) // 4, dtype=torch.int32, device=device)
        abft_workspace_init(self.tensor)


# ---------------------------------------------------------------------------------------------
# include/abft_eb.h

class EbTable:
    """Owner of an abft_eb_table handle."""

    def __init__(self, handle: int, rows: int, d: int):
        self.handle, self.rows, self.d = handle, rows, d

    def destroy(self):
        if self.handle:
            torch.cuda.synchronize()
            lib.abft_eb_table_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def abft_eb_pack_rowsum(T: torch.Tensor, scale: torch.Tensor, bias: torch.Tensor, flags: int = 0, stream=None) -> EbTable:
    """T: uint8 device tensor, rows x d codes (rows x d/2 bytes with ABFT_EB_PACK_INT4); scale, bias: float32 [rows]."""
    ptr = _ptr(T, torch.uint8, "T")
    ldt = _ld(T, "T")
    rows, d = T.shape
    if flags & ABFT_EB_PACK_INT4:
        d *= 2
    if scale.numel() != rows or bias.numel() != rows or not scale.is_contiguous() or not bias.is_contiguous():
        raise ValueError("scale and bias must be contiguous with one entry per table row")
    out = ctypes.c_void_p()
    _check(lib.abft_eb_pack_rowsum(ptr, ldt, _ptr(scale, torch.float32, "scale"), _ptr(bias, torch.float32, "bias"),
                                   rows, d, int(flags), _stream(stream), ctypes.byref(out)))
    return EbTable(out.value, rows, d)


def abft_eb_table_dims(Tp: EbTable):
    rows, d, rec, bits = ctypes.c_int64(), ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(lib.abft_eb_table_dims(Tp.handle, ctypes.byref(rows), ctypes.byref(d), ctypes.byref(rec), ctypes.byref(bits)))
    return rows.value, d.value, rec.value, bits.value


def abft_eb_table_get_rowsums(Tp: EbTable, C_T: torch.Tensor, stream=None):
    if C_T.numel() < Tp.rows or not C_T.is_contiguous():
        raise ValueError("C_T must be contiguous with one entry per table row")
    _check(lib.abft_eb_table_get_rowsums(Tp.handle, _ptr(C_T, torch.int32, "C_T"), _stream(stream)))


def abft_eb_table_flip_bit(Tp: EbTable, row: int, col: int, bit: int, stream=None):
    _check(lib.abft_eb_table_flip_bit(Tp.handle, int(row), int(col), int(bit), _stream(stream)))


def abft_eb_u8_checked(Tp: EbTable, indices: torch.Tensor, offsets: torch.Tensor, R: torch.Tensor,
                       bag_flags: torch.Tensor | None, weights: torch.Tensor | None = None,
                       rsum: torch.Tensor | None = None, csum: torch.Tensor | None = None,
                       rel_bound: float = 1e-5, flags: int = 0, stream=None):
    """Algorithm 2 for a batch: offsets has one entry more than there are lookups."""
    n_bags = offsets.numel() - 1
    if n_bags < 0 or not offsets.is_contiguous() or not indices.is_contiguous():
        raise ValueError("indices and offsets must be contiguous; offsets needs n_bags + 1 entries")
    if R.dim() != 2 or R.shape[0] < n_bags or R.shape[1] != Tp.d:
        raise ValueError("R must be n_bags x d")
    for name, t in (("bag_flags", bag_flags), ("rsum", rsum), ("csum", csum)):
        if t is not None and (t.numel() < n_bags or not t.is_contiguous()):
            raise ValueError(f"{name} must be contiguous with one entry per lookup")
    if weights is not None and (weights.numel() != indices.numel() or not weights.is_contiguous()):
        raise ValueError("weights must be contiguous with one entry per index")
    _check(lib.abft_eb_u8_checked(Tp.handle, _ptr(indices, torch.int64, "indices"), indices.numel(),
                                  _ptr(offsets, torch.int64, "offsets"), n_bags, _ptr(weights, torch.float32, "weights"),
                                  _ptr(R, torch.float32, "R"), _ld(R, "R"), _ptr(bag_flags, torch.int32, "bag_flags"),
                                  _ptr(rsum, torch.float64, "rsum"), _ptr(csum, torch.float64, "csum"),
                                  float(rel_bound), int(flags), _stream(stream)))
