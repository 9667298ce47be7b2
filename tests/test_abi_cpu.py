"""Host-side checks that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2103_00130_amd import binding as b
    return b


def declared_functions(header="abft_gemm.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(abft_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(binding):
    names = declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(binding.lib, n), f"{n} is declared in include/abft_gemm.h but not exported"
    assert sorted(binding.EXPORTS) == names
    names_eb = declared_functions("abft_eb.h")
    assert len(names_eb) >= 6
    for n in names_eb:
        assert hasattr(binding.lib, n), f"{n} is declared in include/abft_eb.h but not exported"
    assert sorted(binding.EXPORTS_EB) == names_eb
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["abft_eb.h", "abft_gemm.h"]


def test_bad_arguments_are_rejected_on_the_host(binding):
    L = binding.lib
    out = ctypes.c_void_p()
    assert L.abft_pack_b_checksum(None, 8, 8, 8, 0, None, ctypes.byref(out)) == binding.ABFT_EINVAL
    assert b"null" in L.abft_last_error()
    dummy = ctypes.c_void_p(0x1000)
    assert L.abft_pack_b_checksum(dummy, 8, 0, 8, 0, None, ctypes.byref(out)) == binding.ABFT_EINVAL
    assert L.abft_pack_b_checksum(dummy, 4, 8, 8, 0, None, ctypes.byref(out)) == binding.ABFT_EINVAL   # ldb < N
    assert L.abft_gemm_u8s8s32_checked(None, 8, 1, None, None, 0, None, None, None, None, 0, None, 0, 0, None, 0,
                                       None) == binding.ABFT_EINVAL
    assert L.abft_packed_b_dims(None, None, None) == binding.ABFT_EINVAL
    assert L.abft_workspace_init(None, 64, None) == binding.ABFT_EINVAL
    assert L.abft_gemm_workspace_bytes(0, None) == 0
    assert L.abft_gemm_workspace_bytes(100, None) == (64 + 2 * (32 * 64 + 64)) * 4
    assert L.abft_gemm_workspace_bytes(4096, None) == (64 + 2 * 4096) * 4
    assert L.abft_verify_rows(None, 0, 1, 1, None, None, None, None) == binding.ABFT_EINVAL
    assert L.abft_requantize_u8(None, 0, 1, 1, None, None, None, 0, None) == binding.ABFT_EINVAL
    assert L.abft_row_checksum(None, 0, 1, None, None, None) == binding.ABFT_EINVAL
    assert L.abft_recover_scratch_bytes(0, 1, None) == 0
    assert L.abft_recompute_flagged_rows(None, 0, 1, None, None, 0, None, None, None, None, 0, 1, None, 0, None, None,
                                         None) == binding.ABFT_EINVAL
    assert L.abft_calib_copy(None, None, 16, None) == binding.ABFT_EINVAL
    assert L.abft_calib_copy(4096, 8192, 24, None) == binding.ABFT_EINVAL      # not a multiple of 16
    assert L.abft_calib_copy(4096, 8200, 32, None) == binding.ABFT_EINVAL      # misaligned


def test_eb_bad_arguments_are_rejected_on_the_host(binding):
    L = binding.lib
    out = ctypes.c_void_p()
    dummy = ctypes.c_void_p(0x1000)
    assert L.abft_eb_pack_rowsum(None, 64, dummy, dummy, 10, 64, 0, None, ctypes.byref(out)) == binding.ABFT_EINVAL
    assert L.abft_eb_pack_rowsum(dummy, 64, dummy, dummy, 0, 64, 0, None, ctypes.byref(out)) == binding.ABFT_EINVAL
    assert L.abft_eb_pack_rowsum(dummy, 32, dummy, dummy, 10, 64, 0, None, ctypes.byref(out)) == binding.ABFT_EINVAL  # ldt < d
    assert L.abft_eb_pack_rowsum(dummy, 100, dummy, dummy, 10, 100, 0, None, ctypes.byref(out)) == binding.ABFT_EUNSUPPORTED
    assert b"d=100" in L.abft_last_error()
    assert L.abft_eb_pack_rowsum(dummy, 64, dummy, dummy, 10, 64, 12, None, ctypes.byref(out)) == binding.ABFT_EINVAL  # unknown flag
    assert L.abft_eb_pack_rowsum(dummy, 64, dummy, dummy, 10, 16, 2, None, ctypes.byref(out)) == binding.ABFT_EUNSUPPORTED  # 8 bytes a row
    assert L.abft_eb_table_dims(None, None, None, None, None) == binding.ABFT_EINVAL
    assert L.abft_eb_table_get_rowsums(None, dummy, None) == binding.ABFT_EINVAL
    assert L.abft_eb_table_flip_bit(None, 0, 0, 0, None) == binding.ABFT_EINVAL
    assert L.abft_eb_u8_checked(None, dummy, 0, dummy, 0, None, dummy, 64, dummy, None, None, 1e-5, 0, None) == binding.ABFT_EINVAL
    L.abft_eb_table_destroy(None)


def test_injection_struct_layout(binding):
    assert ctypes.sizeof(binding.abft_inject_t) == 12
    assert ctypes.sizeof(binding.abft_requant_t) == 32
    t = binding.abft_requant_t
    assert (t.zA.offset, t.zC.offset, t.mult.offset, t.per_channel.offset, t.bias.offset) == (0, 4, 8, 16, 24)
