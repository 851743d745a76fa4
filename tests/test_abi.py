"""The C-ABI library loads, exports every symbol include/lowbit_gemm.h declares, and validates arguments
before touching the GPU (so these run without one).  No compute call is made here."""
import ctypes
import os
import re

import pytest

from paper_2205_09120_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2205_09120_amd import build
        build.build()
    return binding.lib()


def _declared():
    text = open(os.path.join(ROOT, "include", "lowbit_gemm.h")).read()
    return sorted(set(re.findall(r"LB_API\s+[\w\s\*]+?\b(\w+)\s*\(", text)))


def test_header_symbols_exported(L):
    names = _declared()
    assert len(names) >= 13
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_format_version(L):
    assert L.lb_format_version() == 1


def test_size_helpers(L):
    assert L.packed_binary_bytes(64, 576) == 64 * 9 * 8
    assert L.packed_ternary_bytes(64, 576) == 64 * 9 * 16
    assert L.packed_binary_bytes(3, 65) == 3 * 2 * 8
    assert L.packed_ternary_bytes(0, 100) == 0
    assert L.packed_binary_bytes(-1, 5) == 0
    assert L.packed_ternary_bytes(2 ** 62, 2 ** 40) == 0            # overflow -> 0


def test_gemm_argument_validation(L):
    fake = 0x1000                                                   # never dereferenced: validation fails first
    for f in (L.gemm_bnn, L.gemm_tnn, L.gemm_tbn):
        assert f(-1, 4, 64, fake, fake, fake, 4, None) == binding.LB_EINVAL
        assert f(4, 4, 0, fake, fake, fake, 4, None) == binding.LB_EINVAL
        assert f(4, 4, 2 ** 31, fake, fake, fake, 4, None) == binding.LB_EOVERFLOW
        assert f(4, 4, 64, None, fake, fake, 4, None) == binding.LB_EINVAL
        assert f(4, 4, 64, fake, fake, None, 4, None) == binding.LB_EINVAL
        assert f(4, 8, 64, fake, fake, fake, 7, None) == binding.LB_EINVAL          # ldc < N
        assert f(4, 4, 64, fake + 8, fake, fake, 4, None) == binding.LB_EINVAL      # misaligned packed operand
        assert f(0, 4, 64, None, None, None, 4, None) == binding.LB_OK              # empty problem
        assert f(4, 0, 64, None, None, None, 0, None) == binding.LB_OK
    assert b"ldc" in L.lb_last_error() or b"aligned" in L.lb_last_error()


def test_pack_argument_validation(L):
    fake = 0x1000
    for f in (L.pack_binary, L.pack_ternary):
        assert f(fake, -1, 64, 64, 1, fake, None) == binding.LB_EINVAL
        assert f(None, 4, 64, 64, 1, fake, None) == binding.LB_EINVAL
        assert f(fake, 4, 64, 32, 1, fake, None) == binding.LB_EINVAL               # stride_r < K
        assert f(fake, 4, 64, 1, 3, fake, None) == binding.LB_EINVAL                # stride_k < rows
        assert f(fake, 4, 64, 2, 2, fake, None) == binding.LB_EINVAL                # neither stride is 1
        assert f(fake, 4, 64, 64, 1, fake + 4, None) == binding.LB_EINVAL           # dst misaligned
        assert f(fake, 2 ** 31, 64, 64, 1, fake, None) == binding.LB_EOVERFLOW
        assert f(None, 0, 64, 64, 1, None, None) == binding.LB_OK
        assert f(None, 4, 0, 1, 1, None, None) == binding.LB_OK


def test_i8_argument_validation(L):
    fake = 0x1000
    f = L.gemm_i8_mfma
    assert f(4, 4, 0, fake, 4, fake, 4, fake, 4, None) == binding.LB_EINVAL
    assert f(4, 4, 16, fake, 8, fake, 4, fake, 4, None) == binding.LB_EINVAL        # lda < K
    assert f(4, 4, 16, fake, 16, fake, 3, fake, 4, None) == binding.LB_EINVAL       # ldb < N
    assert f(4, 4, 1 << 20, fake, 1 << 20, fake, 4, fake, 4, None) == binding.LB_EOVERFLOW
    assert f(0, 4, 16, None, 16, None, 4, None, 4, None) == binding.LB_OK


def test_im2col_argument_validation(L):
    fake = 0x1000
    f = L.im2col_packed
    assert f(fake, 3, 1, 8, 8, 64, 3, 3, 1, 1, 1, 1, fake, None) == binding.LB_EINVAL          # planes
    assert f(fake, 2, 1, 8, 8, 64, 3, 3, 0, 1, 1, 1, fake, None) == binding.LB_EINVAL          # stride 0
    assert f(fake, 2, 1, 8, 8, 64, 3, 3, 1, 1, -1, 1, fake, None) == binding.LB_EINVAL         # negative padding
    assert f(fake, 2, 1, 8, 8, 72, 3, 3, 1, 1, 1, 1, fake, None) == binding.LB_EUNSUPPORTED    # C % 64 != 0
    assert f(None, 2, 1, 8, 8, 64, 3, 3, 1, 1, 1, 1, fake, None) == binding.LB_EINVAL
    assert f(fake, 2, 1, 8, 8, 64, 3, 3, 1, 1, 1, 1, fake + 8, None) == binding.LB_EINVAL      # misaligned
    assert f(None, 2, 0, 8, 8, 64, 3, 3, 1, 1, 1, 1, None, None) == binding.LB_OK              # empty batch
    assert f(None, 1, 4, 2, 2, 64, 5, 5, 1, 1, 0, 0, None, None) == binding.LB_OK              # window larger than map
    assert f(fake, 2, 1, 1 << 25, 8, 64, 3, 3, 1, 1, 1, 1, fake, None) == binding.LB_EOVERFLOW


def test_u8_argument_validation(L):
    fake = 0x1000
    f = L.gemm_u8_mfma
    assert f(4, 4, 16, fake, 16, fake, 4, 256, 0, fake, 4, None) == binding.LB_EINVAL      # zero point out of range
    assert f(4, 4, 16, fake, 16, fake, 4, 0, -1, fake, 4, None) == binding.LB_EINVAL
    assert f(4, 4, 33026, fake, 33026, fake, 4, 0, 0, fake, 4, None) == binding.LB_EOVERFLOW
    assert f(4, 4, 16, fake, 8, fake, 4, 0, 0, fake, 4, None) == binding.LB_EINVAL         # lda < K
    assert f(0, 4, 16, None, 16, None, 4, 0, 0, None, 4, None) == binding.LB_OK


def test_requant_argument_validation(L):
    fake = 0x1000
    f = L.gemm_requant
    assert f(3, 2, 4, 4, 64, fake, fake, fake, fake, fake, None) == binding.LB_EINVAL        # kind
    assert f(1, 3, 4, 4, 64, fake, fake, fake, fake, fake, None) == binding.LB_EINVAL        # planes
    assert f(1, 2, 4, 4, 0, fake, fake, fake, fake, fake, None) == binding.LB_EINVAL         # K
    assert f(1, 2, 4, 4, 64, fake, fake, fake, None, fake, None) == binding.LB_EINVAL        # ternary needs hi
    assert f(1, 2, 4, 4, 64, fake, fake, fake, fake, fake + 8, None) == binding.LB_EINVAL    # Out misaligned
    assert f(0, 1, 0, 4, 64, None, None, None, None, None, None) == binding.LB_OK


def test_calibration_argument_validation(L):
    fake = 0x1000
    assert L.lb_calib_sink_bytes() > 0
    assert L.lb_calib_valu_lane_instr(1) > 0 and L.lb_calib_valu_lane_instr(0) == 0
    assert L.lb_calib_valu(0, 0, fake, None) == binding.LB_EINVAL
    assert L.lb_calib_valu(0, 10, None, None) == binding.LB_EINVAL
    assert L.lb_calib_valu(2, 10, fake, None) == binding.LB_EINVAL
    assert L.lb_calib_stream(3, fake, fake, 16, fake, None) == binding.LB_EINVAL
    assert L.lb_calib_stream(2, fake, fake, 15, fake, None) == binding.LB_EINVAL
    assert L.lb_calib_stream(0, None, None, 16, fake, None) == binding.LB_EINVAL
    assert L.lb_calib_stream(1, None, None, 16, None, None) == binding.LB_EINVAL


def test_variant_hooks(L):
    for op in range(3):
        n = L.lb_num_variants(op)
        assert n >= 1
        for v in range(n):
            assert L.lb_variant_name(op, v)
        assert L.lb_variant_name(op, n) is None
        assert L.lb_set_variant(op, n) == binding.LB_EINVAL
        assert L.lb_set_variant(op, n - 1) == binding.LB_OK
        assert L.lb_set_variant(op, -1) == binding.LB_OK
    assert L.lb_num_variants(3) >= 1 and L.lb_set_variant(3, 0) == binding.LB_OK
    assert L.lb_set_variant(3, -1) == binding.LB_OK
    assert L.lb_set_variant(3, L.lb_num_variants(3)) == binding.LB_EINVAL
    assert L.lb_set_variant(4, 0) == binding.LB_OK and L.lb_set_variant(4, -1) == binding.LB_OK
    assert L.lb_set_variant(5, 0) == binding.LB_EINVAL
    assert L.lb_num_variants(7) == 0


def test_binding_raises_with_message(L):
    with pytest.raises(binding.LowbitError) as e:
        binding._check(L.gemm_tnn(4, 8, 64, 0x1000, 0x1000, 0x1000, 7, None))
    assert e.value.status == binding.LB_EINVAL and "ldc" in str(e.value)
