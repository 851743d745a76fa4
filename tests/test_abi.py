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
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
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


def test_c16_argument_validation(L):
    fake = 0x1000
    f = L.gemm_c16
    assert f(3, 4, 4, 64, fake, fake, fake, 4, None) == binding.LB_EINVAL           # no such operand class
    assert f(1, 4, 4, 32768, fake, fake, fake, 4, None) == binding.LB_EOVERFLOW     # Table II: k_max = 32767
    assert b"32767" in L.lb_last_error()
    assert f(1, 4, 4, 0, fake, fake, fake, 4, None) == binding.LB_EINVAL
    assert f(0, 4, 8, 64, fake, fake, fake, 7, None) == binding.LB_EINVAL           # ldc < N
    assert f(2, 4, 4, 64, fake, fake, fake + 1, 4, None) == binding.LB_EINVAL       # C not 2-byte aligned
    assert f(2, 0, 4, 64, None, None, None, 4, None) == binding.LB_OK               # empty problem


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


def test_u4_argument_validation(L):
    fake = 0x1000
    assert L.packed_u4_bytes(1, 1) == 2 * 1536
    assert L.packed_u4_bytes(33, 129) == 2 * 4 * 1536
    assert L.packed_u4_bytes(1024, 4608) == 32 * 72 * 1536
    assert L.packed_u4_bytes(0, 5) == 0 and L.packed_u4_bytes(-1, 5) == 0
    p = L.pack_u4
    assert p(None, 4, 64, 64, 1, fake, fake, None) == binding.LB_EINVAL                      # null source
    assert p(fake, 4, 64, 32, 1, fake, fake, None) == binding.LB_EINVAL                      # stride_r < K
    assert p(fake, 4, 64, 2, 2, fake, fake, None) == binding.LB_EINVAL                       # neither stride is 1
    assert p(fake, 4, 64, 64, 1, fake + 8, fake, None) == binding.LB_EINVAL                  # dst misaligned
    assert p(fake, 4, 74566, 74566, 1, fake, fake, None) == binding.LB_EOVERFLOW
    assert p(None, 0, 64, 64, 1, None, None, None) == binding.LB_OK
    g = L.gemm_u4_mfma
    assert g(4, 4, 64, fake, fake, fake, fake, 16, 0, fake, 4, None) == binding.LB_EINVAL    # zero point out of range
    assert g(4, 4, 64, fake, fake, fake, fake, 0, -1, fake, 4, None) == binding.LB_EINVAL
    assert g(4, 4, 0, fake, fake, fake, fake, 0, 0, fake, 4, None) == binding.LB_EINVAL
    assert g(4, 4, 74566, fake, fake, fake, fake, 0, 0, fake, 4, None) == binding.LB_EOVERFLOW
    assert b"74565" in L.lb_last_error()
    assert g(4, (1 << 31) - 255, 64, fake, fake, fake, fake, 0, 0, fake, 1 << 31, None) == binding.LB_EOVERFLOW
    assert g(4, 4, 64, fake, None, fake, fake, 0, 0, fake, 4, None) == binding.LB_EINVAL     # null sums
    assert g(4, 4, 64, fake, fake, fake, fake, 0, 0, fake, 3, None) == binding.LB_EINVAL     # ldc < N
    assert g(4, 4, 64, fake + 4, fake, fake, fake, 0, 0, fake, 4, None) == binding.LB_EINVAL  # Ap misaligned
    assert g(0, 4, 64, None, None, None, None, 0, 0, None, 4, None) == binding.LB_OK


def test_t4_argument_validation(L):
    fake = 0x1000
    assert L.packed_t4_bytes(1, 1) == 2 * 1024 and L.packed_t4_bytes(1024, 4608) == 32 * 72 * 1024
    assert L.packed_t4_bytes(0, 5) == 0
    p = L.pack_t4
    assert p(None, 4, 64, 64, 1, fake, None) == binding.LB_EINVAL
    assert p(fake, 4, 64, 32, 1, fake, None) == binding.LB_EINVAL                            # stride_r < K
    assert p(fake, 4, 64, 64, 1, fake + 8, None) == binding.LB_EINVAL                        # dst misaligned
    assert p(fake, 4, 1 << 24, 1 << 24, 1, fake, None) == binding.LB_EOVERFLOW
    assert p(None, 0, 64, 64, 1, None, None) == binding.LB_OK
    g = L.gemm_t4_mfma
    assert g(4, 4, 0, fake, fake, fake, 4, None) == binding.LB_EINVAL
    assert g(4, 4, 1 << 24, fake, fake, fake, 4, None) == binding.LB_EOVERFLOW
    assert g(4, 4, 64, fake, None, fake, 4, None) == binding.LB_EINVAL
    assert g(4, 4, 64, fake, fake, fake, 3, None) == binding.LB_EINVAL                       # ldc < N
    assert g((1 << 31) - 255, 4, 64, fake, fake, fake, 4, None) == binding.LB_EOVERFLOW      # tile indices past int32
    assert g(4, 4, 64, fake + 4, fake, fake, 4, None) == binding.LB_EINVAL                   # Ap misaligned
    assert g(0, 4, 64, None, None, None, 4, None) == binding.LB_OK


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
    assert L.lb_calib_sink_bytes() > 0 and L.lb_calib_clocks_bytes() > 0
    assert L.lb_calib_valu_lane_instr(0, 1, 8) > 0 and L.lb_calib_valu_lane_instr(0, 0, 8) == 0
    assert L.lb_calib_valu_lane_instr(1, 10, 4) == 2 * L.lb_calib_valu_lane_instr(0, 10, 4)   # 4 against 2 per unit
    assert L.lb_calib_valu_lane_instr(7, 10, 4) == 0 and L.lb_calib_valu_lane_instr(0, 10, 9) == 0
    assert L.lb_calib_valu(0, 0, 8, fake, None, None) == binding.LB_EINVAL
    assert L.lb_calib_valu(0, 10, 8, None, None, None) == binding.LB_EINVAL
    assert L.lb_calib_valu(7, 10, 8, fake, None, None) == binding.LB_EINVAL
    assert L.lb_calib_valu(0, 10, 0, fake, None, None) == binding.LB_EINVAL
    assert L.lb_calib_valu(0, 10, 8, fake, fake + 4, None) == binding.LB_EINVAL     # misaligned clock buffer
    assert L.lb_calib_stream(3, fake, fake, 16, 0, fake, None) == binding.LB_EINVAL
    assert L.lb_calib_stream(2, fake, fake, 15, 0, fake, None) == binding.LB_EINVAL
    assert L.lb_calib_stream(0, None, None, 16, 0, fake, None) == binding.LB_EINVAL
    assert L.lb_calib_stream(1, None, None, 16, 0, None, None) == binding.LB_EINVAL
    assert L.lb_calib_stream(0, fake, None, 16, -1, fake, None) == binding.LB_EINVAL


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
    assert L.lb_set_variant(4, L.lb_num_variants(4)) == binding.LB_EINVAL
    assert L.lb_set_variant(5, 0) == binding.LB_OK and L.lb_set_variant(5, -1) == binding.LB_OK
    assert L.lb_set_variant(5, L.lb_num_variants(5)) == binding.LB_EINVAL
    assert L.lb_set_variant(6, 0) == binding.LB_EINVAL
    assert L.lb_num_variants(7) == 0


def test_binding_raises_with_message(L):
    with pytest.raises(binding.LowbitError) as e:
        binding._check(L.gemm_tnn(4, 8, 64, 0x1000, 0x1000, 0x1000, 7, None))
    assert e.value.status == binding.LB_EINVAL and "ldc" in str(e.value)


def test_grouped_planning_is_host_logic(L):
    """gemm_grouped_plan runs without a GPU: the table it writes is checked against its documented structure."""
    import numpy as np
    P = binding.GemmProblem
    probs = [P(72, 24, 128, 0x1000, 0x2000, 0x3000, 24),    # narrow N: B rides on the scalar side (transposed)
             P(0, 5, 64, None, None, None, 5),               # empty: owns no workgroup
             P(100, 96, 512, 0x4000, 0x5000, 0x6000, 100)]   # lanes own columns
    for kind, want_tr in (("bnn", [1, 0]), ("tnn", [1, 0]), ("tbn", [1, 1])):
        table, wg = binding.gemm_grouped_plan(kind, probs)
        assert table.numel() == binding.gemm_grouped_table_bytes(kind, probs) and table.numel() % 16 == 0
        raw = table.numpy()
        magic, k, count, total = raw[:16].view(np.uint32)
        assert (magic, k, count, total) == (0x4C424754, binding._OPS[kind], 3, wg)
        recs = raw[16:16 + 64 * 3].view(np.int32).reshape(3, 16)
        owner = raw[16 + 64 * 3:16 + 64 * 3 + 4 * wg].view(np.uint32)
        live = [recs[0], recs[2]]
        tiles = []
        for r, tr, (M, N, K, a, b) in zip(live, want_tr, [(72, 24, 128, 0x1000, 0x2000), (100, 96, 512, 0x4000, 0x5000)]):
            rowsS, rowsV = (N, M) if tr else (M, N)
            assert r[14] == tr and (r[8], r[9], r[10], r[11]) == (rowsS, rowsV, (K + 63) // 64, K)
            assert (r[0], r[2]) == ((b, a) if tr else (a, b))
            assert r[12] == -(-rowsS // 16)
            tiles.append(int(r[12]) * -(-rowsV // 64))
        assert wg == sum(tiles)
        assert recs[0][13] == 0 and recs[1][13] == tiles[0] and recs[2][13] == tiles[0]
        assert list(owner) == [0] * tiles[0] + [2] * tiles[1]


def test_grouped_argument_validation(L):
    P = binding.GemmProblem
    ok = P(8, 8, 64, 0x1000, 0x2000, 0x3000, 8)
    for bad in (P(8, 8, 0, 0x1000, 0x2000, 0x3000, 8), P(8, 8, 64, None, 0x2000, 0x3000, 8),
                P(8, 8, 64, 0x1000, 0x2000, 0x3000, 7), P(-1, 8, 64, 0x1000, 0x2000, 0x3000, 8),
                P(8, 8, 64, 0x1008, 0x2000, 0x3000, 8)):
        assert binding.gemm_grouped_table_bytes("tnn", [ok, bad]) == 0
        assert b"problem 1" in L.lb_last_error()
        with pytest.raises(binding.LowbitError) as e:
            binding.gemm_grouped_plan("tnn", [ok, bad])
        assert e.value.status == binding.LB_EINVAL
    with pytest.raises(binding.LowbitError) as e:
        binding.gemm_grouped_plan("tnn", [P(8, 8, 2 ** 31, 0x1000, 0x2000, 0x3000, 8)])
    assert e.value.status == binding.LB_EOVERFLOW
    assert binding.gemm_grouped_table_bytes(3, [ok]) == 0
    # too small a table buffer, null outputs
    arr = (P * 1)(ok)
    buf = ctypes.create_string_buffer(64)
    wg = ctypes.c_int64(0)
    assert L.gemm_grouped_plan(1, 1, arr, buf, 64, ctypes.byref(wg)) == binding.LB_EINVAL
    assert L.gemm_grouped_plan(1, 1, arr, None, 4096, ctypes.byref(wg)) == binding.LB_EINVAL
    assert L.gemm_grouped_plan(1, 1, None, buf, 64, ctypes.byref(wg)) == binding.LB_EINVAL
    # launch call: everything is checked before the first HIP call
    assert L.gemm_grouped(1, 0, None, 0, None) == binding.LB_OK
    assert L.gemm_grouped(5, 1, 0x1000, 1, None) == binding.LB_EINVAL
    assert L.gemm_grouped(1, 1, None, 1, None) == binding.LB_EINVAL
    assert L.gemm_grouped(1, 1, 0x1004, 1, None) == binding.LB_EINVAL
    assert L.gemm_grouped(1, 0, 0x1000, 1, None) == binding.LB_EINVAL
    assert L.gemm_grouped(1, -1, 0x1000, 1, None) == binding.LB_EINVAL
    assert L.gemm_grouped(1, 1, 0x1000, 2 ** 31, None) == binding.LB_EOVERFLOW
    # an empty group plans to a header-only table
    table, wg2 = binding.gemm_grouped_plan("bnn", [])
    assert wg2 == 0 and table.numel() == 16


def test_dispatch_plan_is_host_logic(L):
    """Which kernel a call would run, decided on the host: the headline shape takes the large tile, the
    fully connected configuration the depth-split-across-lanes kernel, many shallow rows the tiled kernel with a low
    tile, few tiles with a long depth the depth ranges, gemm_tbn with few ternary rows the swapped roles."""
    d = binding.lb_describe_plan
    assert d("tnn", 1024, 50176, 4608) == "tnn tiled kernel [KIND_TNN ts4 tv2 w8 kg8 sg4], A on the scalar side"
    assert d("tnn", 64, 256, 576) == "tnn tiled kernel [KIND_TNN ts1 tv1 w8 kg16 sg4], A on the scalar side"
    assert d("bnn", 256, 3136, 1152) == "bnn tiled kernel [KIND_BNN ts4 tv1 w8 kg16 sg8], A on the scalar side"
    assert d("tbn", 512, 784, 2304) == "tbn tiled kernel [KIND_TBN ts4 tv1 w8 kg16 sg8], B on the scalar side"
    for kind in ("tnn", "tbn", "bnn"):
        assert d(kind, 4096, 8, 16384) == f"{kind} depth-split-across-lanes kernel, A streamed"
        # many shallow rows: not the depth-split kernel, but 8-row tiles with the 8 strings of B in scalar registers
        t = d(kind, 100000, 8, 576)
        assert "tiled kernel" in t and " ts1 tv1 w8 " in t and t.endswith("B on the scalar side")
        # 9..16 short strings: 16-row tiles once the problem is large
        assert " ts4 tv1 w4 " in d(kind, 262144, 16, 1024)
    assert d("tnn", 128, 128, 16384).startswith("tnn tiled kernel, ") and "depth ranges" in d("tnn", 128, 128, 16384)
    assert "depth ranges" not in d("tnn", 128, 128, 16384, c16=True)        # a 16-bit C cannot take atomic adds
    assert "depth ranges" not in d("tnn", 4096, 48, 16384)                  # enough tiles to fill the machine
    assert "depth ranges" in d("tbn", 256, 256, 16384) and "depth ranges" in d("bnn", 512, 49, 16384)
    assert "depth ranges" not in d("tnn", 128, 128, 4608)                   # too shallow to pay for a cleared C
    assert d("tbn", 8, 50176, 4608).startswith("tbn (ternary operand on the scalar side")
    assert d("tbn", 8, 4096, 16384) == "tbn (ternary operand on the scalar side / in LDS) " \
                                         "depth-split-across-lanes kernel, B streamed"
    assert d("tbn", 48, 50176, 4608).startswith("tbn tiled kernel")         # enough ternary rows: binary on scalar side
    assert "depth-split-across-lanes" in d("tnn", 4096, 32, 16384)          # up to 32 short strings, deep and few rows
    assert "tiled kernel" in d("tnn", 65536, 32, 16384) and "tiled kernel" in d("tnn", 4096, 32, 2304)
    assert "tiled kernel" in d("tnn", 4096, 33, 16384)
    assert d("tnn", 0, 5, 64) is None and d("tnn", 4, 4, 0) is None and L.lb_describe_plan(7, 4, 4, 64, 0) is None
    try:
        assert L.lb_set_variant(1, 0) == binding.LB_OK                      # a forced variant overrides all of it
        assert d("tnn", 4096, 8, 16384) == "tnn tiled kernel [KIND_TNN ts4 tv1 w4 kg16 sg4], B on the scalar side"
    finally:
        L.lb_set_variant(1, -1)


def test_eight_wave_tiles_are_chosen_by_depth_and_tile_count(L):
    """The 32 x 128 / 32 x 64 tiles of eight waves: from 32 depth words on, from about a thousand workgroups on, or
    when their workgroups fill whole rounds of two per compute unit; never for shallow products."""
    d = binding.lb_describe_plan
    wide, narrow = "ts4 tv2 w8 kg8 sg4", "ts4 tv1 w8 kg16 sg4"
    assert wide in d("tnn", 512, 8192, 2304)          # 16 x 64 = 1024 tiles of 32 x 128
    assert wide in d("tnn", 1024, 12544, 4608)
    assert narrow in d("tnn", 1024, 3136, 9216)       # 800 tiles of 32 x 128, but 1568 of 32 x 64
    assert narrow in d("tnn", 384, 6272, 3456)
    assert wide in d("tnn", 512, 4096, 2304)          # 512 tiles of 32 x 128: exactly two per compute unit
    assert wide not in d("tnn", 2048, 6272, 1152) and narrow not in d("tnn", 2048, 6272, 1152)   # 18 depth words
    assert wide in d("bnn", 512, 8192, 2304) and wide in d("bnn", 512, 4096, 2304)
    assert wide in d("bnn", 300, 9000, 4096)          # 710 tiles >= 600
    assert wide not in d("bnn", 1536, 1536, 6144)     # 576 tiles: neither enough nor whole rounds
    assert "ts8 tv2 w8 kg8 sg4" in d("bnn", 1024, 50176, 4608)   # the 64 x 128 tile keeps the largest problems
    assert "ts8 tv2 w8 kg8 sg4" in d("tbn", 1024, 12544, 4608)   # ternary-binary: eight waves of eight rows from 1024 tiles
    assert "ts8 tv4 w8 kg4 sg1" in d("tbn", 1024, 50176, 4608)
    assert "ts8 tv1 w4 kg8 sg4" in d("tbn", 384, 6272, 3456)     # 1176 tiles of 32 x 64


def test_grouped_static_argument_validation(L):
    """The allocation-free grouped launch checks its table on the host before any HIP call."""
    P = binding.GemmProblem
    ok = P(20, 30, 100, 0x1000, 0x2000, 0x3000, 30)
    table, wg = binding.gemm_grouped_plan("tnn", [ok])
    n = table.numel()
    assert L.gemm_grouped_static_max_bytes() == 64 * 1024
    assert L.gemm_grouped_static(1, 0, None, 0, 0, None) == binding.LB_OK                    # nothing to do
    assert L.gemm_grouped_static(7, 1, table.data_ptr(), n, wg, None) == binding.LB_EINVAL   # kind
    assert L.gemm_grouped_static(1, 1, None, n, wg, None) == binding.LB_EINVAL               # null table
    assert L.gemm_grouped_static(1, 1, table.data_ptr(), n + 16, wg, None) == binding.LB_EINVAL   # size mismatch
    assert L.gemm_grouped_static(0, 1, table.data_ptr(), n, wg, None) == binding.LB_EINVAL   # planned for TNN
    assert L.gemm_grouped_static(1, -1, table.data_ptr(), n, wg, None) == binding.LB_EINVAL
    assert L.gemm_grouped_static(1, 1, table.data_ptr(), n, 2 ** 31, None) == binding.LB_EOVERFLOW
    # a table beyond the library's array is refused with a clear message, nothing is enqueued
    many = [P(16, 64, 64, 0x1000, 0x2000, 0x3000 + 0x10000 * i, 64) for i in range(1100)]
    big, wgb = binding.gemm_grouped_plan("bnn", many)
    assert big.numel() > 64 * 1024
    assert L.gemm_grouped_static(0, len(many), big.data_ptr(), big.numel(), wgb, None) == binding.LB_EUNSUPPORTED
    assert b"exceeds" in L.lb_last_error()


def test_arch_check_is_host_logic(L):
    """Only gfx950 devices are served: the rule every entry point applies before its first launch on a device."""
    assert binding.lb_arch_supported("gfx950")
    assert binding.lb_arch_supported("gfx950:sramecc+:xnack-")
    for other in ("gfx942", "gfx942:sramecc+:xnack-", "gfx90a", "gfx9500", "gfx95", "", "sm_90"):
        assert not binding.lb_arch_supported(other), other
    assert L.lb_arch_supported(None) == 0


def test_i8_grouped_planning_and_validation(L):
    """The grouped launch of the 8-bit comparator plans on the host: table structure and argument rules, no GPU."""
    import numpy as np
    P = binding.I8Problem
    probs = [P(72, 24, 128, 0x10000, 128, 0x20000, 24, 0x30000, 24),      # 2 x 1 tiles, N not a multiple of 16
             P(0, 9, 64, None, 64, None, 9, None, 9),                     # empty: owns no workgroup
             P(130, 70, 191, 0x40001, 191, 0x50003, 70, 0x60000, 75)]     # unaligned operands, ragged: 3 x 2 tiles
    table, wg = binding.gemm_i8_grouped_plan(probs)
    assert wg == 2 + 0 + 6
    assert table.numel() == binding.gemm_i8_grouped_table_bytes(probs) == (16 + 3 * 80 + 8 * 4 + 15) // 16 * 16
    t = table.numpy()
    hdr = t[:16].view(np.uint32)
    assert hdr[0] == 0x4c423847 and hdr[1] == 3 and hdr[2] == 8
    owner = t[16 + 3 * 80: 16 + 3 * 80 + 8 * 4].view(np.uint32)
    assert owner.tolist() == [0, 0, 2, 2, 2, 2, 2, 2]
    rec2 = t[16 + 2 * 80: 16 + 3 * 80]
    assert rec2[:8].view(np.uint64)[0] == 0x40001 and rec2[48:60].view(np.int32).tolist() == [130, 70, 191]
    assert rec2[60:64].view(np.int32)[0] == 3 and rec2[64:68].view(np.uint32)[0] == 2     # tiles along M, first workgroup
    assert rec2[68:72].view(np.int32)[0] == 2                     # unaligned, K >= 64, N >= 4: the overlap fetch
    assert t[16:16 + 80][68:72].view(np.int32)[0] == 1            # aligned, N % 4 == 0, K % 16 == 0: clamped fetch
    bad = P(8, 8, 64, 0x1000, 32, 0x2000, 8, 0x3000, 8)           # lda < K
    assert binding.gemm_i8_grouped_table_bytes([probs[0], bad]) == 0 and b"problem 1" in L.lb_last_error()
    with pytest.raises(binding.LowbitError):
        binding.gemm_i8_grouped_plan([P(8, 8, 2 ** 17, 0x1000, 2 ** 17, 0x2000, 8, 0x3000, 8)])
    assert L.gemm_i8_grouped(0, None, 0, None) == binding.LB_OK
    assert L.gemm_i8_grouped(1, None, 1, None) == binding.LB_EINVAL
    assert L.gemm_i8_grouped(1, 0x1004, 1, None) == binding.LB_EINVAL
    assert L.gemm_i8_grouped(0, 0x1000, 1, None) == binding.LB_EINVAL
    assert L.gemm_i8_grouped(1, 0x1000, 2 ** 31, None) == binding.LB_EOVERFLOW
