"""ctypes binding of liblowbit_gemm.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA (ROCm) tensors; torch provides device memory and the stream, nothing else.  Every
function raises LowbitError when the library returns a status other than LB_OK, and RuntimeError when the
library is missing: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblowbit_gemm.so")

LB_OK, LB_EINVAL, LB_EOVERFLOW, LB_EHIP, LB_EUNSUPPORTED = 0, -1, -2, -3, -4
OP_BNN, OP_TNN, OP_TBN = 0, 1, 2
_OPS = {"bnn": OP_BNN, "tnn": OP_TNN, "tbn": OP_TBN}

EXPORTS = ("lb_last_error", "lb_format_version", "packed_binary_bytes", "packed_ternary_bytes", "pack_binary",
           "pack_ternary", "im2col_packed", "conv_gemm", "gemm_bnn", "gemm_tnn", "gemm_tbn", "gemm_c16", "gemm_grouped_table_bytes",
           "gemm_grouped_plan", "gemm_grouped", "gemm_grouped_static", "gemm_grouped_static_max_bytes", "gemm_requant", "gemm_i8_mfma", "gemm_i8_grouped_table_bytes", "gemm_i8_grouped_plan", "gemm_i8_grouped", "gemm_u8_mfma", "packed_u4_bytes", "pack_u4", "gemm_u4_mfma", "packed_t4_bytes", "pack_t4", "gemm_t4_mfma", "lb_set_variant", "lb_num_variants",
           "lb_variant_name", "lb_describe_plan", "lb_arch_supported", "lb_calib_sink_bytes", "lb_calib_clocks_bytes",
           "lb_calib_wall_clock_khz", "lb_calib_valu_lane_instr", "lb_calib_valu", "lb_calib_stream")


class GemmProblem(ctypes.Structure):
    """lb_gemm_problem of the C header: one product of a grouped launch (device addresses as integers)."""
    _fields_ = [("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("Ap", ctypes.c_void_p),
                ("Bp", ctypes.c_void_p), ("C", ctypes.c_void_p), ("ldc", ctypes.c_int64)]


class I8Problem(ctypes.Structure):
    """lb_i8_problem of the C header: one product of a grouped launch of the 8-bit comparator."""
    _fields_ = [("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("A", ctypes.c_void_p),
                ("lda", ctypes.c_int64), ("B", ctypes.c_void_p), ("ldb", ctypes.c_int64), ("C", ctypes.c_void_p),
                ("ldc", ctypes.c_int64)]


class LowbitError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"lowbit_gemm status {status}: {message}")
        self.status = status


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """The loaded C library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2205_09120_amd.build` "
                               "(there is no fallback implementation)")
        L = ctypes.CDLL(LIB_PATH)
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        L.lb_last_error.restype = ctypes.c_char_p
        L.lb_last_error.argtypes = []
        L.lb_format_version.restype = ci
        L.lb_format_version.argtypes = []
        for f in (L.packed_binary_bytes, L.packed_ternary_bytes):
            f.restype = ctypes.c_size_t
            f.argtypes = [i64, i64]
        for f in (L.pack_binary, L.pack_ternary):
            f.restype = ci
            f.argtypes = [vp, i64, i64, i64, i64, vp, vp]
        for f in (L.gemm_bnn, L.gemm_tnn, L.gemm_tbn):
            f.restype = ci
            f.argtypes = [i64, i64, i64, vp, vp, vp, i64, vp]
        L.gemm_c16.restype = ci
        L.gemm_c16.argtypes = [ci, i64, i64, i64, vp, vp, vp, i64, vp]
        L.gemm_grouped_table_bytes.restype = ctypes.c_size_t
        L.gemm_grouped_table_bytes.argtypes = [ci, i64, vp]
        L.gemm_grouped_plan.restype = ci
        L.gemm_grouped_plan.argtypes = [ci, i64, vp, vp, ctypes.c_size_t, ctypes.POINTER(i64)]
        L.gemm_grouped.restype = ci
        L.gemm_grouped.argtypes = [ci, i64, vp, i64, vp]
        L.gemm_grouped_static_max_bytes.restype = ctypes.c_size_t
        L.gemm_grouped_static_max_bytes.argtypes = []
        L.gemm_grouped_static.restype = ci
        L.gemm_grouped_static.argtypes = [ci, i64, vp, ctypes.c_size_t, i64, vp]
        L.im2col_packed.restype = ci
        L.im2col_packed.argtypes = [vp, ci, i64, i64, i64, i64, ci, ci, ci, ci, ci, ci, vp, vp]
        L.conv_gemm.restype = ci
        L.conv_gemm.argtypes = [ci, i64, vp, vp, i64, i64, i64, i64, ci, ci, ci, ci, ci, ci, vp, i64, vp]
        L.gemm_i8_mfma.restype = ci
        L.gemm_i8_mfma.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, vp]
        L.gemm_i8_grouped_table_bytes.restype = ctypes.c_size_t
        L.gemm_i8_grouped_table_bytes.argtypes = [i64, vp]
        L.gemm_i8_grouped_plan.restype = ci
        L.gemm_i8_grouped_plan.argtypes = [i64, vp, vp, ctypes.c_size_t, ctypes.POINTER(i64)]
        L.gemm_i8_grouped.restype = ci
        L.gemm_i8_grouped.argtypes = [i64, vp, i64, vp]
        L.gemm_requant.restype = ci
        L.gemm_requant.argtypes = [ci, ci, i64, i64, i64, vp, vp, vp, vp, vp, vp]
        L.gemm_u8_mfma.restype = ci
        L.gemm_u8_mfma.argtypes = [i64, i64, i64, vp, i64, vp, i64, ctypes.c_int32, ctypes.c_int32, vp, i64, vp]
        L.packed_u4_bytes.restype = ctypes.c_size_t
        L.packed_u4_bytes.argtypes = [i64, i64]
        L.pack_u4.restype = ci
        L.pack_u4.argtypes = [vp, i64, i64, i64, i64, vp, vp, vp]
        L.gemm_u4_mfma.restype = ci
        L.gemm_u4_mfma.argtypes = [i64, i64, i64, vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32, vp, i64, vp]
        L.packed_t4_bytes.restype = ctypes.c_size_t
        L.packed_t4_bytes.argtypes = [i64, i64]
        L.pack_t4.restype = ci
        L.pack_t4.argtypes = [vp, i64, i64, i64, i64, vp, vp]
        L.gemm_t4_mfma.restype = ci
        L.gemm_t4_mfma.argtypes = [i64, i64, i64, vp, vp, vp, i64, vp]
        L.lb_calib_sink_bytes.restype = ctypes.c_size_t
        L.lb_calib_sink_bytes.argtypes = []
        L.lb_calib_valu_lane_instr.restype = i64
        L.lb_calib_valu_lane_instr.argtypes = [ci, i64, ci]
        L.lb_calib_valu.restype = ci
        L.lb_calib_valu.argtypes = [ci, i64, ci, vp, vp, vp]
        L.lb_calib_clocks_bytes.restype = ctypes.c_size_t
        L.lb_calib_clocks_bytes.argtypes = []
        L.lb_calib_wall_clock_khz.restype = ci
        L.lb_calib_wall_clock_khz.argtypes = []
        L.lb_arch_supported.restype = ci
        L.lb_arch_supported.argtypes = [ctypes.c_char_p]
        L.lb_calib_stream.restype = ci
        L.lb_calib_stream.argtypes = [ci, vp, vp, i64, ci, vp, vp]
        L.lb_set_variant.restype = ci
        L.lb_set_variant.argtypes = [ci, ci]
        L.lb_num_variants.restype = ci
        L.lb_num_variants.argtypes = [ci]
        L.lb_variant_name.restype = ctypes.c_char_p
        L.lb_variant_name.argtypes = [ci, ci]
        L.lb_describe_plan.restype = ctypes.c_char_p
        L.lb_describe_plan.argtypes = [ci, i64, i64, i64, ci]
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != LB_OK:
        raise LowbitError(status, lib().lb_last_error().decode())


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ptr(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None else t.data_ptr()


def lb_last_error() -> str:
    return lib().lb_last_error().decode()


def lb_format_version() -> int:
    return lib().lb_format_version()


def packed_binary_bytes(rows: int, K: int) -> int:
    return lib().packed_binary_bytes(rows, K)


def packed_ternary_bytes(rows: int, K: int) -> int:
    return lib().packed_ternary_bytes(rows, K)


def _pack(fn, nbytes_fn, src, rows, K, stride_r, stride_k, dst, stream):
    if dst is None:
        dst = torch.empty(max(nbytes_fn(rows, K) // 8, 0), dtype=torch.int64, device=src.device)
    _check(fn(_ptr(src), rows, K, stride_r, stride_k, _ptr(dst), _stream(stream)))
    return dst


def pack_binary(src: torch.Tensor, rows: int, K: int, stride_r: int, stride_k: int,
                dst: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Element (r,k) = src.flatten()[r*stride_r + k*stride_k].  Returns dst (int64 words, rows*ceil(K/64))."""
    return _pack(lib().pack_binary, packed_binary_bytes, src, rows, K, stride_r, stride_k, dst, stream)


def pack_ternary(src: torch.Tensor, rows: int, K: int, stride_r: int, stride_k: int,
                 dst: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Returns dst (int64 words, rows*ceil(K/64)*2: plus word, minus word, ...)."""
    return _pack(lib().pack_ternary, packed_ternary_bytes, src, rows, K, stride_r, stride_k, dst, stream)


def im2col_packed(Fp: torch.Tensor, planes: int, batch: int, H: int, W: int, C: int, kh: int, kw: int,
                  stride_h: int = 1, stride_w: int = 1, pad_h: int = 0, pad_w: int = 0,
                  Bp: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Packed right operand (batch*OH*OW strings of depth kh*kw*C) gathered from a channel-packed feature map."""
    if Bp is None:
        OH = (H + 2 * pad_h - kh) // stride_h + 1 if H + 2 * pad_h >= kh else 0
        OW = (W + 2 * pad_w - kw) // stride_w + 1 if W + 2 * pad_w >= kw else 0
        words = batch * OH * OW * kh * kw * (C // 64) * planes
        Bp = torch.empty(max(words, 0), dtype=torch.int64, device=Fp.device)
    _check(lib().im2col_packed(_ptr(Fp), planes, batch, H, W, C, kh, kw, stride_h, stride_w, pad_h, pad_w, _ptr(Bp),
                               _stream(stream)))
    return Bp


def conv_gemm(kind, M: int, Ap: torch.Tensor, Fp: torch.Tensor, batch: int, H: int, W: int, C: int, kh: int, kw: int,
              stride_h: int = 1, stride_w: int = 1, pad_h: int = 0, pad_w: int = 0, Cout: Optional[torch.Tensor] = None,
              ldc: Optional[int] = None, stream=None) -> torch.Tensor:
    """Convolution as an implicit product: (M filters) x (batch*OH*OW output pixels), int32, row-major."""
    OH = (H + 2 * pad_h - kh) // stride_h + 1 if H + 2 * pad_h >= kh else 0
    OW = (W + 2 * pad_w - kw) // stride_w + 1 if W + 2 * pad_w >= kw else 0
    N = batch * OH * OW
    if Cout is None:
        Cout = torch.empty((M, N), dtype=torch.int32, device=Fp.device if Fp is not None else "cuda")
        ldc = max(N, 1)
    elif ldc is None:
        ldc = Cout.stride(0) if Cout.dim() == 2 else N
    _check(lib().conv_gemm(_OPS.get(kind, kind), M, _ptr(Ap), _ptr(Fp), batch, H, W, C, kh, kw, stride_h, stride_w,
                           pad_h, pad_w, _ptr(Cout), ldc, _stream(stream)))
    return Cout


def _gemm(fn, M, N, K, Ap, Bp, C, ldc, stream):
    if C is None:
        C = torch.empty((M, N), dtype=torch.int32, device=Ap.device)
        ldc = N
    elif ldc is None:
        ldc = C.stride(0) if C.dim() == 2 else N
    _check(fn(M, N, K, _ptr(Ap), _ptr(Bp), _ptr(C), ldc, _stream(stream)))
    return C


def gemm_bnn(M, N, K, Ap, Bp, C=None, ldc=None, stream=None):
    return _gemm(lib().gemm_bnn, M, N, K, Ap, Bp, C, ldc, stream)


def gemm_tnn(M, N, K, Ap, Bp, C=None, ldc=None, stream=None):
    return _gemm(lib().gemm_tnn, M, N, K, Ap, Bp, C, ldc, stream)


def gemm_tbn(M, N, K, Ap, Bp, C=None, ldc=None, stream=None):
    return _gemm(lib().gemm_tbn, M, N, K, Ap, Bp, C, ldc, stream)


def gemm_c16(kind, M, N, K, Ap, Bp, C=None, ldc=None, stream=None):
    """gemm_<kind> with a signed 16-bit C (K <= 32767)."""
    if C is None:
        C = torch.empty((M, N), dtype=torch.int16, device=Ap.device)
        ldc = N
    elif ldc is None:
        ldc = C.stride(0) if C.dim() == 2 else N
    _check(lib().gemm_c16(_OPS.get(kind, kind), M, N, K, _ptr(Ap), _ptr(Bp), _ptr(C), ldc, _stream(stream)))
    return C


def gemm_i8_mfma(M, N, K, A, lda, B, ldb, C=None, ldc=None, stream=None):
    if C is None:
        C = torch.empty((M, N), dtype=torch.int32, device=A.device)
        ldc = N
    elif ldc is None:
        ldc = C.stride(0)
    _check(lib().gemm_i8_mfma(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, _stream(stream)))
    return C


def _problem_array(problems: Sequence[GemmProblem]):
    return (GemmProblem * max(len(problems), 1))(*problems)


def gemm_grouped_table_bytes(kind, problems: Sequence[GemmProblem]) -> int:
    """Bytes of the launch table for these problems (0 with lb_last_error() set if they are invalid)."""
    return lib().gemm_grouped_table_bytes(_OPS.get(kind, kind), len(problems), _problem_array(problems))


def gemm_grouped_plan(kind, problems: Sequence[GemmProblem]):
    """Host-side planning: returns (table as a uint8 CPU tensor, workgroups)."""
    arr = _problem_array(problems)
    nbytes = lib().gemm_grouped_table_bytes(_OPS.get(kind, kind), len(problems), arr)
    wg = ctypes.c_int64(0)
    if nbytes == 0:  # invalid problems: let the planning call report which rule they break
        scratch = torch.zeros(16, dtype=torch.uint8)
        _check(lib().gemm_grouped_plan(_OPS.get(kind, kind), len(problems), arr, scratch.data_ptr(), 16,
                                       ctypes.byref(wg)))
        raise LowbitError(LB_EINVAL, "gemm_grouped_table_bytes returned 0")
    table = torch.zeros(nbytes, dtype=torch.uint8)
    _check(lib().gemm_grouped_plan(_OPS.get(kind, kind), len(problems), arr, table.data_ptr(), nbytes,
                                   ctypes.byref(wg)))
    return table, wg.value


def gemm_grouped(kind, count: int, table_dev: Optional[torch.Tensor], workgroups: int, stream=None) -> None:
    """Launch a planned group; table_dev is the device copy of the table gemm_grouped_plan returned."""
    _check(lib().gemm_grouped(_OPS.get(kind, kind), count, _ptr(table_dev), workgroups, _stream(stream)))


def gemm_grouped_static_max_bytes() -> int:
    return lib().gemm_grouped_static_max_bytes()


def gemm_grouped_static(kind, count: int, table_host: Optional[torch.Tensor], workgroups: int, stream=None) -> None:
    """Launch a planned group from its HOST table (uint8 CPU tensor); the device copy lives inside the library."""
    nbytes = 0 if table_host is None else table_host.numel()
    _check(lib().gemm_grouped_static(_OPS.get(kind, kind), count, _ptr(table_host), nbytes, workgroups,
                                     _stream(stream)))


def gemm_i8_grouped_table_bytes(problems: Sequence[I8Problem]) -> int:
    return lib().gemm_i8_grouped_table_bytes(len(problems), (I8Problem * max(len(problems), 1))(*problems))


def gemm_i8_grouped_plan(problems: Sequence[I8Problem]):
    """Host-side planning: returns (table as a uint8 CPU tensor, workgroups)."""
    arr = (I8Problem * max(len(problems), 1))(*problems)
    nbytes = lib().gemm_i8_grouped_table_bytes(len(problems), arr)
    wg = ctypes.c_int64(0)
    if nbytes == 0:  # invalid problems: let the planning call report which rule they break
        scratch = torch.zeros(16, dtype=torch.uint8)
        _check(lib().gemm_i8_grouped_plan(len(problems), arr, scratch.data_ptr(), 16, ctypes.byref(wg)))
        raise LowbitError(LB_EINVAL, "gemm_i8_grouped_table_bytes returned 0")
    table = torch.zeros(nbytes, dtype=torch.uint8)
    _check(lib().gemm_i8_grouped_plan(len(problems), arr, table.data_ptr(), nbytes, ctypes.byref(wg)))
    return table, wg.value


def gemm_i8_grouped(count: int, table_dev: Optional[torch.Tensor], workgroups: int, stream=None) -> None:
    _check(lib().gemm_i8_grouped(count, _ptr(table_dev), workgroups, _stream(stream)))


def gemm_requant(kind, out_planes: int, M, N, K, Ap, Bp, lo, hi=None, Out=None, stream=None):
    """Thresholded product written as N packed strings of depth M (1 = binary, 2 = ternary planes)."""
    if Out is None:
        nbytes = packed_ternary_bytes(N, M) if out_planes == 2 else packed_binary_bytes(N, M)
        Out = torch.empty(nbytes // 8, dtype=torch.int64, device=Ap.device)
    _check(lib().gemm_requant(_OPS.get(kind, kind), out_planes, M, N, K, _ptr(Ap), _ptr(Bp), _ptr(lo), _ptr(hi),
                              _ptr(Out), _stream(stream)))
    return Out


def gemm_u8_mfma(M, N, K, A, lda, B, ldb, zA: int, zB: int, C=None, ldc=None, stream=None):
    """C = sum_t (A - zA)(B - zB) for uint8 A (M x K), B (K x N)."""
    if C is None:
        C = torch.empty((M, N), dtype=torch.int32, device=A.device)
        ldc = N
    elif ldc is None:
        ldc = C.stride(0)
    _check(lib().gemm_u8_mfma(M, N, K, _ptr(A), lda, _ptr(B), ldb, zA, zB, _ptr(C), ldc, _stream(stream)))
    return C


def packed_u4_bytes(rows: int, K: int) -> int:
    return lib().packed_u4_bytes(rows, K)


def pack_u4(src: torch.Tensor, rows: int, K: int, stride_r: int, stride_k: int, dst: Optional[torch.Tensor] = None,
            sums: Optional[torch.Tensor] = None, stream=None):
    """4-bit values (one per byte) -> (packed strings as uint8 vector, int32 row sums)."""
    if dst is None:
        dst = torch.empty(packed_u4_bytes(rows, K), dtype=torch.uint8, device=src.device)
    if sums is None:
        sums = torch.empty(rows, dtype=torch.int32, device=src.device)
    _check(lib().pack_u4(_ptr(src), rows, K, stride_r, stride_k, _ptr(dst), _ptr(sums), _stream(stream)))
    return dst, sums


def gemm_u4_mfma(M, N, K, Ap, sumA, Bp, sumB, zA: int, zB: int, C=None, ldc=None, stream=None):
    """C = sum_t (A - zA)(B - zB) for 4-bit A (M x K), B (K x N) packed by pack_u4."""
    if C is None:
        C = torch.empty((M, N), dtype=torch.int32, device=Ap.device)
        ldc = N
    elif ldc is None:
        ldc = C.stride(0)
    _check(lib().gemm_u4_mfma(M, N, K, _ptr(Ap), _ptr(sumA), _ptr(Bp), _ptr(sumB), zA, zB, _ptr(C), ldc,
                              _stream(stream)))
    return C


def packed_t4_bytes(rows: int, K: int) -> int:
    return lib().packed_t4_bytes(rows, K)


def pack_t4(src: torch.Tensor, rows: int, K: int, stride_r: int, stride_k: int, dst: Optional[torch.Tensor] = None,
            stream=None) -> torch.Tensor:
    """Ternary / binary int8 values -> 4-bit floats in matrix-core fragment order (uint8 vector)."""
    if dst is None:
        dst = torch.empty(packed_t4_bytes(rows, K), dtype=torch.uint8, device=src.device)
    _check(lib().pack_t4(_ptr(src), rows, K, stride_r, stride_k, _ptr(dst), _stream(stream)))
    return dst


def gemm_t4_mfma(M, N, K, Ap, Bp, C=None, ldc=None, stream=None):
    """C = A B for operands packed by pack_t4 (the matrix-core counterpart of gemm_tnn / gemm_tbn / gemm_bnn)."""
    if C is None:
        C = torch.empty((M, N), dtype=torch.int32, device=Ap.device)
        ldc = N
    elif ldc is None:
        ldc = C.stride(0)
    _check(lib().gemm_t4_mfma(M, N, K, _ptr(Ap), _ptr(Bp), _ptr(C), ldc, _stream(stream)))
    return C


def lb_describe_plan(kind, M: int, N: int, K: int, c16: bool = False) -> Optional[str]:
    """Which kernel a gemm call of this shape would run (host logic, no GPU needed)."""
    t = lib().lb_describe_plan(_OPS.get(kind, kind), M, N, K, 1 if c16 else 0)
    return None if t is None else t.decode()


def lb_calib_sink_bytes() -> int:
    return lib().lb_calib_sink_bytes()


def lb_calib_valu_lane_instr(mix: int, iters: int, waves_per_simd: int = 8) -> int:
    return lib().lb_calib_valu_lane_instr(mix, iters, waves_per_simd)


def lb_calib_valu(mix: int, iters: int, sink: torch.Tensor, clocks: Optional[torch.Tensor] = None,
                  waves_per_simd: int = 8, stream=None) -> None:
    _check(lib().lb_calib_valu(mix, iters, waves_per_simd, _ptr(sink), _ptr(clocks), _stream(stream)))


def lb_calib_clocks_bytes() -> int:
    return lib().lb_calib_clocks_bytes()


def lb_calib_wall_clock_khz() -> int:
    return lib().lb_calib_wall_clock_khz()


def lb_arch_supported(arch: str) -> bool:
    return bool(lib().lb_arch_supported(arch.encode()))


def lb_calib_stream(mode: int, src, dst, nbytes: int, sink, blocks: int = 0, stream=None) -> None:
    _check(lib().lb_calib_stream(mode, _ptr(src), _ptr(dst), nbytes, blocks, _ptr(sink), _stream(stream)))


def lb_set_variant(op, variant: int) -> None:
    _check(lib().lb_set_variant(_OPS.get(op, op), variant))


def lb_num_variants(op) -> int:
    return lib().lb_num_variants(_OPS.get(op, op))


def lb_variant_name(op, variant: int) -> Optional[str]:
    s = lib().lb_variant_name(_OPS.get(op, op), variant)
    return None if s is None else s.decode()


# ------------------------------------------------------------------ conveniences built only from the calls above

def pack_a(kind: str, A: torch.Tensor, stream=None) -> torch.Tensor:
    """Pack the left matrix A (M x K, row-major int8) for gemm_<kind>: ternary for tnn/tbn, binary for bnn."""
    M, K = A.shape
    assert A.dtype == torch.int8 and A.stride(1) == 1
    f = pack_binary if kind == "bnn" else pack_ternary
    return f(A, M, K, A.stride(0), 1, stream=stream)


def pack_b(kind: str, B: torch.Tensor, stream=None) -> torch.Tensor:
    """Pack the right matrix B (K x N, row-major int8) along its columns: ternary for tnn, binary otherwise."""
    K, N = B.shape
    assert B.dtype == torch.int8 and B.stride(1) == 1
    f = pack_ternary if kind == "tnn" else pack_binary
    return f(B, N, K, 1, B.stride(0), stream=stream)


class GemmGroup:
    """A planned grouped launch: holds the operands, outputs and the device copy of the launch table."""

    def __init__(self, kind: str, packed_pairs, shapes, Cs=None):
        """packed_pairs: [(Ap, Bp)], shapes: [(M, N, K)]; Cs: optional list of int32 (M, >=N) tensors."""
        self.kind, self.shapes = kind, list(shapes)
        self.operands = list(packed_pairs)
        dev = self.operands[0][0].device if self.operands else torch.device("cuda")
        self.Cs = list(Cs) if Cs is not None else [torch.empty((M, N), dtype=torch.int32, device=dev)
                                                   for (M, N, K) in self.shapes]
        probs = [GemmProblem(M, N, K, _ptr(Ap) or None, _ptr(Bp) or None, _ptr(C) or None,
                             C.stride(0) if C.dim() == 2 and C.numel() else max(N, 1))
                 for (M, N, K), (Ap, Bp), C in zip(self.shapes, self.operands, self.Cs)]
        self.table_host, self.workgroups = gemm_grouped_plan(kind, probs)
        self.table_dev = self.table_host.to(dev)

    def run(self, stream=None):
        gemm_grouped(self.kind, len(self.shapes), self.table_dev, self.workgroups, stream)
        return self.Cs

    def run_static(self, stream=None):
        """The same launch through the entry point that keeps the table in the library's own device array."""
        gemm_grouped_static(self.kind, len(self.shapes), self.table_host, self.workgroups, stream)
        return self.Cs


class I8Group:
    """A planned grouped launch of the 8-bit comparator over unpacked int8 operand pairs."""

    def __init__(self, pairs, shapes, Cs=None):
        """pairs: [(A, B)] int8 device tensors (M x K, K x N, row-major, any row stride); shapes: [(M, N, K)]."""
        self.shapes, self.operands = list(shapes), list(pairs)
        dev = self.operands[0][0].device if self.operands else torch.device("cuda")
        self.Cs = list(Cs) if Cs is not None else [torch.empty((M, N), dtype=torch.int32, device=dev)
                                                   for (M, N, K) in self.shapes]
        probs = [I8Problem(M, N, K, _ptr(A) or None, A.stride(0) if A.dim() == 2 and A.numel() else max(K, 1),
                           _ptr(B) or None, B.stride(0) if B.dim() == 2 and B.numel() else max(N, 1), _ptr(C) or None,
                           C.stride(0) if C.dim() == 2 and C.numel() else max(N, 1))
                 for (M, N, K), (A, B), C in zip(self.shapes, self.operands, self.Cs)]
        table, self.workgroups = gemm_i8_grouped_plan(probs)
        self.table_dev = table.to(dev)

    def run(self, stream=None):
        gemm_i8_grouped(len(self.shapes), self.table_dev, self.workgroups, stream)
        return self.Cs


def gemm(kind: str, M, N, K, Ap, Bp, C=None, ldc=None, stream=None):
    return {"bnn": gemm_bnn, "tnn": gemm_tnn, "tbn": gemm_tbn}[kind](M, N, K, Ap, Bp, C, ldc, stream)
