"""CPU oracle for blockwise NF4 (de)quantisation -- TEST INFRASTRUCTURE ONLY.

A thin numpy/ctypes face over nf4_oracle.c.  Only tests, the smoke check and
the benchmark's CPU-baseline leg may import this package; the GPU library and
its Python binding never do, and this package imports nothing of theirs.

Every function cites the passage of the paper it follows in nf4_oracle.c.
Parity unpinned: dq_encode and dq_encode_group (no external reference for the second-level
encoder; its decoder and invariants are pinned by tests).
"""
import ctypes
import os

import numpy as np

from . import build as _build

FP16, BF16, FP32 = 0, 1, 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        # NF4_ORACLE_LIB: load another build of the oracle instead.  Only the mutation
        # tests set it, to show that a planted mistake makes the pins fail.
        path = os.environ.get("NF4_ORACLE_LIB") or _build.build()
        L = ctypes.CDLL(path)
        c = ctypes
        vp, i64, i32 = c.c_void_p, c.c_int64, c.c_int
        L.nf4o_table.argtypes = [vp]
        L.nf4o_f32_to_f16.argtypes = [c.c_float]
        L.nf4o_f32_to_f16.restype = c.c_uint16
        L.nf4o_f32_to_bf16.argtypes = [c.c_float]
        L.nf4o_f32_to_bf16.restype = c.c_uint16
        L.nf4o_dequantize.argtypes = [vp, vp, i32, i64, vp, i32]
        L.nf4o_dequantize_range.argtypes = [vp, vp, i32, i64, i64, vp, i32]
        L.nf4o_dq_decode.argtypes = [vp, vp, vp, vp, i64, vp]
        L.nf4o_dequantize_dq.argtypes = [vp, vp, vp, vp, vp, i32, i64, vp, i32]
        L.nf4o_quantize.argtypes = [vp, i64, i32, vp, vp]
        L.nf4o_dq_encode.argtypes = [vp, i64, vp, vp, vp, vp]
        L.nf4o_dequant_gemv.argtypes = [vp, vp, vp, vp, vp, i32, i64, i64, vp, i32, vp, vp]
        L.nf4o_dequant_gemv_rows.argtypes = [vp, vp, vp, vp, vp, i32, i64, vp, i32, i64, i64, vp, vp]
        L.nf4o_dequant_gemv_rows.restype = None
        L.nf4o_dequant_gemm_rows.argtypes = [vp, vp, vp, vp, vp, i32, i64, vp, i32, i64, i64, vp, vp]
        L.nf4o_dequant_gemm_rows.restype = None
        L.nf4o_dequantize_codebook.argtypes = [vp, vp, vp, i32, i64, vp, i32]
        L.nf4o_dequantize_dq_codebook.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, i64, vp, i32]
        L.nf4o_quantize_codebook.argtypes = [vp, i64, i32, vp, vp, vp]
        L.nf4o_dq_encode_group.argtypes = [vp, i64, i32, vp, vp, vp, vp]
        L.nf4o_dequant_gemv_rows_codebook.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, i64, vp, i32, i64, i64, i32, vp, vp]
        L.nf4o_dequant_gemv_rows_codebook.restype = None
        for name in ("nf4o_dequantize_codebook", "nf4o_dequantize_dq_codebook", "nf4o_quantize_codebook",
                     "nf4o_dq_encode_group"):
            getattr(L, name).restype = None
        for name in ("nf4o_table", "nf4o_dequantize", "nf4o_dequantize_range", "nf4o_dq_decode",
                     "nf4o_dequantize_dq", "nf4o_quantize", "nf4o_dq_encode", "nf4o_dequant_gemv"):
            getattr(L, name).restype = None
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _chk(a, dtype, size=None, name="array"):
    a = np.ascontiguousarray(a, dtype=dtype)
    if size is not None and a.size < size:
        raise ValueError(f"{name}: need {size} elements, got {a.size}")
    return a


def _out(n, out_dtype):
    return np.empty(n, dtype=np.float32 if out_dtype == FP32 else np.uint16)


def nblocks(n, blocksize=64):
    return (n + blocksize - 1) // blocksize


def table():
    """The 16 NF4 levels as float32 (Sec. II-B)."""
    t = np.empty(16, dtype=np.float32)
    lib().nf4o_table(_p(t))
    return t


def f32_to_f16_bits(values):
    v = np.asarray(values, dtype=np.float32).ravel()
    f = lib().nf4o_f32_to_f16
    return np.fromiter((f(float(x)) for x in v), dtype=np.uint16, count=v.size)


def f32_to_bf16_bits(values):
    v = np.asarray(values, dtype=np.float32).ravel()
    f = lib().nf4o_f32_to_bf16
    return np.fromiter((f(float(x)) for x in v), dtype=np.uint16, count=v.size)


def quantize(src, blocksize=64):
    """float32[n] -> (packed uint8[ceil(n/2)], absmax float32[ceil(n/bs)])."""
    src = _chk(src, np.float32).ravel()
    n = src.size
    packed = np.zeros((n + 1) // 2, dtype=np.uint8)
    absmax = np.zeros(nblocks(n, blocksize), dtype=np.float32)
    lib().nf4o_quantize(_p(src), n, blocksize, _p(packed), _p(absmax))
    return packed, absmax


def dequantize(packed, absmax, n, blocksize=64, out_dtype=FP16):
    """Returns uint16 bit patterns (fp16 / bf16) or float32 for FP32."""
    packed = _chk(packed, np.uint8, (n + 1) // 2, "packed")
    absmax = _chk(absmax, np.float32, nblocks(n, blocksize), "absmax")
    out = _out(n, out_dtype)
    lib().nf4o_dequantize(_p(packed), _p(absmax), blocksize, n, _p(out), out_dtype)
    return out


def dequantize_range(packed, absmax, first, count, out, blocksize=64, out_dtype=FP16):
    """Fill out[first:first+count] in place (lets a caller split over threads)."""
    lib().nf4o_dequantize_range(_p(packed), _p(absmax), blocksize, first, count, _p(out), out_dtype)


def dq_encode(absmax):
    """float32[nb] -> (q8 uint8[nb], scale2 float32[ceil(nb/256)], offset float32[1], code2 float32[256])."""
    absmax = _chk(absmax, np.float32).ravel()
    nb = absmax.size
    q8 = np.zeros(nb, dtype=np.uint8)
    scale2 = np.zeros((nb + 255) // 256, dtype=np.float32)
    offset = np.zeros(1, dtype=np.float32)
    code2 = np.zeros(256, dtype=np.float32)
    lib().nf4o_dq_encode(_p(absmax), nb, _p(q8), _p(scale2), _p(offset), _p(code2))
    return q8, scale2, offset, code2


def dq_decode(q8, scale2, offset, code2):
    q8 = _chk(q8, np.uint8).ravel()
    nb = q8.size
    scale2 = _chk(scale2, np.float32, (nb + 255) // 256, "scale2")
    offset = _chk(offset, np.float32, 1, "offset")
    code2 = _chk(code2, np.float32, 256, "code2")
    absmax = np.empty(nb, dtype=np.float32)
    lib().nf4o_dq_decode(_p(q8), _p(scale2), _p(offset), _p(code2), nb, _p(absmax))
    return absmax


def dequantize_dq(packed, q8, scale2, offset, code2, n, blocksize=64, out_dtype=FP16):
    nb = nblocks(n, blocksize)
    packed = _chk(packed, np.uint8, (n + 1) // 2, "packed")
    q8 = _chk(q8, np.uint8, nb, "absmax_q8")
    scale2 = _chk(scale2, np.float32, (nb + 255) // 256, "scale2")
    offset = _chk(offset, np.float32, 1, "offset")
    code2 = _chk(code2, np.float32, 256, "code2")
    out = _out(n, out_dtype)
    lib().nf4o_dequantize_dq(_p(packed), _p(q8), _p(scale2), _p(offset), _p(code2), blocksize, n,
                             _p(out), out_dtype)
    return out


def dequant_gemv(packed, q8, scale2, offset, code2, N, K, x_bits, blocksize=64):
    """x_bits: uint16[B][K] fp16 patterns.  Returns (y_bits uint16[B][N], y float64[B][N])."""
    x_bits = _chk(x_bits, np.uint16)
    B = x_bits.size // K
    n = N * K
    nb = nblocks(n, blocksize)
    packed = _chk(packed, np.uint8, (n + 1) // 2, "packed")
    q8 = _chk(q8, np.uint8, nb, "absmax_q8")
    scale2 = _chk(scale2, np.float32, (nb + 255) // 256, "scale2")
    offset = _chk(offset, np.float32, 1, "offset")
    code2 = _chk(code2, np.float32, 256, "code2")
    y = np.empty((B, N), dtype=np.uint16)
    y64 = np.empty((B, N), dtype=np.float64)
    lib().nf4o_dequant_gemv(_p(packed), _p(q8), _p(scale2), _p(offset), _p(code2), blocksize, N, K,
                            _p(x_bits), B, _p(y), _p(y64))
    return y, y64


def dequant_gemv_rows(packed, q8, scale2, offset, code2, N, K, x_bits, r_first, r_count, blocksize=64):
    """Rows [r_first, r_first + r_count) of dequant_gemv: (y_bits uint16[B][r_count], y float64[B][r_count])."""
    x_bits = _chk(x_bits, np.uint16)
    B = x_bits.size // K
    n = N * K
    nb = nblocks(n, blocksize)
    packed = _chk(packed, np.uint8, (n + 1) // 2, "packed")
    q8 = _chk(q8, np.uint8, nb, "absmax_q8")
    scale2 = _chk(scale2, np.float32, (nb + 255) // 256, "scale2")
    offset = _chk(offset, np.float32, 1, "offset")
    code2 = _chk(code2, np.float32, 256, "code2")
    if r_first < 0 or r_first + r_count > N:
        raise ValueError("row range outside the matrix")
    y = np.empty((B, r_count), dtype=np.uint16)
    y64 = np.empty((B, r_count), dtype=np.float64)
    lib().nf4o_dequant_gemv_rows(_p(packed), _p(q8), _p(scale2), _p(offset), _p(code2), blocksize, K,
                                 _p(x_bits), B, r_first, r_count, _p(y), _p(y64))
    return y, y64


def dequant_gemm_rows(packed, q8, scale2, offset, code2, N, K, x_bits, r_first, r_count, blocksize=64):
    """Like dequant_gemv_rows with every weight rounded to fp16 first (the dequantise-then-matmul flow)."""
    x_bits = _chk(x_bits, np.uint16)
    B = x_bits.size // K
    n = N * K
    nb = nblocks(n, blocksize)
    packed = _chk(packed, np.uint8, (n + 1) // 2, "packed")
    q8 = _chk(q8, np.uint8, nb, "absmax_q8")
    scale2 = _chk(scale2, np.float32, (nb + 255) // 256, "scale2")
    offset = _chk(offset, np.float32, 1, "offset")
    code2 = _chk(code2, np.float32, 256, "code2")
    if r_first < 0 or r_first + r_count > N:
        raise ValueError("row range outside the matrix")
    y = np.empty((B, r_count), dtype=np.uint16)
    y64 = np.empty((B, r_count), dtype=np.float64)
    lib().nf4o_dequant_gemm_rows(_p(packed), _p(q8), _p(scale2), _p(offset), _p(code2), blocksize, K,
                                 _p(x_bits), B, r_first, r_count, _p(y), _p(y64))
    return y, y64


# ---- the data type as a parameter (Sec. V-A): any 16 levels, any second-level group size ----

def quantize_codebook(src, codebook, blocksize=64):
    src = _chk(src, np.float32).ravel()
    codebook = _chk(codebook, np.float32, 16, "codebook")
    n = src.size
    packed = np.zeros((n + 1) // 2, dtype=np.uint8)
    absmax = np.zeros(nblocks(n, blocksize), dtype=np.float32)
    lib().nf4o_quantize_codebook(_p(src), n, blocksize, _p(codebook), _p(packed), _p(absmax))
    return packed, absmax


def dequantize_codebook(packed, absmax, codebook, n, blocksize=64, out_dtype=FP16):
    packed = _chk(packed, np.uint8, (n + 1) // 2, "packed")
    absmax = _chk(absmax, np.float32, nblocks(n, blocksize), "absmax")
    codebook = _chk(codebook, np.float32, 16, "codebook")
    out = _out(n, out_dtype)
    lib().nf4o_dequantize_codebook(_p(packed), _p(absmax), _p(codebook), blocksize, n, _p(out), out_dtype)
    return out


def dq_encode_group(absmax, group):
    """float32[nb] -> (q8 uint8[nb], scale2 float32[ceil(nb/group)], offset float32[1], code2 float32[256])."""
    absmax = _chk(absmax, np.float32).ravel()
    nb = absmax.size
    q8 = np.zeros(nb, dtype=np.uint8)
    scale2 = np.zeros((nb + group - 1) // group, dtype=np.float32)
    offset = np.zeros(1, dtype=np.float32)
    code2 = np.zeros(256, dtype=np.float32)
    lib().nf4o_dq_encode_group(_p(absmax), nb, group, _p(q8), _p(scale2), _p(offset), _p(code2))
    return q8, scale2, offset, code2


def dequantize_dq_codebook(packed, q8, scale2, offset, code2, group, codebook, n, blocksize=64, out_dtype=FP16):
    nb = nblocks(n, blocksize)
    packed = _chk(packed, np.uint8, (n + 1) // 2, "packed")
    q8 = _chk(q8, np.uint8, nb, "absmax_q8")
    scale2 = _chk(scale2, np.float32, (nb + group - 1) // group, "scale2")
    offset = _chk(offset, np.float32, 1, "offset")
    code2 = _chk(code2, np.float32, 256, "code2")
    codebook = _chk(codebook, np.float32, 16, "codebook")
    out = _out(n, out_dtype)
    lib().nf4o_dequantize_dq_codebook(_p(packed), _p(q8), _p(scale2), _p(offset), _p(code2), group, _p(codebook),
                                      blocksize, n, _p(out), out_dtype)
    return out


def dequant_gemv_rows_codebook(packed, q8, scale2, offset, code2, group, codebook, N, K, x_bits, r_first, r_count,
                               blocksize=64, round_weights_to_fp16=False):
    """dequant_gemv_rows (or, with round_weights_to_fp16, dequant_gemm_rows) for any 16 levels and any number of
    blocks per second-level scale: (y_bits uint16[B][r_count], y float64[B][r_count])."""
    x_bits = _chk(x_bits, np.uint16)
    B = x_bits.size // K
    n = N * K
    nb = nblocks(n, blocksize)
    packed = _chk(packed, np.uint8, (n + 1) // 2, "packed")
    q8 = _chk(q8, np.uint8, nb, "absmax_q8")
    scale2 = _chk(scale2, np.float32, (nb + group - 1) // group, "scale2")
    offset = _chk(offset, np.float32, 1, "offset")
    code2 = _chk(code2, np.float32, 256, "code2")
    codebook = _chk(codebook, np.float32, 16, "codebook")
    if r_first < 0 or r_first + r_count > N:
        raise ValueError("row range outside the matrix")
    y = np.empty((B, r_count), dtype=np.uint16)
    y64 = np.empty((B, r_count), dtype=np.float64)
    lib().nf4o_dequant_gemv_rows_codebook(_p(packed), _p(q8), _p(scale2), _p(offset), _p(code2), group, _p(codebook),
                                          blocksize, K, _p(x_bits), B, r_first, r_count,
                                          1 if round_weights_to_fp16 else 0, _p(y), _p(y64))
    return y, y64
