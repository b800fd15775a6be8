"""Thin Python face of libnf4 (include/nf4.h): same names, argument marshalling
only.  torch supplies device memory and streams; every step of the computation
runs in the HIP kernels.  There is no fallback: if the library has not been
built, or a call returns an error status, this raises.
"""
import ctypes
import os

import torch

from . import build as _build

NF4_FP16, NF4_BF16 = 0, 1
_DTYPE_CODE = {torch.float16: NF4_FP16, torch.bfloat16: NF4_BF16}

_lib = None

NF4_BATCH_MAX = 8


class Nf4Tensor(ctypes.Structure):
    """nf4_tensor of include/nf4.h: one tensor of a batched dequantisation (device addresses)."""
    _fields_ = [("packed", ctypes.c_void_p), ("absmax", ctypes.c_void_p), ("absmax_q8", ctypes.c_void_p),
                ("scale2", ctypes.c_void_p), ("offset", ctypes.c_void_p), ("code2", ctypes.c_void_p),
                ("out", ctypes.c_void_p), ("n", ctypes.c_int64)]


class NF4Error(RuntimeError):
    def __init__(self, status, name, hip_error=0):
        self.status, self.hip_error = status, hip_error
        extra = f" (hipError_t {hip_error})" if hip_error else ""
        super().__init__(f"libnf4: {name}{extra}")


def lib():
    """Load libnf4.so (built in-tree by paper_2604_02556_amd.build); never builds."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.lib_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: run `python -m paper_2604_02556_amd.build` "
                           "(or __graft_entry__.build()) first; there is no CPU fallback")
    L = ctypes.CDLL(path)
    c = ctypes
    vp, i64, i32 = c.c_void_p, c.c_int64, c.c_int
    L.nf4_dequantize.argtypes = [vp, vp, i32, i64, vp, i32, vp]
    L.nf4_dequantize_dq.argtypes = [vp, vp, vp, vp, vp, i32, i64, vp, i32, vp]
    L.nf4_dequant_gemv.argtypes = [vp, vp, vp, vp, vp, i32, i64, i64, vp, i32, vp, vp]
    L.nf4_dequantize_batch.argtypes = [c.POINTER(Nf4Tensor), i32, i32, i32, vp]
    L.nf4_dequant_gemm.argtypes = [vp, vp, vp, vp, vp, i32, i64, i64, vp, i32, vp, vp, c.c_size_t, vp]
    L.nf4_dequant_gemm.restype = i32
    L.nf4_dequant_gemm_workspace_bytes.argtypes = [i64, i64, i32]
    L.nf4_dequant_gemm_workspace_bytes.restype = c.c_size_t
    L.nf4_dequant_gemv_ws.argtypes = [vp, vp, vp, vp, vp, i32, i64, i64, vp, i32, vp, vp, c.c_size_t, vp]
    L.nf4_dequant_gemv_ws.restype = i32
    L.nf4_dequant_gemv_workspace_bytes.argtypes = [i64, i64, i32]
    L.nf4_dequant_gemv_static.argtypes = [vp, vp, vp, vp, vp, i32, i64, i64, vp, i32, vp, vp]
    L.nf4_dequant_gemv_static.restype = i32
    L.nf4_dequant_gemv_workspace_bytes.restype = c.c_size_t
    for f in (L.nf4_dequant_gemv_codebook, L.nf4_dequant_gemm_codebook):
        f.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, i64, i64, vp, i32, vp, vp, c.c_size_t, vp]
        f.restype = i32
    L.nf4_quantize_ref.argtypes = [vp, i64, i32, vp, vp, vp, vp, vp, vp, vp]
    L.nf4_dequantize_codebook.argtypes = [vp, vp, vp, i32, i64, vp, i32, vp]
    L.nf4_dequantize_dq_codebook.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, i64, vp, i32, vp]
    L.nf4_quantize_ref_codebook.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, vp, vp, vp, vp]
    for f in (L.nf4_dequantize_codebook, L.nf4_dequantize_dq_codebook, L.nf4_quantize_ref_codebook):
        f.restype = i32
    L.nf4_quantize.argtypes = [vp, i64, i32, vp, vp, vp]
    L.nf4_quantize_codebook.argtypes = [vp, i64, i32, vp, vp, vp, vp, c.c_size_t, vp]
    L.nf4_quantize_codebook.restype = i32
    L.nf4_dq_encode.argtypes = [vp, i64, i32, vp, vp, vp, vp, vp]
    for f in (L.nf4_dequantize, L.nf4_dequantize_dq, L.nf4_dequant_gemv, L.nf4_quantize_ref, L.nf4_quantize,
              L.nf4_last_hip_error):
        f.restype = i32
    L.nf4_last_hip_error.argtypes = []
    L.nf4_status_string.argtypes = [i32]
    L.nf4_status_string.restype = c.c_char_p
    _lib = L
    return L


def status_string(status):
    return lib().nf4_status_string(int(status)).decode()


def _check(status):
    if status != 0:
        L = lib()
        raise NF4Error(status, status_string(status), L.nf4_last_hip_error() if status == 7 else 0)


def _ptr(t):
    """Device address of a tensor (None -> NULL).  Raw ints pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("libnf4 takes contiguous tensors")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def nf4_dequantize(packed, absmax, blocksize, n, out, stream=None):
    """out[i] = rne16(level[code(i)] * absmax[i // blocksize]); out is fp16 or bf16 (its dtype picks)."""
    _check(lib().nf4_dequantize(_ptr(packed), _ptr(absmax), blocksize, n, _ptr(out),
                                _DTYPE_CODE[out.dtype], _stream(stream)))
    return out


def nf4_dequantize_dq(packed, absmax_q8, scale2, offset, code2, blocksize, n, out, stream=None):
    _check(lib().nf4_dequantize_dq(_ptr(packed), _ptr(absmax_q8), _ptr(scale2), _ptr(offset), _ptr(code2),
                                   blocksize, n, _ptr(out), _DTYPE_CODE[out.dtype], _stream(stream)))
    return out


def nf4_dequantize_codebook(packed, absmax, codebook, blocksize, n, out, stream=None):
    """nf4_dequantize with the caller's 16 levels (a float32 device tensor; None = NF4)."""
    _check(lib().nf4_dequantize_codebook(_ptr(packed), _ptr(absmax), _ptr(codebook), blocksize, n, _ptr(out),
                                         _DTYPE_CODE[out.dtype], _stream(stream)))
    return out


def nf4_dequantize_dq_codebook(packed, absmax_q8, scale2, offset, code2, dq_group, codebook, blocksize, n, out,
                               stream=None):
    _check(lib().nf4_dequantize_dq_codebook(_ptr(packed), _ptr(absmax_q8), _ptr(scale2), _ptr(offset), _ptr(code2),
                                            dq_group, _ptr(codebook), blocksize, n, _ptr(out),
                                            _DTYPE_CODE[out.dtype], _stream(stream)))
    return out


def nf4_quantize_ref_codebook(src, n, blocksize, codebook, dq_group, packed, absmax, absmax_q8=None, scale2=None,
                              offset=None, code2=None, stream=None):
    _check(lib().nf4_quantize_ref_codebook(_ptr(src), n, blocksize, _ptr(codebook), dq_group, _ptr(packed),
                                           _ptr(absmax), _ptr(absmax_q8), _ptr(scale2), _ptr(offset), _ptr(code2),
                                           _stream(stream)))


def nf4_dequantize_batch(tensors, blocksize, stream=None):
    """One launch for up to NF4_BATCH_MAX tensors.  tensors: dicts with packed, out (a torch tensor whose dtype
    picks FP16 or BF16, the same for all), n, and either absmax or absmax_q8 + scale2 + offset + code2."""
    items = (Nf4Tensor * max(len(tensors), 1))()
    dtypes = set()
    for it, t in zip(items, tensors):
        it.packed, it.absmax = _ptr(t["packed"]), _ptr(t.get("absmax"))
        it.absmax_q8, it.scale2 = _ptr(t.get("absmax_q8")), _ptr(t.get("scale2"))
        it.offset, it.code2 = _ptr(t.get("offset")), _ptr(t.get("code2"))
        it.out, it.n = _ptr(t["out"]), t["n"]
        dtypes.add(t["out"].dtype)
    if len(dtypes) > 1:
        raise ValueError("all outputs of a batch must have one dtype")
    dt = _DTYPE_CODE[next(iter(dtypes))] if dtypes else NF4_FP16
    _check(lib().nf4_dequantize_batch(items, len(tensors), blocksize, dt, _stream(stream)))


def nf4_dequant_gemv(packed, absmax_q8, scale2, offset, code2, blocksize, N, K, x, B, y, stream=None):
    _check(lib().nf4_dequant_gemv(_ptr(packed), _ptr(absmax_q8), _ptr(scale2), _ptr(offset), _ptr(code2),
                                  blocksize, N, K, _ptr(x), B, _ptr(y), _stream(stream)))
    return y


def nf4_dequant_gemv_ws(packed, absmax_q8, scale2, offset, code2, blocksize, N, K, x, B, y, workspace, stream=None):
    """workspace: a device tensor of at least nf4_dequant_gemv_workspace_bytes(N, K, B) bytes."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().nf4_dequant_gemv_ws(_ptr(packed), _ptr(absmax_q8), _ptr(scale2), _ptr(offset), _ptr(code2),
                                     blocksize, N, K, _ptr(x), B, _ptr(y), _ptr(workspace), ws_bytes,
                                     _stream(stream)))
    return y


def nf4_dequant_gemv_static(packed, absmax_q8, scale2, offset, code2, blocksize, N, K, x, B, y, stream=None):
    """nf4_dequant_gemv_ws over the library's own static scratch array: allocates nothing."""
    _check(lib().nf4_dequant_gemv_static(_ptr(packed), _ptr(absmax_q8), _ptr(scale2), _ptr(offset), _ptr(code2),
                                         blocksize, N, K, _ptr(x), B, _ptr(y), _stream(stream)))
    return y


def nf4_dequant_gemv_workspace_bytes(N, K, B):
    return int(lib().nf4_dequant_gemv_workspace_bytes(N, K, B))


def nf4_dequant_gemm(packed, absmax_q8, scale2, offset, code2, blocksize, N, K, x, B, y, workspace=None,
                     stream=None):
    """workspace: a device tensor of at least nf4_dequant_gemm_workspace_bytes(N, K, B) bytes, or None."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().nf4_dequant_gemm(_ptr(packed), _ptr(absmax_q8), _ptr(scale2), _ptr(offset), _ptr(code2),
                                  blocksize, N, K, _ptr(x), B, _ptr(y), _ptr(workspace), ws_bytes,
                                  _stream(stream)))
    return y


def nf4_dequant_gemv_codebook(packed, absmax_q8, scale2, offset, code2, dq_group, codebook, blocksize, N, K, x, B, y,
                              workspace=None, stream=None):
    """nf4_dequant_gemv (workspace None) or nf4_dequant_gemv_ws for any 16 levels and second-level group size."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().nf4_dequant_gemv_codebook(_ptr(packed), _ptr(absmax_q8), _ptr(scale2), _ptr(offset), _ptr(code2),
                                           dq_group, _ptr(codebook), blocksize, N, K, _ptr(x), B, _ptr(y),
                                           _ptr(workspace), ws_bytes, _stream(stream)))
    return y


def nf4_dequant_gemm_codebook(packed, absmax_q8, scale2, offset, code2, dq_group, codebook, blocksize, N, K, x, B, y,
                              workspace=None, stream=None):
    """nf4_dequant_gemm for any 16 levels and second-level group size."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().nf4_dequant_gemm_codebook(_ptr(packed), _ptr(absmax_q8), _ptr(scale2), _ptr(offset), _ptr(code2),
                                           dq_group, _ptr(codebook), blocksize, N, K, _ptr(x), B, _ptr(y),
                                           _ptr(workspace), ws_bytes, _stream(stream)))
    return y


def nf4_dequant_gemm_workspace_bytes(N, K, B):
    return int(lib().nf4_dequant_gemm_workspace_bytes(N, K, B))


def nf4_quantize_ref(src, n, blocksize, packed, absmax, absmax_q8=None, scale2=None, offset=None,
                     code2=None, stream=None):
    _check(lib().nf4_quantize_ref(_ptr(src), n, blocksize, _ptr(packed), _ptr(absmax), _ptr(absmax_q8),
                                  _ptr(scale2), _ptr(offset), _ptr(code2), _stream(stream)))


def nf4_dq_encode(absmax, nb, dq_group, absmax_q8, scale2, offset, code2, stream=None):
    _check(lib().nf4_dq_encode(_ptr(absmax), nb, dq_group, _ptr(absmax_q8), _ptr(scale2), _ptr(offset), _ptr(code2),
                               _stream(stream)))


def nf4_quantize(src, n, blocksize, packed, absmax, stream=None):
    _check(lib().nf4_quantize(_ptr(src), n, blocksize, _ptr(packed), _ptr(absmax), _stream(stream)))


QUANTIZE_CODEBOOK_WORKSPACE_BYTES = 1024         # NF4_QUANTIZE_CODEBOOK_WORKSPACE_BYTES of include/nf4.h


def nf4_quantize_codebook(src, n, blocksize, codebook, packed, absmax, workspace, stream=None):
    _check(lib().nf4_quantize_codebook(_ptr(src), n, blocksize, _ptr(codebook), _ptr(packed), _ptr(absmax),
                                       _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
                                       _stream(stream)))


# ---- allocation helpers (plumbing only: sizes of the format's arrays) ----

def alloc_quantized(n, blocksize=64, dq=False, device="cuda", dq_group=256):
    """Empty device buffers for a tensor of n elements: dict of packed, absmax and (dq) q8/scale2/offset/code2."""
    nb = (n + blocksize - 1) // blocksize
    bufs = {
        "packed": torch.empty(max((n + 1) // 2, 1), dtype=torch.uint8, device=device),
        "absmax": torch.empty(max(nb, 1), dtype=torch.float32, device=device),
    }
    if dq:
        bufs["absmax_q8"] = torch.empty(max(nb, 1), dtype=torch.uint8, device=device)
        bufs["scale2"] = torch.empty(max((nb + dq_group - 1) // dq_group, 1), dtype=torch.float32, device=device)
        bufs["offset"] = torch.empty(1, dtype=torch.float32, device=device)
        bufs["code2"] = torch.empty(256, dtype=torch.float32, device=device)
    return bufs
