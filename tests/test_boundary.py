"""Host-side checks of the C-ABI: the library loads, exports what include/nf4.h
declares, and rejects bad arguments before launching anything (so these run
without a GPU)."""
import os
import re

import pytest

from paper_2604_02556_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "nf4.h")

OK, E_NULL, E_SIZE, E_BS, E_DT, E_ALIGN, E_SHAPE, E_HIP = range(8)
P = 4096          # a well-aligned fake device address; never dereferenced on these paths


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(build.lib_path()):
        build.build()
    return binding.lib()


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return re.findall(r"\b(nf4_[a-z0-9_]+)\s*\(", text)


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert set(names) >= {"nf4_dequantize", "nf4_dequantize_dq", "nf4_dequant_gemv", "nf4_quantize_ref",
                          "nf4_quantize", "nf4_quantize_codebook", "nf4_dq_encode", "nf4_dequant_gemm", "nf4_dequant_gemm_workspace_bytes", "nf4_dequantize_batch", "nf4_dequantize_codebook",
                          "nf4_dequant_gemv_ws", "nf4_dequant_gemv_workspace_bytes",
                          "nf4_dequantize_dq_codebook", "nf4_quantize_ref_codebook", "nf4_last_hip_error", "nf4_status_string"}
    for name in names:
        assert hasattr(L, name), name


def test_status_strings(L):
    names = ["NF4_OK", "NF4_ERR_NULL", "NF4_ERR_SIZE", "NF4_ERR_BLOCKSIZE", "NF4_ERR_DTYPE", "NF4_ERR_ALIGN",
             "NF4_ERR_SHAPE", "NF4_ERR_HIP"]
    for code, name in enumerate(names):
        assert binding.status_string(code) == name
    assert binding.status_string(99) == "NF4_ERR_UNKNOWN"
    assert L.nf4_last_hip_error() == 0


def test_dequantize_argument_checks(L):
    f = L.nf4_dequantize
    assert f(P, P, 64, -1, P, 0, None) == E_SIZE
    for bs in (0, 32, 63, 96, 8192, -64):
        assert f(P, P, bs, 10, P, 0, None) == E_BS
    assert f(P, P, 64, 10, P, 2, None) == E_DT
    assert f(None, None, 64, 0, None, 0, None) == OK            # empty tensor: nothing to do
    assert f(None, P, 64, 10, P, 0, None) == E_NULL
    assert f(P, None, 64, 10, P, 0, None) == E_NULL
    assert f(P, P, 64, 10, None, 1, None) == E_NULL
    assert f(P + 8, P, 64, 10, P, 0, None) == E_ALIGN
    assert f(P, P + 2, 64, 10, P, 0, None) == E_ALIGN
    assert f(P, P, 64, 10, P + 2, 0, None) == E_ALIGN


def test_dequantize_dq_argument_checks(L):
    f = L.nf4_dequantize_dq
    assert f(P, P, P, P, P, 64, -5, P, 0, None) == E_SIZE
    assert f(P, P, P, P, P, 100, 5, P, 0, None) == E_BS
    assert f(P, P, P, P, P, 64, 5, P, 7, None) == E_DT
    assert f(None, None, None, None, None, 64, 0, None, 1, None) == OK
    for hole in range(5):
        args = [P] * 5
        args[hole] = None
        assert f(*args, 64, 5, P, 0, None) == E_NULL
    assert f(P, P + 1, P + 2, P, P, 64, 5, P, 0, None) == E_ALIGN     # q8 may be odd, scale2 may not
    assert f(P, P + 1, P, P, P, 64, 5, P + 4, 0, None) == E_ALIGN


def test_gemv_argument_checks(L):
    f = L.nf4_dequant_gemv
    a = [P] * 5
    assert f(*a, 64, -1, 64, P, 1, P, None) == E_SIZE
    assert f(*a, 48, 4, 64, P, 1, P, None) == E_BS
    assert f(*a, 64, 4, 64, P, 0, P, None) == E_SHAPE
    assert f(*a, 64, 4, 64, P, 17, P, None) == E_SHAPE
    assert f(*a, 64, 4, 96, P, 1, P, None) == E_SHAPE
    assert f(*a, 64, 4, 0, P, 1, P, None) == E_SHAPE
    assert f(*a, 64, 0, 64, P, 1, P, None) == OK
    assert f(*a, 64, 4, 64, None, 1, P, None) == E_NULL
    assert f(*a, 64, 4, 64, P, 1, None, None) == E_NULL
    assert f(*a, 64, 4, 64, P + 2, 1, P, None) == E_ALIGN
    assert f(*a, 64, 4, 64, P, 1, P + 1, None) == E_ALIGN


def test_gemm_argument_checks(L):
    f = L.nf4_dequant_gemm
    a = [P] * 5
    for ws in ((None, 0), (P, 1 << 40)):
        assert f(*a, 64, -1, 64, P, 1, P, *ws, None) == E_SIZE
        assert f(*a, 48, 4, 64, P, 1, P, *ws, None) == E_BS
        assert f(*a, 64, 4, 64, P, 0, P, *ws, None) == E_SHAPE
        assert f(*a, 64, 4, 64, P, 65, P, *ws, None) == E_SHAPE
        assert f(*a, 64, 4, 96, P, 1, P, *ws, None) == E_SHAPE
        assert f(*a, 64, 0, 64, P, 1, P, *ws, None) == OK
        assert f(*a, 64, 4, 64, None, 1, P, *ws, None) == E_NULL
        assert f(*a, 64, 4, 64, P, 1, None, *ws, None) == E_NULL
        assert f(*a, 64, 4, 64, P + 2, 1, P, *ws, None) == E_ALIGN
    # a workspace that is misaligned or smaller than the split needs is refused before any launch
    assert f(*a, 64, 4, 64, P, 1, P, P + 4, 1 << 40, None) == E_ALIGN
    need = L.nf4_dequant_gemm_workspace_bytes(4096, 8192, 64)
    assert need >= 2 * 64 * 4096 * 4                      # at least two splits of FP32 partial sums
    assert f(*a, 64, 4096, 8192, P, 64, P, P, need - 1, None) == E_SIZE


def test_dequantize_batch_argument_checks(L):
    T = binding.Nf4Tensor

    def call(items, count=None, bs=64, dt=0):
        arr = (T * max(len(items), 1))(*items)
        return L.nf4_dequantize_batch(arr, len(items) if count is None else count, bs, dt, None)
    fp32 = lambda n=5, packed=P, absmax=P, out=P: T(packed, absmax, None, None, None, None, out, n)
    dq = lambda n=5, q8=P, s2=P, off=P, c2=P: T(P, None, q8, s2, off, c2, P, n)
    assert call([]) == OK
    assert L.nf4_dequantize_batch(None, 0, 64, 0, None) == OK
    assert L.nf4_dequantize_batch(None, 2, 64, 0, None) == E_NULL
    assert call([fp32()], count=-1) == E_SIZE
    assert call([fp32()], count=binding.NF4_BATCH_MAX + 1) == E_SIZE
    assert call([fp32()], bs=48) == E_BS
    assert call([fp32()], dt=2) == E_DT
    assert call([fp32(n=-1)]) == E_SIZE
    assert call([fp32(n=0), fp32(n=0, packed=None, out=None)]) == OK      # empty tensors are skipped unchecked
    assert call([fp32(packed=None)]) == E_NULL
    assert call([fp32(out=None)]) == E_NULL
    assert call([fp32(out=P + 2)]) == E_ALIGN
    assert call([fp32(packed=P + 8)]) == E_ALIGN
    assert call([fp32(absmax=P + 2)]) == E_ALIGN
    assert call([dq(q8=None)]) == E_NULL
    assert call([dq(c2=None)]) == E_NULL
    assert call([dq(s2=P + 1)]) == E_ALIGN
    assert call([fp32(n=0), fp32(), dq()]) == E_SHAPE                      # two kinds of scales in one call


def test_gemv_with_workspace_argument_checks(L):
    f = L.nf4_dequant_gemv_ws
    a = [P] * 5
    big = 1 << 40
    assert f(*a, 64, -1, 64, P, 1, P, P, big, None) == E_SIZE
    assert f(*a, 48, 4, 64, P, 1, P, P, big, None) == E_BS
    assert f(*a, 64, 4, 64, P, 0, P, P, big, None) == E_SHAPE
    assert f(*a, 64, 4, 64, P, 17, P, P, big, None) == E_SHAPE
    assert f(*a, 64, 4, 96, P, 1, P, P, big, None) == E_SHAPE
    assert f(*a, 64, 0, 64, P, 1, P, P, big, None) == OK              # no rows: nothing to do
    assert f(*a, 64, 4, 64, None, 1, P, P, big, None) == E_NULL
    assert f(*a, 64, 4, 64, P, 1, None, P, big, None) == E_NULL
    assert f(*a, 64, 4, 64, P, 1, P, None, 0, None) == E_NULL         # the workspace is not optional here
    assert f(*a, 64, 4, 64, P + 2, 1, P, P, big, None) == E_ALIGN
    assert f(*a, 64, 4, 64, P, 1, P, P + 4, big, None) == E_ALIGN
    need = L.nf4_dequant_gemv_workspace_bytes(4096, 8192, 16)
    assert need >= 2 * 16 * 4096 * 4
    assert f(*a, 64, 4096, 8192, P, 16, P, P, need - 1, None) == E_SIZE
    g = L.nf4_dequant_gemv_workspace_bytes
    assert g(0, 64, 1) == 0 and g(4, 0, 1) == 0 and g(4, 64, 0) == 0 and g(4, 64, 17) == 0
    assert g(4, 64, 1) > 0


def test_gemm_workspace_bytes_of_rejected_shapes_is_zero(L):
    g = L.nf4_dequant_gemm_workspace_bytes
    assert g(0, 64, 1) == 0 and g(4, 0, 1) == 0 and g(4, 64, 0) == 0 and g(4, 64, 65) == 0
    assert g(4, 64, 1) > 0


def test_quantize_ref_argument_checks(L):
    f = L.nf4_quantize_ref
    assert f(P, -1, 64, P, P, None, None, None, None, None) == E_SIZE
    assert f(P, 5, 65, P, P, None, None, None, None, None) == E_BS
    assert f(None, 0, 64, None, None, None, None, None, None, None) == OK
    assert f(None, 5, 64, P, P, None, None, None, None, None) == E_NULL
    assert f(P, 5, 64, P, None, None, None, None, None, None) == E_NULL
    assert f(P, 5, 64, P, P, P, None, P, P, None) == E_NULL             # DQ wants all four outputs
    assert f(P + 2, 5, 64, P, P, None, None, None, None, None) == E_ALIGN


def test_dq_encode_argument_checks(L):
    f = L.nf4_dq_encode
    assert f(P, -1, 256, P, P, P, P, None) == E_SIZE
    assert f(P, 10, 100, P, P, P, P, None) == E_SHAPE
    assert f(P, 10, 0, P, P, P, P, None) == E_SHAPE
    assert f(None, 0, 256, None, None, None, None, None) == OK
    assert f(None, 10, 256, P, P, P, P, None) == E_NULL
    assert f(P, 10, 256, None, P, P, P, None) == E_NULL
    assert f(P, 10, 256, P, P, None, P, None) == E_NULL
    assert f(P + 2, 10, 256, P, P, P, P, None) == E_ALIGN
    assert f(P, 10, 256, P + 1, P + 2, P, P, None) == E_ALIGN           # absmax_q8 is bytes; scale2 is not


def test_codebook_entry_points_argument_checks(L):
    f = L.nf4_dequantize_codebook
    assert f(P, P, P, 64, -1, P, 0, None) == E_SIZE
    assert f(P, P, P, 96, 10, P, 0, None) == E_BS
    assert f(P, P, None, 64, 0, None, 0, None) == OK
    assert f(P, P, P + 2, 64, 10, P, 0, None) == E_ALIGN             # codebook is read as floats
    assert f(None, P, P, 64, 10, P, 0, None) == E_NULL
    g = L.nf4_dequantize_dq_codebook
    a = [P] * 5
    for bad in (0, 3, 100, 1 << 17, -256):
        assert g(*a, bad, P, 64, 10, P, 0, None) == E_SHAPE         # group must be a power of two in [1, 65536]
    assert g(*a, 64, None, 64, 0, None, 1, None) == OK
    assert g(P, P, None, P, P, 64, P, 64, 10, P, 0, None) == E_NULL
    h = L.nf4_quantize_ref_codebook
    assert h(P, -1, 64, P, 256, P, P, None, None, None, None, None) == E_SIZE
    assert h(P, 5, 64, P, 100, P, P, P, P, P, P, None) == E_SHAPE
    assert h(None, 0, 64, None, 256, None, None, None, None, None, None, None) == OK
    assert h(P, 5, 64, P + 1, 256, P, P, None, None, None, None, None) == E_ALIGN
    assert h(P, 5, 64, P, 256, P, P, P, None, P, P, None) == E_NULL


def test_quantize_argument_checks(L):
    f = L.nf4_quantize
    assert f(P, -1, 64, P, P, None) == E_SIZE
    assert f(P, 5, 100, P, P, None) == E_BS
    assert f(None, 0, 64, None, None, None) == OK
    assert f(None, 5, 64, P, P, None) == E_NULL
    assert f(P, 5, 64, None, P, None) == E_NULL
    assert f(P, 5, 64, P, None, None) == E_NULL
    assert f(P + 4, 5, 64, P, P, None) == E_ALIGN
    assert f(P, 5, 64, P + 1, P, None) == E_ALIGN


def test_quantize_codebook_argument_checks(L):
    f = L.nf4_quantize_codebook                  # (src, n, blocksize, codebook, packed, absmax, workspace, bytes, stream)
    assert f(P, -1, 64, P, P, P, P, 1024, None) == E_SIZE
    assert f(P, 5, 100, P, P, P, P, 1024, None) == E_BS
    assert f(None, 0, 64, P, None, None, None, 0, None) == OK
    assert f(None, 5, 64, P, P, P, P, 1024, None) == E_NULL
    assert f(P, 5, 64, P, None, P, P, 1024, None) == E_NULL
    assert f(P, 5, 64, P, P, None, P, 1024, None) == E_NULL
    assert f(P, 5, 64, P, P, P, None, 1024, None) == E_NULL      # a table needs the workspace
    assert f(P, 5, 64, P, P, P, P, 1023, None) == E_SIZE
    assert f(P + 4, 5, 64, P, P, P, P, 1024, None) == E_ALIGN
    assert f(P, 5, 64, P + 2, P, P, P, 1024, None) == E_ALIGN
    assert f(P, 5, 64, P, P, P, P + 4, 1024, None) == E_ALIGN
    # no table: nf4_quantize, whose checks answer (no workspace asked for)
    assert f(P, 5, 100, None, P, P, None, 0, None) == E_BS
    assert f(None, 5, 64, None, P, P, None, 0, None) == E_NULL


def test_binding_raises_with_the_status_name():
    with pytest.raises(binding.NF4Error, match="NF4_ERR_BLOCKSIZE"):
        binding._check(E_BS)


def test_product_code_never_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2604_02556_amd")
    for dirpath, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, name)).read()
                for needle in ("import oracle", "from oracle", "nf4_oracle", "nf4o_"):
                    assert needle not in text, (needle, os.path.join(dirpath, name))
