"""GPU parity for the fused kernels with the data type as a parameter (Sec. V-A): nf4_dequant_gemv_codebook and
nf4_dequant_gemm_codebook against the oracle's dequant_gemv_rows_codebook, with an FP4-style (E2M1) table read
from memory, block sizes 64 and 128, and second-level groups of 1, 2, 64 and 1024 blocks.  Shapes and token counts
are chosen so that every kernel behind the two calls is exercised: the single-wave and eight-wave FMA kernels, the
column-slice kernel, the matrix-core kernel with two-term levels, and both split-K forms."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_02556_amd import binding as nf4
from paper_2604_02556_amd import synth
from gpu_util import dev

pytestmark = pytest.mark.gpu


def make_case(N, K, seed, blocksize, group, table):
    w = synth.gaussian_weights(N * K, 0.02, seed)
    p, a = oracle.quantize_codebook(w, table, blocksize)
    return (p,) + tuple(oracle.dq_encode_group(a, group))


def within_bar(y, ref):
    err = np.abs(y.astype(np.float64) - ref)
    rms = np.sqrt(np.mean(ref ** 2))
    return np.all(err <= 1e-2 * np.abs(ref) + 1e-2 * rms) and err.max() / np.abs(ref).max() < 2e-3


# (N, K): short rows (single-wave kernel), slice-kernel rows, long rows (eight-wave kernel), very long rows
SHAPES = [(37, 1024), (50, 8192 + 2048), (21, 16384 + 4096), (6, 32768 + 4096)]


@pytest.mark.parametrize("blocksize,group", [(64, 64), (64, 1024), (128, 2), (64, 1), (64, 256)])
@pytest.mark.parametrize("N,K", SHAPES)
def test_gemv_with_a_codebook_and_other_group_sizes(N, K, blocksize, group):
    table = synth.e2m1_codebook()
    case = make_case(N, K, seed=N + K + group, blocksize=blocksize, group=group, table=table)
    d = [dev(a) for a in case]
    dt = dev(table)
    for B in (1, 2, 4, 16):
        x = synth.activations_fp16(B, K, seed=B + group)
        _, ref = oracle.dequant_gemv_rows_codebook(*case, group, table, N, K, x.view(np.uint16), 0, N, blocksize=blocksize)
        y = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
        nf4.nf4_dequant_gemv_codebook(*d, group, dt, blocksize, N, K, dev(x), B, y)
        ws = torch.full((nf4.nf4_dequant_gemv_workspace_bytes(N, K, B),), 0xFF, dtype=torch.uint8, device="cuda")
        y_ws = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
        nf4.nf4_dequant_gemv_codebook(*d, group, dt, blocksize, N, K, dev(x), B, y_ws, workspace=ws)
        torch.cuda.synchronize()
        assert within_bar(y.cpu().numpy(), ref), ("no workspace", B)
        assert within_bar(y_ws.cpu().numpy(), ref), ("workspace", B)


def test_null_codebook_and_group_256_are_the_plain_calls():
    N, K = 40, 8192
    table = oracle.table()
    case = make_case(N, K, seed=3, blocksize=64, group=256, table=table)
    d = [dev(a) for a in case]
    for B in (1, 2, 5):
        x = dev(synth.activations_fp16(B, K, seed=B))
        y0 = torch.empty((B, N), dtype=torch.float16, device="cuda")
        y1 = torch.empty((B, N), dtype=torch.float16, device="cuda")
        y2 = torch.empty((B, N), dtype=torch.float16, device="cuda")
        nf4.nf4_dequant_gemv(*d, 64, N, K, x, B, y0)
        nf4.nf4_dequant_gemv_codebook(*d, 256, None, 64, N, K, x, B, y1)
        nf4.nf4_dequant_gemv_codebook(*d, 256, dev(table), 64, N, K, x, B, y2)       # the NF4 levels from memory
        torch.cuda.synchronize()
        assert torch.equal(y0.view(torch.int16), y1.view(torch.int16))
        assert torch.equal(y0.view(torch.int16), y2.view(torch.int16))


@pytest.mark.parametrize("blocksize,group", [(64, 64), (128, 1024), (64, 1)])
@pytest.mark.parametrize("N,K", [(37, 1024), (300, 4096 + 512)])
def test_gemm_with_a_codebook_and_other_group_sizes(N, K, blocksize, group):
    table = synth.e2m1_codebook()
    case = make_case(N, K, seed=2 * N + K + group, blocksize=blocksize, group=group, table=table)
    d = [dev(a) for a in case]
    dt = dev(table)
    for B in (8, 40):
        x = synth.activations_fp16(B, K, seed=B + group)
        _, ref = oracle.dequant_gemv_rows_codebook(*case, group, table, N, K, x.view(np.uint16), 0, N, blocksize=blocksize,
                                                   round_weights_to_fp16=True)
        for split in (False, True):
            ws = None
            if split:
                ws = torch.full((nf4.nf4_dequant_gemm_workspace_bytes(N, K, B),), 0xFF, dtype=torch.uint8, device="cuda")
            y = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
            nf4.nf4_dequant_gemm_codebook(*d, group, dt, blocksize, N, K, dev(x), B, y, workspace=ws)
            torch.cuda.synchronize()
            assert within_bar(y.cpu().numpy(), ref), (B, split)


def test_bad_group_size_is_rejected():
    t = torch.zeros(64, dtype=torch.float32, device="cuda")
    L = nf4.lib()
    a = t.data_ptr()
    for group in (0, 3, 100, 1 << 17):
        assert nf4.status_string(L.nf4_dequant_gemv_codebook(a, a, a, a, a, group, None, 64, 4, 64, a, 1, a, None, 0, None)) == "NF4_ERR_SHAPE"
        assert nf4.status_string(L.nf4_dequant_gemm_codebook(a, a, a, a, a, group, None, 64, 4, 64, a, 1, a, None, 0, None)) == "NF4_ERR_SHAPE"
    torch.cuda.synchronize()
