"""GPU parity: the fused dequantise + MFMA GEMM (nf4_dequant_gemm) against the
oracle's dequantise-to-FP16-then-matmul definition.  Same tolerance as the GEMV
(summation order differs): |y - y_ref| <= 1e-2 |y_ref| + 1e-2 rms(y_ref); with
unit-vector activations the result must be the FP16 weight itself, bit for bit.
Every case runs both algorithms of the entry point: the single kernel (no
workspace) and the split along K with a caller-provided workspace."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_02556_amd import binding as nf4
from paper_2604_02556_amd import synth
from gpu_util import dev

pytestmark = pytest.mark.gpu


def make_case(N, K, seed, sigma=0.015, blocksize=64):
    w = synth.gaussian_weights(N * K, sigma, seed)
    p, a = oracle.quantize(w, blocksize)
    q8, s2, off, c2 = oracle.dq_encode(a)
    return p, q8, s2, off, c2


def gemm_gpu(case, N, K, x, blocksize=64, split=False):
    p, q8, s2, off, c2 = case
    B = x.shape[0]
    y = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
    ws = None
    if split:
        need = nf4.nf4_dequant_gemm_workspace_bytes(N, K, B)
        assert need > 0
        # NaN-filled and with a guard band behind it: partial sums must be written before they are read,
        # and nothing may be written past the stated size
        ws = torch.full((need // 4 + 64,), float("nan"), dtype=torch.float32, device="cuda")
    nf4.nf4_dequant_gemm(dev(p), dev(q8), dev(s2), dev(off), dev(c2), blocksize, N, K, dev(x), B, y, workspace=ws)
    torch.cuda.synchronize()
    if split:
        assert torch.isnan(ws[need // 4 + (1 if need % 4 else 0):]).all()
    return y.cpu().numpy()


SPLIT = pytest.mark.parametrize("split", [False, True], ids=["single", "splitk"])


@SPLIT
@pytest.mark.parametrize("B", [1, 2, 4, 15, 16, 17, 32, 33, 48, 64])
@pytest.mark.parametrize("N,K", [(37, 256), (64, 2048 + 512), (16, 8192), (130, 64), (5, 320), (530, 1024)])
def test_small_shapes_all_batches(N, K, B, split):
    case = make_case(N, K, seed=N * 7 + K)
    x = synth.activations_fp16(B, K, seed=B)
    _, ref = oracle.dequant_gemm_rows(*case, N, K, x.view(np.uint16), 0, N)
    y = gemm_gpu(case, N, K, x, split=split)
    assert np.isfinite(y).all()
    rms = np.sqrt(np.mean(ref ** 2))
    assert np.all(np.abs(y.astype(np.float64) - ref) <= 1e-2 * np.abs(ref) + 1e-2 * rms)
    assert np.abs(y - ref).max() / np.abs(ref).max() < 2e-3


@SPLIT
def test_unit_vectors_reproduce_fp16_dequantized_columns_exactly(split):
    N, K = 40, 512
    case = make_case(N, K, seed=5)
    w16 = oracle.dequantize_dq(*case, N * K, out_dtype=oracle.FP16).reshape(N, K)
    ks = [0, 1, 7, 8, 63, 64, 255, 256, 300, 511]
    x = np.zeros((len(ks), K), np.float16)
    for b, k in enumerate(ks):
        x[b, k] = 1.0
    y = gemm_gpu(case, N, K, x, split=split)
    assert np.array_equal(y.view(np.uint16), w16[:, ks].T)


@SPLIT
def test_other_blocksize_and_zero_activations(split):
    N, K = 48, 1024
    case = make_case(N, K, seed=9, blocksize=256)
    x = synth.activations_fp16(20, K, seed=3)
    _, ref = oracle.dequant_gemm_rows(*case, N, K, x.view(np.uint16), 0, N, blocksize=256)
    y = gemm_gpu(case, N, K, x, blocksize=256, split=split)
    assert np.abs(y - ref).max() / np.abs(ref).max() < 2e-3
    y0 = gemm_gpu(case, N, K, np.zeros((3, K), np.float16), blocksize=256, split=split)
    assert np.all(y0 == 0)


def test_split_is_deterministic_and_workspace_size_is_as_declared():
    N, K, B = 300, 4096, 24
    case = make_case(N, K, seed=21)
    x = synth.activations_fp16(B, K, seed=8)
    a = gemm_gpu(case, N, K, x, split=True)
    b = gemm_gpu(case, N, K, x, split=True)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    need = nf4.nf4_dequant_gemm_workspace_bytes(N, K, B)
    assert need % (B * N * 4) == 0 and need // (B * N * 4) >= 2          # whole FP32 partial planes, K really split
    small = torch.empty(need // 4 - 1, dtype=torch.float32, device="cuda")
    y = torch.empty((B, N), dtype=torch.float16, device="cuda")
    p, q8, s2, off, c2 = case
    with pytest.raises(nf4.NF4Error):
        nf4.nf4_dequant_gemm(dev(p), dev(q8), dev(s2), dev(off), dev(c2), 64, N, K, dev(x), B, y, workspace=small)
