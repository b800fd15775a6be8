"""GPU parity: the fused dequantise + MFMA GEMM (nf4_dequant_gemm) against the
oracle's dequantise-to-FP16-then-matmul definition.  Same tolerance as the GEMV
(summation order differs): |y - y_ref| <= 1e-2 |y_ref| + 1e-2 rms(y_ref); with
unit-vector activations the result must be the FP16 weight itself, bit for bit."""
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


def gemm_gpu(case, N, K, x, blocksize=64):
    p, q8, s2, off, c2 = case
    B = x.shape[0]
    y = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
    nf4.nf4_dequant_gemm(dev(p), dev(q8), dev(s2), dev(off), dev(c2), blocksize, N, K, dev(x), B, y)
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("B", [1, 2, 4, 15, 16, 17, 32, 33, 48, 64])
@pytest.mark.parametrize("N,K", [(37, 256), (64, 2048 + 512), (16, 8192), (130, 64), (5, 320)])
def test_small_shapes_all_batches(N, K, B):
    case = make_case(N, K, seed=N * 7 + K)
    x = synth.activations_fp16(B, K, seed=B)
    _, ref = oracle.dequant_gemm_rows(*case, N, K, x.view(np.uint16), 0, N)
    y = gemm_gpu(case, N, K, x)
    assert np.isfinite(y).all()
    rms = np.sqrt(np.mean(ref ** 2))
    assert np.all(np.abs(y.astype(np.float64) - ref) <= 1e-2 * np.abs(ref) + 1e-2 * rms)
    assert np.abs(y - ref).max() / np.abs(ref).max() < 2e-3


def test_unit_vectors_reproduce_fp16_dequantized_columns_exactly():
    N, K = 40, 512
    case = make_case(N, K, seed=5)
    w16 = oracle.dequantize_dq(*case, N * K, out_dtype=oracle.FP16).reshape(N, K)
    ks = [0, 1, 7, 8, 63, 64, 255, 256, 300, 511]
    x = np.zeros((len(ks), K), np.float16)
    for b, k in enumerate(ks):
        x[b, k] = 1.0
    y = gemm_gpu(case, N, K, x)
    assert np.array_equal(y.view(np.uint16), w16[:, ks].T)


def test_other_blocksize_and_zero_activations():
    N, K = 48, 1024
    case = make_case(N, K, seed=9, blocksize=256)
    x = synth.activations_fp16(20, K, seed=3)
    _, ref = oracle.dequant_gemm_rows(*case, N, K, x.view(np.uint16), 0, N, blocksize=256)
    y = gemm_gpu(case, N, K, x, blocksize=256)
    assert np.abs(y - ref).max() / np.abs(ref).max() < 2e-3
    y0 = gemm_gpu(case, N, K, np.zeros((3, K), np.float16), blocksize=256)
    assert np.all(y0 == 0)
