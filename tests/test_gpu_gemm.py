"""GPU parity: the fused dequantise + MFMA GEMM (nf4_dequant_gemm) against the
oracle's dequantise-to-FP16-then-matmul definition.  Same tolerance as the GEMV
(summation order differs): |y - y_ref| <= 1e-2 |y_ref| + 1e-2 rms(y_ref); with
unit-vector activations the result must be the kernel's FP16 weight itself, bit
for bit (the product narrowed in one rounding, see the test).
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
def test_unit_vectors_reproduce_the_fp16_weights(split):
    """With unit-vector activations y is the kernel's FP16 weight itself.  The kernel narrows level * scale to
    FP16 in ONE rounding (a mixed-precision multiply-add instruction), while the dequantise-then-matmul flow
    rounds the product to FP32 first and then to FP16.  The two agree except where the FP32-rounded product is
    exactly half way between two FP16 values (about 1 weight in 10^4), and then differ by one FP16 ulp.  Asserted:
    every output is the once-rounded product bit for bit, is within one ulp of the twice-rounded one, and at
    least 99.9 % equal it."""
    N, K = 4096, 256
    case = make_case(N, K, seed=5)
    p, q8, s2, off, c2 = case
    ks = [0, 1, 7, 8, 31, 32, 63, 64, 65, 127, 128, 200, 254, 255, 100, 17]
    x = np.zeros((len(ks), K), np.float16)
    for b, k in enumerate(ks):
        x[b, k] = 1.0
    y = gemm_gpu(case, N, K, x, split=split)
    # the exact products in float64 (24 x 24 significant bits fit), rounded once by numpy
    codes = np.stack([p >> 4, p & 15], axis=1).reshape(N, K)
    scale = oracle.dq_decode(q8, s2, off, c2).astype(np.float64).repeat(64).reshape(N, K)
    once = (oracle.table().astype(np.float64)[codes] * scale).astype(np.float16)
    twice = oracle.dequantize_dq(*case, N * K, out_dtype=oracle.FP16).reshape(N, K)
    assert np.array_equal(y.view(np.uint16), once[:, ks].T.view(np.uint16))
    differ = y.view(np.uint16) != twice[:, ks].T
    print(f"{int(differ.sum())} of {y.size} weights differ between one and two roundings")
    assert differ.mean() < 1e-3
    a, b = y.view(np.uint16).astype(np.int32), twice[:, ks].T.astype(np.int32)
    assert np.all(np.abs(a - b) <= 1)                       # neighbouring FP16 values of the same sign


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
