"""GPU parity for the one-token GEMV kernel that works by column slices (a wave owns 2048 columns and streams the
rows through it; taken for one token and 4096 <= K <= 32768).  The general GEMV tests cover it on their shapes;
these aim at its own edges: a last slice that is partly or almost wholly past K, K at both ends of its range,
row counts that leave workgroups and row streams without rows, more rows than one round of workgroups takes
(rows per workgroup capped by the LDS the block scales need), block sizes other than 64, scale codes at an
address that is not a multiple of 4, and single weights picked by unit vectors (exact)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_02556_amd import binding as nf4
from paper_2604_02556_amd import synth
from gpu_util import dev, oracle_rows_threaded

pytestmark = pytest.mark.gpu


def make_case(N, K, seed, blocksize=64):
    w = synth.gaussian_weights(N * K, 0.015, seed)
    p, a = oracle.quantize(w, blocksize)
    return (p,) + tuple(oracle.dq_encode(a))


def gemv(case, N, K, x, blocksize=64, q8_offset=0):
    p, q8, s2, off, c2 = case
    dq8 = dev(q8)
    if q8_offset:
        shifted = torch.empty(q8.size + q8_offset, dtype=torch.uint8, device="cuda")
        shifted[q8_offset:] = dq8
        dq8 = shifted[q8_offset:]
    y = torch.full((1, N), float("nan"), dtype=torch.float16, device="cuda")
    nf4.nf4_dequant_gemv(dev(p), dq8, dev(s2), dev(off), dev(c2), blocksize, N, K, dev(x), 1, y)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def check(y, ref):
    err = np.abs(y.astype(np.float64) - ref)
    rms = np.sqrt(np.mean(ref ** 2))
    assert np.all(err <= 1e-2 * np.abs(ref) + 1e-2 * rms)
    assert err.max() / np.abs(ref).max() < 2e-3


@pytest.mark.parametrize("N,K,blocksize", [
    (33, 4096, 64),             # two slices, eight row streams, 33 rows over 256 workgroups
    (1, 4096, 64),              # a single row
    (70, 4096 + 64, 64),        # the third slice holds one block: 62 of its 64 lanes have no columns
    (300, 6144 + 1984, 64),     # the last slice lacks one block
    (5, 32768, 64),             # sixteen slices, the longest rows the kernel takes
    (41, 18496, 64),            # 9.03 slices
    (300, 6144, 128), (19, 8192, 4096), (64, 12288, 1024),      # other block sizes: several lanes or slices per block
    (1000, 5120, 64), (777, 25600, 64),                          # Qwen3-32B row lengths, ragged row counts
])
def test_shapes_against_the_oracle(N, K, blocksize):
    case = make_case(N, K, seed=N + K + blocksize, blocksize=blocksize)
    x = synth.activations_fp16(1, K, seed=K % 97)
    _, ref = oracle.dequant_gemv(*case, N, K, x.view(np.uint16), blocksize)
    check(gemv(case, N, K, x, blocksize), ref)


@pytest.mark.parametrize("q8_offset", [1, 2, 3])
def test_scale_codes_at_any_address(q8_offset):
    N, K = 50, 8192 + 2048
    case = make_case(N, K, seed=11)
    x = synth.activations_fp16(1, K, seed=12)
    y0 = gemv(case, N, K, x)
    y1 = gemv(case, N, K, x, q8_offset=q8_offset)
    assert np.array_equal(y0.view(np.uint16), y1.view(np.uint16))       # same arithmetic, byte loads instead of dwords
    _, ref = oracle.dequant_gemv(*case, N, K, x.view(np.uint16))
    check(y1, ref)


def test_more_rows_than_one_round_of_workgroups():
    """10240 rows of 32768: 512 blocks per row cap a workgroup at 30 rows, so 342 workgroups share 256 compute units;
    every output against the oracle."""
    N, K = 10240, 32768
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    w = torch.empty(N * K, dtype=torch.float32, device="cuda").normal_(0.0, 0.015, generator=g)
    b = nf4.alloc_quantized(N * K, 64, dq=True)
    nf4.nf4_quantize_ref(w, N * K, 64, b["packed"], b["absmax"], b["absmax_q8"], b["scale2"], b["offset"], b["code2"])
    del w
    x = synth.activations_fp16(1, K, seed=78)
    y = torch.full((1, N), float("nan"), dtype=torch.float16, device="cuda")
    nf4.nf4_dequant_gemv(b["packed"], b["absmax_q8"], b["scale2"], b["offset"], b["code2"], 64, N, K, dev(x), 1, y)
    torch.cuda.synchronize()
    host = {k: v.cpu().numpy() for k, v in b.items()}
    ref = oracle_rows_threaded(oracle.dequant_gemv_rows, host, N, K, x.view(np.uint16))
    check(y.cpu().numpy(), ref)


def test_unit_vectors_pick_single_weights_exactly():
    N, K = 37, 4096 + 2048 + 128
    case = make_case(N, K, seed=21)
    w = oracle.dequantize_dq(*case, N * K, out_dtype=oracle.FP32).reshape(N, K)
    for k in (0, 1, 30, 31, 32, 33, 63, 64, 2047, 2048, 4095, 4096, 6143, 6144, K - 65, K - 64, K - 2, K - 1):
        x = np.zeros((1, K), np.float16)
        x[0, k] = 1.0
        y = gemv(case, N, K, x)
        want = w[:, k].astype(np.float16)                # one product, one rounding: exact
        assert np.array_equal(y[0].view(np.uint16), want.view(np.uint16)), k
