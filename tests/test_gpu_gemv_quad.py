"""GPU parity for the GEMV kernel on the 4 x 4 x 4 matrix-core instruction (a lane owns a 32-column piece of one of
four rows; taken for three and four tokens when 4096 <= K and four passes of a workgroup cover a row).  The general
GEMV tests cover it on their shapes; these aim at its own edges: one to four passes over the rows, a last column
wave that is partly or wholly past K, row counts that are not multiples of four or leave row streams and
workgroups without rows, more workgroups than compute units (rows per workgroup capped by the LDS the block scales
need), block sizes other than 64, scale codes at an address that is not a multiple of 4, tokens that differ (a
token landing in another token's slot would show), and single weights picked by unit vectors.

The levels enter the matrix cores as two FP16 terms, so a single weight comes back as rne_fp16(W (1 + e)) with
|e| <= 2^-21 (as on the other matrix-core paths) rather than bit for bit."""
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


def gemv(case, N, K, x, blocksize=64, q8_offset=0, workspace=False):
    p, q8, s2, off, c2 = case
    B = x.shape[0]
    dq8 = dev(q8)
    if q8_offset:
        shifted = torch.empty(q8.size + q8_offset, dtype=torch.uint8, device="cuda")
        shifted[q8_offset:] = dq8
        dq8 = shifted[q8_offset:]
    y = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
    if workspace:
        ws = torch.full((max(nf4.nf4_dequant_gemv_workspace_bytes(N, K, B), 16),), 0xFF, dtype=torch.uint8, device="cuda")
        nf4.nf4_dequant_gemv_ws(dev(p), dq8, dev(s2), dev(off), dev(c2), blocksize, N, K, dev(x), B, y, ws)
    else:
        nf4.nf4_dequant_gemv(dev(p), dq8, dev(s2), dev(off), dev(c2), blocksize, N, K, dev(x), B, y)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def check(y, ref):
    err = np.abs(y.astype(np.float64) - ref)
    rms = np.sqrt(np.mean(ref ** 2))
    assert np.all(err <= 1e-2 * np.abs(ref) + 1e-2 * rms)
    assert err.max() / np.abs(ref).max() < 2e-3


@pytest.mark.parametrize("B", [3, 4])
@pytest.mark.parametrize("N,K,blocksize", [
    (33, 4096, 64),             # eight column waves, one pass, two row streams; 33 rows over 256 workgroups
    (1, 4096, 64), (3, 8192, 64),                  # fewer rows than a group of four
    (70, 4096 + 64, 64),        # the ninth column wave holds one block: 62 of its 64 lanes have no columns
    (300, 8192 + 512, 64),      # 17 column pieces in two passes of nine waves: the last wave of the second pass is wholly past K
    (41, 18496, 64),            # 36.1 pieces: three passes of thirteen waves
    (5, 32768, 64),             # four passes of sixteen waves, the longest rows the kernel takes
    (9000, 8192, 64),           # 36 rows per workgroup: four column waves, four passes, four row streams
    (28672 // 8, 8192, 64),     # 16 rows per workgroup on 224 workgroups
    (300, 6144, 128), (19, 8192, 4096), (64, 12288, 1024),      # other block sizes: several lanes or waves per block
    (1000, 5120, 64), (777, 25600, 64),                          # Qwen3-32B row lengths, ragged row counts
])
def test_shapes_against_the_oracle(N, K, blocksize, B):
    case = make_case(N, K, seed=N + K + blocksize, blocksize=blocksize)
    x = synth.activations_fp16(B, K, seed=K % 97 + B)
    host = dict(zip(("packed", "absmax_q8", "scale2", "offset", "code2"), case))
    if N * K > 1 << 24 and blocksize == 64:
        ref = oracle_rows_threaded(oracle.dequant_gemv_rows, host, N, K, x.view(np.uint16))
    else:
        _, ref = oracle.dequant_gemv(*case, N, K, x.view(np.uint16), blocksize)
    y = gemv(case, N, K, x, blocksize)
    check(y, ref)
    y_ws = gemv(case, N, K, x, blocksize, workspace=True)                # the workspace form takes the same kernel
    assert np.array_equal(y.view(np.uint16), y_ws.view(np.uint16))


@pytest.mark.parametrize("q8_offset", [1, 2, 3])
def test_scale_codes_at_any_address(q8_offset):
    N, K, B = 50, 8192 + 2048, 4
    case = make_case(N, K, seed=11)
    x = synth.activations_fp16(B, K, seed=12)
    y0 = gemv(case, N, K, x)
    y1 = gemv(case, N, K, x, q8_offset=q8_offset)
    assert np.array_equal(y0.view(np.uint16), y1.view(np.uint16))       # same arithmetic, byte loads instead of dwords
    _, ref = oracle.dequant_gemv(*case, N, K, x.view(np.uint16))
    check(y1, ref)


def test_more_workgroups_than_compute_units():
    """10240 rows of 32768: 512 blocks per row cap a workgroup at 28 rows, so 366 workgroups share 256 compute
    units; every output against the oracle."""
    N, K, B = 10240, 32768, 4
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    w = torch.empty(N * K, dtype=torch.float32, device="cuda").normal_(0.0, 0.015, generator=g)
    b = nf4.alloc_quantized(N * K, 64, dq=True)
    nf4.nf4_quantize_ref(w, N * K, 64, b["packed"], b["absmax"], b["absmax_q8"], b["scale2"], b["offset"], b["code2"])
    del w
    x = synth.activations_fp16(B, K, seed=78)
    y = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
    nf4.nf4_dequant_gemv(b["packed"], b["absmax_q8"], b["scale2"], b["offset"], b["code2"], 64, N, K, dev(x), B, y)
    torch.cuda.synchronize()
    host = {k: v.cpu().numpy() for k, v in b.items()}
    ref = oracle_rows_threaded(oracle.dequant_gemv_rows, host, N, K, x.view(np.uint16))
    check(y.cpu().numpy(), ref)


@pytest.mark.parametrize("B", [3, 4])
def test_unit_vectors_pick_single_weights_to_22_bits(B):
    """Token b looks at column ks[b] only, a different column per token: y[b][r] is W[r][ks[b]] to 2^-21 and one
    FP16 rounding, and almost always rne_fp16(W) bit for bit."""
    N, K = 37, 8192 + 2048 + 128                         # two passes; the second one's last waves are partly empty
    case = make_case(N, K, seed=21)
    w = oracle.dequantize_dq(*case, N * K, out_dtype=oracle.FP32).reshape(N, K)
    ks = [0, 1, 30, 31, 32, 33, 63, 64, 511, 512, 2047, 2048, 4095, 4096, 6143, 6144, 8191, 8192, K - 65, K - 64,
          K - 2, K - 1, 17, 1000]
    exact = total = 0
    for k0 in range(0, len(ks), B):
        chunk = ks[k0:k0 + B]
        x = np.zeros((B, K), np.float16)
        for b, k in enumerate(chunk):
            x[b, k] = 1.0
        y = gemv(case, N, K, x)[:len(chunk)]
        want = w[:, chunk].T
        ulp = np.spacing(np.abs(want).astype(np.float16)).astype(np.float64)
        err = np.abs(y.astype(np.float64) - want.astype(np.float64))
        assert np.all(err <= 0.5 * ulp + np.abs(want) * 2.0 ** -21 + 2.0 ** -24), chunk
        exact += int(np.sum(y.view(np.uint16) == want.astype(np.float16).view(np.uint16)))
        total += y.size
    assert exact > 0.99 * total


def test_tokens_keep_their_places():
    """Four tokens that are multiples 1, -2, 4, -1 of one vector (exact scalings in FP16 and FP32): the outputs are
    the same multiples of the first token's, up to the final rounding."""
    N, K = 64, 8192
    case = make_case(N, K, seed=31)
    base = synth.activations_fp16(1, K, seed=32)
    f = np.array([1.0, -2.0, 4.0, -1.0], np.float32)
    x = (base.astype(np.float32) * f[:, None]).astype(np.float16)
    assert np.array_equal(x.astype(np.float32), base.astype(np.float32) * f[:, None])     # the scalings are exact
    y = gemv(case, N, K, x).astype(np.float64)
    _, ref = oracle.dequant_gemv(*case, N, K, x.view(np.uint16))
    check(y, ref)
    for b in range(4):
        assert np.allclose(y[b], f[b] * y[0], rtol=2e-3, atol=1e-3 * np.abs(y).max())
