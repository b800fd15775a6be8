"""GPU parity: the fused dequantise + GEMV against the double-precision oracle.

Tolerance (the summation order differs, so this is not bit-exact): per element
|y - y_ref| <= 1e-2 * |y_ref| + 1e-2 * rms(y_ref).  The fp16 rounding of y
alone is 2^-11 relative; FP32 accumulation over K <= 28672 terms adds about
K * 2^-24 relative to the sum of |terms|, far inside the bar."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_02556_amd import binding as nf4
from paper_2604_02556_amd import synth
from gpu_util import dev

pytestmark = pytest.mark.gpu


def make_case(N, K, seed, sigma=0.015):
    w = synth.gaussian_weights(N * K, sigma, seed)
    p, a = oracle.quantize(w)
    q8, s2, off, c2 = oracle.dq_encode(a)
    return p, q8, s2, off, c2


def gemv_gpu(case, N, K, x):
    p, q8, s2, off, c2 = case
    B = x.shape[0]
    y = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
    nf4.nf4_dequant_gemv(dev(p), dev(q8), dev(s2), dev(off), dev(c2), 64, N, K, dev(x), B, y)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def within_bar(y, ref):
    rms = np.sqrt(np.mean(ref ** 2))
    return np.all(np.abs(y.astype(np.float64) - ref) <= 1e-2 * np.abs(ref) + 1e-2 * rms)


@pytest.mark.parametrize("B", [1, 2, 3, 4, 5, 6, 7, 8, 11, 16])
@pytest.mark.parametrize("N,K", [(37, 256), (64, 2048 + 512), (9, 8192), (130, 64),
                                 (37, 16384), (41, 18496), (4, 32768)])      # K >= 16384: the eight-wave kernel
def test_small_shapes_all_batches(N, K, B):
    case = make_case(N, K, seed=N * 7 + K)
    x = synth.activations_fp16(B, K, seed=B)
    _, ref = oracle.dequant_gemv(*case, N, K, x.view(np.uint16))
    y = gemv_gpu(case, N, K, x)
    assert within_bar(y, ref)
    err = np.abs(y - ref).max() / np.abs(ref).max()
    assert err < 2e-3, err


def test_unit_vectors_reproduce_columns_of_dequantized_w():
    N, K = 40, 512
    case = make_case(N, K, seed=5)
    w = oracle.dequantize_dq(*case, N * K, out_dtype=oracle.FP32).reshape(N, K)
    ks = [0, 1, 7, 8, 63, 64, 255, 256, 511]
    for k0 in range(0, len(ks), 2):                      # two tokens: the FP32 path (more go to the matrix cores)
        chunk = ks[k0:k0 + 2]
        x = np.zeros((len(chunk), K), np.float16)
        for b, k in enumerate(chunk):
            x[b, k] = 1.0
        y = gemv_gpu(case, N, K, x)
        want = w[:, chunk].T.astype(np.float16)          # one product, one rounding: exact
        assert np.array_equal(y.view(np.uint16), want.view(np.uint16))


def test_unit_vectors_on_long_rows():
    """The same property through the eight-wave kernel that serves rows of 16384 elements and more (a ragged
    last step and a row count that leaves most waves of the last workgroup without rows)."""
    N, K = 35, 16384 + 2048 + 192
    case = make_case(N, K, seed=21)
    w = oracle.dequantize_dq(*case, N * K, out_dtype=oracle.FP32).reshape(N, K)
    ks = [0, 1, 63, 64, 2047, 2048, 16383, 16384, K - 193, K - 192, K - 65, K - 1]
    for k0 in range(0, len(ks), 2):
        chunk = ks[k0:k0 + 2]
        x = np.zeros((len(chunk), K), np.float16)
        for b, k in enumerate(chunk):
            x[b, k] = 1.0
        y = gemv_gpu(case, N, K, x)
        want = w[:, chunk].T.astype(np.float16)
        assert np.array_equal(y.view(np.uint16), want.view(np.uint16))


@pytest.mark.parametrize("B", [1, 2])
@pytest.mark.parametrize("N,K", [(8, 16384), (12, 18432), (44, 20480)])
def test_long_rows_in_whole_steps(N, K, B):
    """Rows of whole 2048-element steps with a multiple of four rows: the long-row kernel then fetches the scale
    codes of four rows in one load per lane and passes the decoded scales round through LDS.  K / 64 = 256, 288 and
    320 blocks per row put the boundaries of the 256-block second-level groups at the start of a row, inside a step
    and between two steps.  Checked against the oracle, element by element against the form that fetches
    every scale where it is used (taken when the scale codes start at an odd address: bit-identical results), and
    with unit vectors that pick single weights (exact)."""
    case = make_case(N, K, seed=3 * N + K)
    p, q8, s2, off, c2 = case
    x = synth.activations_fp16(B, K, seed=B + 11)
    _, ref = oracle.dequant_gemv(*case, N, K, x.view(np.uint16))
    y = gemv_gpu(case, N, K, x)
    assert within_bar(y, ref)
    assert np.abs(y - ref).max() / np.abs(ref).max() < 2e-3
    # the same call with the scale codes at an odd address
    shifted = torch.empty(q8.size + 1, dtype=torch.uint8, device="cuda")
    shifted[1:] = dev(q8)
    y2 = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
    nf4.nf4_dequant_gemv(dev(p), shifted[1:], dev(s2), dev(off), dev(c2), 64, N, K, dev(x), B, y2)
    torch.cuda.synchronize()
    assert np.array_equal(y2.cpu().numpy().view(np.uint16), y.view(np.uint16))
    # single weights: every block of three rows, at both ends of the block
    w = oracle.dequantize_dq(*case, N * K, out_dtype=oracle.FP32).reshape(N, K)
    ks = [k for blk in range(0, K // 64, 37) for k in (64 * blk, 64 * blk + 63)] + [K - 64, K - 1]
    for k0 in range(0, len(ks), B):
        chunk = ks[k0:k0 + B]
        xu = np.zeros((B, K), np.float16)
        for b, k in enumerate(chunk):
            xu[b, k] = 1.0
        yu = gemv_gpu(case, N, K, xu)
        want = w[:, chunk].T.astype(np.float16)
        assert np.array_equal(yu[:len(chunk)].view(np.uint16), want.view(np.uint16)), chunk


@pytest.mark.parametrize("K,B", [(16384, 3), (17408, 4), (8192, 3), (8192 + 320, 4), (8192, 4), (8192 + 64, 6),
                                 (16384, 11), (2048 + 64, 3), (3072, 4)])
def test_few_tokens_on_tall_matrices(K, B):
    """Matrices of 16384 rows and more.  Three and four tokens on rows of 4096 columns and more take the 4 x 4 x 4
    matrix-core kernel (here with more workgroups than compute units, ragged last workgroup, K that leaves its last
    column wave partly empty); on shorter rows they still take the vector-ALU kernels (fewer rows would send them to
    the 16-row matrix-core tiles); five tokens and more run on those tiles with more workgroups than stay resident.
    Random codes drawn on the GPU; sampled rows against the oracle, the same call with the scale codes at an odd
    address (same arithmetic from byte loads: bit-identical), unit vectors (exact on the vector ALU, to 2^-21 on
    the matrix cores)."""
    N = 16384 + 8
    n = N * K
    nb = n // 64
    g = torch.Generator(device="cuda")
    g.manual_seed(K + B)
    packed = torch.randint(0, 256, (n // 2,), dtype=torch.uint8, device="cuda", generator=g)
    q8 = torch.randint(0, 256, (nb + 1,), dtype=torch.uint8, device="cuda", generator=g)
    scale2 = torch.rand((nb + 255) // 256, device="cuda", generator=g) * 0.02 + 0.001
    offset = torch.tensor([0.03], dtype=torch.float32, device="cuda")
    code2 = (torch.arange(256, device="cuda", dtype=torch.float32) - 127.0) / 127.0
    x = torch.from_numpy(synth.activations_fp16(B, K, seed=B + 3)).cuda()
    y = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
    y_odd = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
    q8_even = q8[:nb].clone()                             # a fresh allocation: even address
    q8_odd = torch.empty(nb + 1, dtype=torch.uint8, device="cuda")
    q8_odd[1:] = q8_even
    nf4.nf4_dequant_gemv(packed, q8_even, scale2, offset, code2, 64, N, K, x, B, y)
    nf4.nf4_dequant_gemv(packed, q8_odd[1:], scale2, offset, code2, 64, N, K, x, B, y_odd)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(y).any().item())
    assert torch.equal(y.view(torch.int16), y_odd.view(torch.int16))

    hp, hq, hs = packed.cpu().numpy(), q8_even.cpu().numpy(), scale2.cpu().numpy()
    ho, hc, hx = offset.cpu().numpy(), code2.cpu().numpy(), x.cpu().numpy().view(np.uint16)
    for r0 in (0, 4093, 16381, N - 5):
        cnt = 5
        _, ref = oracle.dequant_gemv_rows(hp, hq, hs, ho, hc, N, K, hx, r0, cnt)
        rms = max(float(np.sqrt(np.mean(ref ** 2))), 1e-6)
        got = y[:, r0:r0 + cnt].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - ref) <= 1e-2 * np.abs(ref) + 1e-2 * rms), r0
    # unit vectors: single weights of the last five rows, exact
    r0 = N - 5
    ks = [0, 63, 64, 1023, 1024, K // 2 + 5, K - 64, K - 1][:2 * B]
    for k0 in range(0, len(ks), B):
        chunk = ks[k0:k0 + B]
        xu = np.zeros((B, K), np.float16)
        for b, k in enumerate(chunk):
            xu[b, k] = 1.0
        yu = torch.empty((B, N), dtype=torch.float16, device="cuda")
        nf4.nf4_dequant_gemv(packed, q8_even, scale2, offset, code2, 64, N, K, torch.from_numpy(xu).cuda(), B, yu)
        torch.cuda.synchronize()
        # W[r][k] = level * scale in FP32, from the definition, for the five rows
        for b, k in enumerate(chunk):
            for r in range(r0, N):
                e = r * K + k
                byte = int(hp[e // 2])
                code = (byte >> 4) if e % 2 == 0 else (byte & 15)
                blk = e // 64
                scale = np.float32(np.float32(hc[hq[blk]]) * np.float32(hs[blk // 256])) + np.float32(ho[0])
                w32 = np.float32(oracle.table()[code]) * np.float32(scale)
                if B < 5 and K < 4096:
                    assert yu[b, r].item() == float(np.float16(w32)), (k, r)
                else:
                    ulp = float(np.spacing(np.abs(np.float16(w32))))
                    assert abs(yu[b, r].item() - float(w32)) <= 0.5 * ulp + abs(float(w32)) * 2.0 ** -21 + 2.0 ** -24, (k, r)


def test_zero_activations_and_all_ones_weights():
    N, K = 16, 1024
    case = make_case(N, K, seed=6)
    y0 = gemv_gpu(case, N, K, np.zeros((2, K), np.float16))
    assert np.all(y0 == 0)
    c2 = ((np.arange(256) - 127) / 127).astype(np.float32)
    ones = (np.full(N * K // 2, 0xFF, np.uint8), np.full(N * K // 64, 254, np.uint8), np.ones(1, np.float32),
            np.zeros(1, np.float32), c2)
    x = synth.activations_fp16(4, K, seed=7)
    y = gemv_gpu(ones, N, K, x)
    want = x.astype(np.float64).sum(axis=1, keepdims=True).repeat(N, 1)
    assert np.allclose(y, want, rtol=2e-3, atol=2e-2)


def test_matrix_core_path_carries_the_weight_to_22_bits():
    """From three tokens on (five on matrices of 16384 rows and more) the levels enter the matrix cores as two FP16
    terms and the block scale multiplies the block's sum in FP32.  With unit-vector activations the result is
    rne_fp16(W (1 + e)), |e| <= 2^-21: equal to rne_fp16(W) except within that distance of an FP16 rounding
    boundary, and never more than one FP16 ulp away."""
    N, K = 64, 1024
    case = make_case(N, K, seed=15)
    w = oracle.dequantize_dq(*case, N * K, out_dtype=oracle.FP32).reshape(N, K)
    ks = [0, 1, 7, 8, 31, 32, 63, 64, 127, 255, 256, 511, 777, 1023]
    x = np.zeros((len(ks), K), np.float16)
    for b, k in enumerate(ks):
        x[b, k] = 1.0
    y = gemv_gpu(case, N, K, x)
    want = w[:, ks].T
    ulp = np.spacing(np.abs(want).astype(np.float16)).astype(np.float64)
    err = np.abs(y.astype(np.float64) - want.astype(np.float64))
    assert np.all(err <= 0.5 * ulp + np.abs(want) * 2.0 ** -21 + 2.0 ** -24)
    exact = np.mean(y.view(np.uint16) == want.astype(np.float16).view(np.uint16))
    print(f"matrix-core path: {exact * 100:.2f} % of {y.size} unit-vector outputs equal rne_fp16(W) bit for bit")
    assert exact > 0.99


def test_matrix_core_path_matches_the_fma_path_closely():
    """The same tokens through both kernels (2 at a time on the vector ALU, 12 at once on the matrix cores)."""
    N, K = 96, 4096
    case = make_case(N, K, seed=16)
    x = synth.activations_fp16(12, K, seed=17)
    y_mfma = gemv_gpu(case, N, K, x).astype(np.float64)
    y_fma = np.concatenate([gemv_gpu(case, N, K, x[i:i + 2]) for i in range(0, 12, 2)]).astype(np.float64)
    _, ref = oracle.dequant_gemv(*case, N, K, x.view(np.uint16))
    scale = np.abs(ref).max()
    assert np.abs(y_mfma - ref).max() / scale < 1e-3 and np.abs(y_fma - ref).max() / scale < 1e-3
    assert np.abs(y_mfma - y_fma).max() / scale < 1e-3


# ---- nf4_dequant_gemv_ws: the same sum with a caller workspace (K split across workgroups from 3 tokens on)

def gemv_ws_gpu(case, N, K, x, poison=True):
    p, q8, s2, off, c2 = case
    B = x.shape[0]
    y = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
    ws = torch.empty(nf4.nf4_dequant_gemv_workspace_bytes(N, K, B), dtype=torch.uint8, device="cuda")
    if poison:
        ws.fill_(0xFF)                                   # NaN patterns: every partial sum read must have been written
    nf4.nf4_dequant_gemv_ws(dev(p), dev(q8), dev(s2), dev(off), dev(c2), 64, N, K, dev(x), B, y, ws)
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("B", [1, 2, 3, 4, 7, 11, 16])
@pytest.mark.parametrize("N,K", [(37, 256), (64, 2048 + 512), (9, 8192), (130, 64), (300, 4096 + 64), (41, 18496)])
def test_workspace_form_small_shapes_all_batches(N, K, B):
    """Ragged rows (N not a multiple of 16 or 256), K from one block to many windows with a ragged last window,
    every token count: against the oracle, to the GEMV's bar."""
    case = make_case(N, K, seed=N * 5 + K)
    x = synth.activations_fp16(B, K, seed=B + 31)
    _, ref = oracle.dequant_gemv(*case, N, K, x.view(np.uint16))
    y = gemv_ws_gpu(case, N, K, x)
    assert np.isfinite(y).all()
    assert within_bar(y, ref)
    assert np.abs(y - ref).max() / np.abs(ref).max() < 2e-3


def test_workspace_form_one_and_two_tokens_equal_the_plain_call():
    """Below three tokens the workspace is not used: the same kernels, bit-identical results."""
    N, K = 48, 4096
    case = make_case(N, K, seed=77)
    for B in (1, 2):
        x = synth.activations_fp16(B, K, seed=B)
        assert np.array_equal(gemv_ws_gpu(case, N, K, x).view(np.uint16), gemv_gpu(case, N, K, x).view(np.uint16))


def test_workspace_form_carries_the_weight_to_22_bits_and_is_deterministic():
    """Unit vectors pick single weights: rne_fp16(W (1 + e)), |e| <= 2^-21, as on the matrix-core path without a
    workspace; and two calls give the same bits (the partial sums are added in a fixed order)."""
    N, K = 272, 6144                                     # two row blocks of 256 rows, several splits of K
    case = make_case(N, K, seed=23)
    w = oracle.dequantize_dq(*case, N * K, out_dtype=oracle.FP32).reshape(N, K)
    ks = [0, 1, 7, 8, 31, 32, 63, 64, 127, 511, 512, 1023, 4095, 4096, K - 65, K - 1]
    x = np.zeros((len(ks), K), np.float16)
    for b, k in enumerate(ks):
        x[b, k] = 1.0
    y = gemv_ws_gpu(case, N, K, x)
    want = w[:, ks].T
    ulp = np.spacing(np.abs(want).astype(np.float16)).astype(np.float64)
    err = np.abs(y.astype(np.float64) - want.astype(np.float64))
    assert np.all(err <= 0.5 * ulp + np.abs(want) * 2.0 ** -21 + 2.0 ** -24)
    assert np.mean(y.view(np.uint16) == want.astype(np.float16).view(np.uint16)) > 0.99
    xr = synth.activations_fp16(16, K, seed=5)
    y1, y2 = gemv_ws_gpu(case, N, K, xr), gemv_ws_gpu(case, N, K, xr, poison=False)
    assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))


def test_workspace_form_with_huge_and_tiny_scales():
    """The block scale stays FP32 on the matrix-core paths, so weights beyond the FP16 range and scales far below it
    are carried like any other (y itself must still fit FP16: the activations are scaled to keep it there)."""
    N, K = 32, 1024
    p = synth.random_codes(N * K // 2, seed=9)
    q8 = np.full(N * K // 64, 254, np.uint8)
    c2 = ((np.arange(256) - 127) / 127).astype(np.float32)
    for scale, xmag in ((3.0e5, 1.0e-4), (1.0e-9, 1.0e4)):
        case = (p, q8, np.full(N * K // 64 // 256, scale, np.float32), np.zeros(1, np.float32), c2)
        x = (synth.activations_fp16(5, K, seed=3).astype(np.float32) * xmag).astype(np.float16)
        _, ref = oracle.dequant_gemv(*case, N, K, x.view(np.uint16))
        for y in (gemv_ws_gpu(case, N, K, x), gemv_gpu(case, N, K, x)):
            assert np.isfinite(y).all()
            assert np.abs(y - ref).max() / np.abs(ref).max() < 2e-3
