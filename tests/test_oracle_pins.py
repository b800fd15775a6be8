"""Pins for the CPU oracle: each test fixes it to something other than itself --
the published level constants, the normal-quantile closed form, numpy/torch
conversions, brute force in a different arithmetic, or an invariant of the
format (Sec. II-B and Algorithm 1 of the paper)."""
import os

import numpy as np
import pytest
import torch
from scipy.stats import norm

import oracle
from paper_2604_02556_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def golden_levels():
    rows = [l.strip() for l in open(os.path.join(GOLDEN, "nf4_levels.txt")) if l.strip() and l[0] != "#"]
    return np.array([int(r, 16) for r in rows], dtype=np.uint32).view(np.float32)


def f16(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16)


# ---------------------------------------------------------------- the table

def test_table_matches_published_bit_patterns():
    assert np.array_equal(oracle.table().view(np.uint32), golden_levels().view(np.uint32))


def test_table_is_the_normal_quantile_construction():
    # Sec. II-B: quantiles of a normal distribution normalised to [-1, 1];
    # asymmetric: 8 positive levels, one zero, 7 negative ones.
    delta = 0.5 * (31.0 / 32.0 + 29.0 / 30.0)
    pos = norm.ppf(np.linspace(delta, 0.5, 9)[:-1])
    neg = -norm.ppf(np.linspace(delta, 0.5, 8)[:-1])
    closed = np.sort(np.concatenate([pos, [0.0], neg]))
    closed /= closed.max()
    assert np.abs(oracle.table().astype(np.float64) - closed).max() < 5e-7


def test_table_invariants():
    t = oracle.table()
    assert t[7] == 0.0 and t[0] == -1.0 and t[15] == 1.0
    assert np.all(np.diff(t) > 0)
    assert (t < 0).sum() == 7 and (t > 0).sum() == 8


# ------------------------------------------------------- fp32 -> 16-bit

def _interesting_f32():
    rng = np.random.Generator(np.random.PCG64(7))
    rand_bits = rng.integers(0, 2**32, size=200_000, dtype=np.uint64).astype(np.uint32)
    # every fp16 value, its neighbours' midpoints and one fp32 ulp either side
    h = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mids = ((h[:-1] + h[1:]) / 2).astype(np.float32)          # exact in fp32
    near = np.concatenate([mids, np.nextafter(mids, np.float32(np.inf)),
                           np.nextafter(mids, np.float32(-np.inf)), h.astype(np.float32)])
    edge = np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 65536.0, 1e38, np.inf, -np.inf,
                     2.0**-24, 2.0**-25, np.nextafter(np.float32(2.0**-25), np.float32(1)),
                     2.0**-14, 2.0**-126, 1e-45], dtype=np.float32)
    vals = np.concatenate([rand_bits.view(np.float32), near, -near, edge, -edge])
    return vals[~np.isnan(vals)]


def test_f32_to_f16_matches_numpy_rne():
    vals = _interesting_f32()
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    got = oracle.f32_to_f16_bits(vals)
    assert np.array_equal(got, want)


def test_f32_to_bf16_matches_torch_rne():
    vals = _interesting_f32()
    u = vals.view(np.uint32)
    mids = ((u & np.uint32(0xFFFF0000)) | np.uint32(0x8000)).view(np.float32)   # exact ties
    vals = np.concatenate([vals, mids[~np.isnan(mids)]])
    want = torch.from_numpy(vals.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.f32_to_bf16_bits(vals)
    assert np.array_equal(got, want)


def test_nan_stays_nan():
    nan = np.array([np.nan], dtype=np.float32)
    h = int(oracle.f32_to_f16_bits(nan)[0])
    b = int(oracle.f32_to_bf16_bits(nan)[0])
    assert (h & 0x7C00) == 0x7C00 and (h & 0x3FF) != 0
    assert (b & 0x7F80) == 0x7F80 and (b & 0x7F) != 0


# --------------------------------------------------------------- dequantize

def test_exhaustive_bytes_high_nibble_first():
    # Algorithm 1: out[2j] = T[q >> 4] * s, out[2j+1] = T[q & 15] * s.
    t = golden_levels()
    packed = np.arange(256, dtype=np.uint8)
    absmax = np.ones(8, dtype=np.float32)
    out = oracle.dequantize(packed, absmax, 512, out_dtype=oracle.FP32)
    assert np.array_equal(out[0::2], t[packed >> 4])
    assert np.array_equal(out[1::2], t[packed & 15])
    out16 = oracle.dequantize(packed, absmax, 512, out_dtype=oracle.FP16)
    assert np.array_equal(out16[0::2], t[packed >> 4].astype(np.float16).view(np.uint16))
    assert np.array_equal(out16[1::2], t[packed & 15].astype(np.float16).view(np.uint16))


def test_extreme_codes_hit_plus_minus_absmax_and_zero():
    absmax = np.array([0.5, 3.0, 1.0 / 1024], dtype=np.float32)       # exact in fp16/bf16
    for code, sign in ((0, -1.0), (15, 1.0), (7, 0.0)):
        packed = np.full(96, code * 17, dtype=np.uint8)
        for dt, view in ((oracle.FP16, lambda a: f16(a).astype(np.float32)),
                         (oracle.BF16, lambda a: (a.astype(np.uint32) << 16).view(np.float32))):
            out = view(oracle.dequantize(packed, absmax, 192, out_dtype=dt))
            assert np.array_equal(out, np.repeat(sign * absmax, 64))


def test_scale_is_per_64_element_block():
    # Sec. II-B: one scaling factor per 64 elements -> Algorithm 1's absmax
    # index is floor(i / 64), not the 512-element tile.
    nb = 24
    absmax = (2.0 ** np.arange(nb)).astype(np.float32) / 4096
    packed = np.full(nb * 32, 0xFF, dtype=np.uint8)                   # all +1
    out = oracle.dequantize(packed, absmax, nb * 64, out_dtype=oracle.FP32)
    assert np.array_equal(out, np.repeat(absmax, 64))
    out128 = oracle.dequantize(packed, absmax, nb * 64, blocksize=128, out_dtype=oracle.FP32)
    assert np.array_equal(out128, np.repeat(absmax[: nb // 2], 128))


def test_dequantize_equals_numpy_gather_multiply_round():
    # the whole definition, rewritten with library routines
    n = 64 * 300 + 37
    packed = synth.random_codes((n + 1) // 2, seed=11)
    absmax = synth.positive_scales(oracle.nblocks(n), seed=12, lo=1e-6, hi=3e4)
    codes = np.stack([packed >> 4, packed & 15], axis=1).reshape(-1)[:n]
    prod = golden_levels()[codes] * np.repeat(absmax, 64)[:n]         # float32 multiply
    assert np.array_equal(oracle.dequantize(packed, absmax, n, out_dtype=oracle.FP32), prod)
    with np.errstate(over="ignore"):
        assert np.array_equal(oracle.dequantize(packed, absmax, n), prod.astype(np.float16).view(np.uint16))
    want_bf = torch.from_numpy(prod).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.dequantize(packed, absmax, n, out_dtype=oracle.BF16), want_bf)


def test_subnormal_overflow_and_nan_products():
    packed = np.full(32 * 4, 0xF0, dtype=np.uint8)                    # +1, -1, +1, ...
    absmax = np.array([2.0**-20, 70000.0, np.inf, 2.0**-26], dtype=np.float32)
    out = f16(oracle.dequantize(packed, absmax, 256))
    assert out[0] == np.float16(2.0**-20) and out[1] == -np.float16(2.0**-20)   # fp16 subnormal kept
    assert np.isposinf(out[64]) and np.isneginf(out[65])                        # overflow -> inf
    assert np.isposinf(out[128])
    assert out[192] == 0 and out[193] == 0 and np.signbit(out[193])             # underflow -> signed 0
    nan_out = f16(oracle.dequantize(np.full(32, 0x77, np.uint8), np.array([np.inf], np.float32), 64))
    assert np.all(np.isnan(nan_out))                                            # 0 * inf


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 127, 1_000_003])
def test_ragged_sizes_never_read_or_write_past_n(n):
    packed = synth.random_codes((n + 1) // 2, seed=n)
    absmax = synth.positive_scales(oracle.nblocks(n), seed=n + 1)
    full = oracle.dequantize(packed, absmax, n)
    assert full.size == n
    # the unused low nibble of an odd tensor's last byte must not matter
    if n % 2:
        other = packed.copy()
        other[-1] ^= 0x0F
        assert np.array_equal(oracle.dequantize(other, absmax, n), full)
    # range form agrees and leaves the rest of its buffer alone
    buf = np.full(n + 8, 0xBEEF, dtype=np.uint16)
    first = min(n - 1, 31)
    oracle.dequantize_range(packed, absmax, first, n - first, buf)
    assert np.array_equal(buf[first:n], full[first:]) and np.all(buf[n:] == 0xBEEF) and np.all(buf[:first] == 0xBEEF)


# ----------------------------------------------------------------- quantize

def _brute_quantize(x, blocksize=64):
    """Nearest level by exhaustive search, distances in float32 like the definition."""
    t = golden_levels()
    n = x.size
    codes = np.empty(n, dtype=np.uint8)
    nb = (n + blocksize - 1) // blocksize
    absmax = np.zeros(nb, dtype=np.float32)
    for b in range(nb):
        blk = x[b * blocksize:(b + 1) * blocksize]
        a = np.abs(blk).max()
        absmax[b] = a
        if a == 0:
            codes[b * blocksize:b * blocksize + blk.size] = 7
            continue
        xn = (blk / a).astype(np.float32)
        d = np.abs(xn[:, None] - t[None, :]).astype(np.float32)
        codes[b * blocksize:b * blocksize + blk.size] = d.argmin(axis=1)     # first minimum = lower index
    if n % 2:
        codes = np.append(codes, 7)
    return ((codes[0::2] << 4) | codes[1::2]).astype(np.uint8), absmax


@pytest.mark.parametrize("n,seed", [(64 * 40, 1), (64 * 7 + 13, 2), (1, 3), (65, 4)])
def test_quantize_matches_brute_force(n, seed):
    x = synth.gaussian_weights(n, 0.02, seed, outlier_p=0.01)
    p, a = oracle.quantize(x)
    bp, ba = _brute_quantize(x)
    assert np.array_equal(a, ba) and np.array_equal(p, bp)


def test_quantize_midpoints_go_to_lower_index():
    t = golden_levels().astype(np.float64)
    mids = ((t[:-1] + t[1:]) / 2)
    exact = mids.astype(np.float32)
    keep = exact.astype(np.float64) == mids                     # midpoints representable in fp32
    x = np.concatenate([[1.0], exact[keep]]).astype(np.float32)  # absmax = 1 so x / absmax = x
    x = np.concatenate([x, np.zeros(64 - x.size, np.float32)])
    p, a = oracle.quantize(x)
    bp, _ = _brute_quantize(x)
    assert a[0] == 1.0 and np.array_equal(p, bp)
    codes = np.stack([p >> 4, p & 15], 1).reshape(-1)
    idx = np.nonzero(keep)[0]
    d = np.abs(exact[keep][:, None].astype(np.float32) - golden_levels()[None, :])
    ties = d[np.arange(idx.size), idx] == d[np.arange(idx.size), idx + 1]
    assert ties.any()
    assert np.array_equal(codes[1:1 + idx.size][ties], idx[ties].astype(np.uint8))


def test_quantize_zero_block_partial_block_and_odd_tail():
    x = np.zeros(64 + 5, dtype=np.float32)
    x[64:] = [0.5, -1.0, 0.25, 0.0, 1.0]
    p, a = oracle.quantize(x)
    assert a[0] == 0 and np.all(p[:32] == 0x77)                # zero block: absmax 0, code 7
    assert a[1] == 1.0                                         # max over the 5 present elements
    assert p.size == 35 and (p[-1] & 15) == 7 and (p[-1] >> 4) == 15
    assert np.all(oracle.dequantize(p, a, 69, out_dtype=oracle.FP32)[:64] == 0)


def test_quantize_dequantize_is_idempotent():
    x = synth.gaussian_weights(64 * 500 + 21, 0.02, 5, outlier_p=0.001)
    p, a = oracle.quantize(x)
    y = oracle.dequantize(p, a, x.size, out_dtype=oracle.FP32)
    p2, a2 = oracle.quantize(y)
    assert np.array_equal(p2, p) and np.array_equal(a2, a)     # +-1 level present in every block
    # through fp16 the codes survive; absmax becomes its fp16 rounding
    y16 = f16(oracle.dequantize(p, a, x.size)).astype(np.float32)
    p3, a3 = oracle.quantize(y16)
    assert np.array_equal(p3, p)
    assert np.array_equal(a3, a.astype(np.float16).astype(np.float32))


def test_quantisation_error_is_within_half_the_level_gap():
    x = synth.gaussian_weights(64 * 2000, 0.02, 6)
    p, a = oracle.quantize(x)
    y = oracle.dequantize(p, a, x.size, out_dtype=oracle.FP32)
    half_gap = np.diff(golden_levels().astype(np.float64)).max() / 2
    assert np.all(np.abs(y.astype(np.float64) - x) <= np.repeat(a, 64) * (half_gap + 1e-6))
    assert np.array_equal(a, np.abs(x.reshape(-1, 64)).max(axis=1))


# ------------------------------------------------------------ double quant

def test_dq_decode_exhaustive_codes():
    # decoder contract: code2[q] * scale2[group] + offset, two rounded fp32 ops
    code2 = np.linspace(-1, 1, 256).astype(np.float32) ** 3
    for s2, off in ((0.37, 0.05), (1e-3, -2.0), (5.0, 0.0)):
        q8 = np.tile(np.arange(256, dtype=np.uint8), 3)
        scale2 = np.array([s2, 2 * s2, -s2], dtype=np.float32)
        got = oracle.dq_decode(q8, scale2, np.array([off], np.float32), code2)
        want = (code2[q8] * np.repeat(scale2, 256)).astype(np.float32) + np.float32(off)
        assert np.array_equal(got, want.astype(np.float32))


def test_dq_encode_invariants():
    nb = 15626                                                  # 1 000 003 elements -> 62 groups, last has 10
    absmax = synth.positive_scales(nb, seed=21, lo=0.03, hi=0.09)
    q8, scale2, offset, code2 = oracle.dq_encode(absmax)
    assert scale2.size == 62 and q8.size == nb
    assert np.array_equal(code2, ((np.arange(256) - 127) / 127).astype(np.float32))
    assert offset[0] == np.float32(absmax.astype(np.float64).sum() / nb)
    dec = oracle.dq_decode(q8, scale2, offset, code2)
    grp = np.arange(nb) // 256
    assert np.all(dec[q8 == 127] == offset[0])
    for g in range(62):
        m = grp == g
        d = np.abs(absmax[m] - offset[0])
        assert scale2[g] == d.max()
        top = np.argmax(d)
        assert q8[m][top] in (0, 254)                          # group extreme -> full-scale code
        assert dec[m][top] == np.float32(np.float32(code2[q8[m][top]] * scale2[g]) + offset[0])
    assert q8.max() <= 254
    err = np.abs(dec.astype(np.float64) - absmax)
    assert np.all(err <= np.repeat(scale2, 256)[:nb] / 254 + 1e-7)


def test_dq_encode_constant_and_negative():
    q8, scale2, offset, code2 = oracle.dq_encode(np.full(300, 0.25, np.float32))
    assert np.all(q8 == 127) and np.all(scale2 == 0) and offset[0] == 0.25
    assert np.all(oracle.dq_decode(q8, scale2, offset, code2) == 0.25)
    # a negative reconstructed scale is not clamped: it flips the sign of the block
    packed = np.full(32, 0xFF, np.uint8)
    out = oracle.dequantize_dq(packed, np.array([0], np.uint8), np.array([2.0], np.float32),
                               np.array([0.5], np.float32), code2, 64, out_dtype=oracle.FP32)
    assert np.all(out == -1.5)


def test_dequantize_dq_equals_decode_then_dequantize():
    n = 1_000_003
    x = synth.gaussian_weights(n, 0.02, 31)
    p, a = oracle.quantize(x)
    q8, s2, off, c2 = oracle.dq_encode(a)
    a_dec = oracle.dq_decode(q8, s2, off, c2)
    for dt in (oracle.FP16, oracle.BF16):
        assert np.array_equal(oracle.dequantize_dq(p, q8, s2, off, c2, n, out_dtype=dt),
                              oracle.dequantize(p, a_dec, n, out_dtype=dt))
    # and with library routines
    codes = np.stack([p >> 4, p & 15], 1).reshape(-1)[:n]
    w = golden_levels()[codes] * np.repeat(a_dec, 64)[:n]
    want = torch.from_numpy(w).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.dequantize_dq(p, q8, s2, off, c2, n, out_dtype=oracle.BF16), want)


# --------------------------------------------------------------------- GEMV

def _small_gemv_case(N=24, K=256, B=3, seed=41):
    w = synth.gaussian_weights(N * K, 0.015, seed)
    p, a = oracle.quantize(w)
    q8, s2, off, c2 = oracle.dq_encode(a)
    x = synth.activations_fp16(B, K, seed + 1)
    return p, q8, s2, off, c2, x


def test_gemv_equals_float64_matmul_of_dequantized_weights():
    N, K, B = 24, 256, 3
    p, q8, s2, off, c2, x = _small_gemv_case(N, K, B)
    w = oracle.dequantize_dq(p, q8, s2, off, c2, N * K, out_dtype=oracle.FP32).reshape(N, K)
    y_bits, y64 = oracle.dequant_gemv(p, q8, s2, off, c2, N, K, x.view(np.uint16))
    want = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.allclose(y64, want, rtol=1e-12, atol=1e-12)
    assert np.array_equal(y_bits, want.astype(np.float32).astype(np.float16).view(np.uint16))


def test_gemv_unit_vector_zero_and_all_ones_cases():
    N, K = 16, 128
    p, q8, s2, off, c2, _ = _small_gemv_case(N, K, 1)
    w = oracle.dequantize_dq(p, q8, s2, off, c2, N * K, out_dtype=oracle.FP32).reshape(N, K)
    for k in (0, 1, 63, 64, 127):
        e = np.zeros((1, K), np.float16)
        e[0, k] = 1
        _, y64 = oracle.dequant_gemv(p, q8, s2, off, c2, N, K, e.view(np.uint16))
        assert np.array_equal(y64[0], w[:, k].astype(np.float64))          # column k of W
    _, y0 = oracle.dequant_gemv(p, q8, s2, off, c2, N, K, np.zeros((1, K), np.uint16))
    assert np.all(y0 == 0)
    # all codes 15 with scale exactly 1 -> y = sum(x)
    ones_p = np.full(N * K // 2, 0xFF, np.uint8)
    nb = N * K // 64
    c2 = ((np.arange(256) - 127) / 127).astype(np.float32)
    x = synth.activations_fp16(2, K, 43)
    _, ys = oracle.dequant_gemv(ones_p, np.full(nb, 254, np.uint8), np.ones(1, np.float32),
                                np.zeros(1, np.float32), c2, N, K, x.view(np.uint16))
    assert np.allclose(ys, x.astype(np.float64).sum(axis=1, keepdims=True).repeat(N, 1), rtol=0, atol=1e-12)


def test_gemv_row_range_is_a_slice_of_the_whole():
    N, K, B = 24, 256, 3
    p, q8, s2, off, c2, x = _small_gemv_case(N, K, B)
    yb, y64 = oracle.dequant_gemv(p, q8, s2, off, c2, N, K, x.view(np.uint16))
    rb, r64 = oracle.dequant_gemv_rows(p, q8, s2, off, c2, N, K, x.view(np.uint16), 5, 7)
    assert np.array_equal(rb, yb[:, 5:12]) and np.array_equal(r64, y64[:, 5:12])


def test_zero_level_times_negative_scale_is_negative_zero():
    # IEEE: (+0) * (negative) = -0; the multiply is a lone FP32 product, never "+ 0"
    packed = np.full(32, 0x77, np.uint8)
    out = oracle.dequantize(packed, np.array([-2.0], np.float32), 64)
    assert np.all(out == 0x8000)
    outb = oracle.dequantize(packed, np.array([-2.0], np.float32), 64, out_dtype=oracle.BF16)
    assert np.all(outb == 0x8000)


def test_gemm_equals_float64_matmul_of_fp16_dequantized_weights():
    # the dequantise-to-FP16-then-matmul flow, rewritten with library routines
    N, K, B = 24, 256, 5
    p, q8, s2, off, c2, x = _small_gemv_case(N, K, B, seed=51)
    w16 = f16(oracle.dequantize_dq(p, q8, s2, off, c2, N * K, out_dtype=oracle.FP16)).reshape(N, K)
    _, y64 = oracle.dequant_gemm_rows(p, q8, s2, off, c2, N, K, x.view(np.uint16), 0, N)
    want = x.astype(np.float64) @ w16.astype(np.float64).T
    assert np.allclose(y64, want, rtol=1e-12, atol=1e-12)
    _, part = oracle.dequant_gemm_rows(p, q8, s2, off, c2, N, K, x.view(np.uint16), 3, 4)
    assert np.array_equal(part, y64[:, 3:7])
    # unit vector -> the FP16 dequantised column, exactly
    e = np.zeros((1, K), np.float16)
    e[0, 77] = 1
    _, col = oracle.dequant_gemm_rows(p, q8, s2, off, c2, N, K, e.view(np.uint16), 0, N)
    assert np.array_equal(col[0], w16[:, 77].astype(np.float64))
    # and it differs from the unrounded GEMV where rounding the weights matters
    _, y_exact = oracle.dequant_gemv(p, q8, s2, off, c2, N, K, x.view(np.uint16))
    assert not np.array_equal(y_exact, y64) and np.allclose(y_exact, y64, rtol=0, atol=2e-3 * np.abs(y64).max())


# ---------------------------------------------- the data type as a parameter (Sec. V-A)

def e2m1_codebook():
    """The 4-bit float of the OCP microscaling format family (1 sign, 2 exponent, 1 mantissa bit), decoded
    from its definition and normalised to [-1, 1]: code = s e e m; e = 0 is subnormal (m / 2), else
    (1 + m / 2) * 2^(e - 1)."""
    vals = []
    for code in range(16):
        s, e, m = code >> 3, (code >> 1) & 3, code & 1
        mag = 0.5 * m if e == 0 else (1.0 + 0.5 * m) * 2.0 ** (e - 1)
        vals.append(-mag if s else mag)
    return (np.array(vals, dtype=np.float64) / 6.0).astype(np.float32)


def test_e2m1_codebook_is_the_published_value_set():
    t = e2m1_codebook().astype(np.float64) * 6.0
    assert np.allclose(t[:8], [0, 0.5, 1, 1.5, 2, 3, 4, 6], atol=1e-6) and np.allclose(t[8:], -t[:8], atol=1e-6)
    assert np.signbit(e2m1_codebook()[8]) and not np.signbit(e2m1_codebook()[0])      # -0 and +0 are two codes
    assert np.array_equal(synth.e2m1_codebook().view(np.uint32), e2m1_codebook().view(np.uint32))   # the shared input


def test_codebook_functions_with_the_nf4_table_are_the_nf4_functions():
    rng = np.random.Generator(np.random.PCG64(41))
    n = 64 * 300 + 37
    w = (rng.standard_normal(n) * 0.02).astype(np.float32)
    t = oracle.table()
    p, a = oracle.quantize(w)
    p2, a2 = oracle.quantize_codebook(w, t)
    assert np.array_equal(p, p2) and np.array_equal(a.view(np.uint32), a2.view(np.uint32))
    for dt in (oracle.FP16, oracle.BF16, oracle.FP32):
        assert np.array_equal(oracle.dequantize(p, a, n, out_dtype=dt).view(np.uint8),
                              oracle.dequantize_codebook(p, a, t, n, out_dtype=dt).view(np.uint8))
    dq = oracle.dq_encode(a)
    dq2 = oracle.dq_encode_group(a, 256)
    for x, y in zip(dq, dq2):
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8))
    assert np.array_equal(oracle.dequantize_dq(p, *dq, n, out_dtype=oracle.BF16),
                          oracle.dequantize_dq_codebook(p, *dq, 256, t, n, out_dtype=oracle.BF16))


def test_codebook_dequantize_with_a_counting_table_returns_the_codes():
    # table[i] = i and scale 1: the output IS the code sequence, high nibble first (Algorithm 1),
    # whatever the NF4 levels are
    rng = np.random.Generator(np.random.PCG64(42))
    n = 1001
    packed = rng.integers(0, 256, (n + 1) // 2, dtype=np.uint8)
    counting = np.arange(16, dtype=np.float32)
    out = oracle.dequantize_codebook(packed, np.ones(oracle.nblocks(n), np.float32), counting, n, out_dtype=oracle.FP32)
    codes = np.stack([packed >> 4, packed & 15], axis=1).ravel()[:n]
    assert np.array_equal(out, codes.astype(np.float32))
    # and with per-block scales 2^b (exact products): block b of 128 elements is scaled by its own entry
    scales = (2.0 ** (np.arange(oracle.nblocks(n, 128)) % 5)).astype(np.float32)
    out = oracle.dequantize_codebook(packed, scales, counting, n, blocksize=128, out_dtype=oracle.FP32)
    assert np.array_equal(out, codes.astype(np.float32) * np.repeat(scales, 128)[:n])


def test_codebook_quantize_is_brute_force_nearest_with_ties_to_the_lower_code():
    t = e2m1_codebook()
    rng = np.random.Generator(np.random.PCG64(43))
    n = 64 * 40
    w = (rng.standard_normal(n) * 0.3).astype(np.float32)
    w[5] = 0.0                                     # +0 / -0 levels tie: the lower code (0) wins
    w[64:128] = 0.0                                # an all-zero block
    # exact midpoints between neighbouring levels (1/12 between 0 and 1/12 ... in a block with absmax 1)
    w[128] = 1.0
    w[129:133] = [1.0 / 24, 3.0 / 24, 0.75, -0.75]
    p, a = oracle.quantize_codebook(w, t)
    codes = np.stack([p >> 4, p & 15], axis=1).ravel()[:n]
    blocks = w.reshape(-1, 64)
    amax = np.abs(blocks).max(axis=1)
    assert np.array_equal(a, amax)
    safe = np.where(amax == 0, np.float32(1), amax)[:, None]
    xn = (blocks / safe).astype(np.float32)
    dist = np.abs(xn[:, :, None] - t[None, None, :]).astype(np.float32)
    brute = dist.argmin(axis=2).ravel()            # numpy's argmin returns the first minimum
    assert np.array_equal(codes, brute)
    assert codes[5] == 0 and np.all(codes[64:128] == 0)
    # odd n: the unused nibble holds the code nearest to zero (for this table code 0, for NF4 code 7)
    p_odd, _ = oracle.quantize_codebook(w[:7], t)
    assert p_odd[3] & 15 == 0
    p_nf4, _ = oracle.quantize_codebook(w[:7], oracle.table())
    assert p_nf4[3] & 15 == 7


@pytest.mark.parametrize("group", [1, 16, 64, 256, 1024])
def test_dq_encode_group_sizes(group):
    rng = np.random.Generator(np.random.PCG64(44 + group))
    nb = 3 * 1024 + 77
    a = np.abs(rng.standard_normal(nb) * 0.01 + 0.05).astype(np.float32)
    q8, s2, off, c2 = oracle.dq_encode_group(a, group)
    ng = (nb + group - 1) // group
    assert s2.size == ng and q8.size == nb
    assert off[0] == np.float32(a.astype(np.float64).sum() / nb)
    pad = np.full(ng * group - nb, off[0], np.float32)
    centred = np.abs(np.concatenate([a, pad]) - off[0]).astype(np.float32).reshape(ng, group)
    assert np.array_equal(s2, centred.max(axis=1))                           # each group has its own scale
    # decoder formula (two separately rounded FP32 operations) and its error bound of half a code step
    dec = (c2[q8] * np.repeat(s2, group)[:nb]).astype(np.float32) + off[0]
    bound = np.repeat(s2, group)[:nb].astype(np.float64) / 254.0 + 1e-7
    assert np.all(np.abs(dec.astype(np.float64) - a) <= bound)
    if group == 1:                                                           # closed form: every block is its own extreme
        assert set(np.unique(q8)) <= {0, 127, 254}
        assert np.array_equal(q8 == 254, a > off[0])


def test_dequantize_dq_codebook_equals_decode_then_dequantize():
    rng = np.random.Generator(np.random.PCG64(45))
    t = e2m1_codebook()
    n = 128 * 70 + 5
    w = (rng.standard_normal(n) * 0.02).astype(np.float32)
    p, a = oracle.quantize_codebook(w, t, blocksize=128)
    for group in (16, 64):
        q8, s2, off, c2 = oracle.dq_encode_group(a, group)
        dec = (c2[q8] * np.repeat(s2, group)[:a.size]).astype(np.float32) + off[0]
        for dt in (oracle.FP16, oracle.BF16):
            want = oracle.dequantize_codebook(p, dec, t, n, blocksize=128, out_dtype=dt)
            got = oracle.dequantize_dq_codebook(p, q8, s2, off, c2, group, t, n, blocksize=128, out_dtype=dt)
            assert np.array_equal(want, got)


def test_codebook_gemv_and_gemm_are_float64_matmuls_of_the_codebook_weights():
    """The fused products for any table and group size: with the NF4 table and groups of 256 they are the NF4
    functions bit for bit; with another table, block size and group size they equal a float64 matmul of the weights
    that dequantize_dq_codebook yields (FP32 for the GEMV, rounded to FP16 for the GEMM), a unit vector picks
    a column exactly, and a row range is a slice of the whole."""
    N, K, B = 24, 256, 3
    p, q8, s2, off, c2, x = _small_gemv_case(N, K, B, seed=61)
    xb = x.view(np.uint16)
    for rnd, plain in ((False, oracle.dequant_gemv_rows), (True, oracle.dequant_gemm_rows)):
        yb, y64 = plain(p, q8, s2, off, c2, N, K, xb, 0, N)
        cb, c64 = oracle.dequant_gemv_rows_codebook(p, q8, s2, off, c2, 256, oracle.table(), N, K, xb, 0, N,
                                                    round_weights_to_fp16=rnd)
        assert np.array_equal(yb, cb) and np.array_equal(y64, c64)
    t = e2m1_codebook()
    rng = np.random.Generator(np.random.PCG64(62))
    N, K, bs, group = 20, 512, 128, 4
    w = (rng.standard_normal(N * K) * 0.02).astype(np.float32)
    p, a = oracle.quantize_codebook(w, t, blocksize=bs)
    q8, s2, off, c2 = oracle.dq_encode_group(a, group)
    x = synth.activations_fp16(B, K, 63)
    xb = x.view(np.uint16)
    w32 = oracle.dequantize_dq_codebook(p, q8, s2, off, c2, group, t, N * K, blocksize=bs, out_dtype=oracle.FP32)
    w16 = f16(oracle.dequantize_dq_codebook(p, q8, s2, off, c2, group, t, N * K, blocksize=bs, out_dtype=oracle.FP16))
    for rnd, wref in ((False, w32), (True, w16)):
        wref = wref.reshape(N, K).astype(np.float64)
        yb, y64 = oracle.dequant_gemv_rows_codebook(p, q8, s2, off, c2, group, t, N, K, xb, 0, N, blocksize=bs,
                                                    round_weights_to_fp16=rnd)
        want = x.astype(np.float64) @ wref.T
        assert np.allclose(y64, want, rtol=1e-12, atol=1e-12)
        assert np.array_equal(yb, want.astype(np.float32).astype(np.float16).view(np.uint16))
        e = np.zeros((1, K), np.float16)
        e[0, 300] = 1
        _, col = oracle.dequant_gemv_rows_codebook(p, q8, s2, off, c2, group, t, N, K, e.view(np.uint16), 0, N,
                                                   blocksize=bs, round_weights_to_fp16=rnd)
        assert np.array_equal(col[0], wref[:, 300])
        _, part = oracle.dequant_gemv_rows_codebook(p, q8, s2, off, c2, group, t, N, K, xb, 7, 5, blocksize=bs,
                                                    round_weights_to_fp16=rnd)
        assert np.array_equal(part, y64[:, 7:12])
    # the rounding flag matters: the two products differ, slightly
    _, a64 = oracle.dequant_gemv_rows_codebook(p, q8, s2, off, c2, group, t, N, K, xb, 0, N, blocksize=bs)
    _, b64 = oracle.dequant_gemv_rows_codebook(p, q8, s2, off, c2, group, t, N, K, xb, 0, N, blocksize=bs,
                                               round_weights_to_fp16=True)
    assert not np.array_equal(a64, b64) and np.allclose(a64, b64, rtol=0, atol=2e-3 * np.abs(a64).max())
