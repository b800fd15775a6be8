"""GPU parity for the format with the data type as a parameter (Sec. V-A): any 16-entry codebook, any
block size and any second-level group size, through the C-ABI against the CPU oracle.  Dequantisation is
bit-exact; the reference quantiser gives identical codes and scales (offset within 1 ulp as for NF4: it is
bit-exact here too because both sum in double in index order)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_02556_amd import binding as nf4
from paper_2604_02556_amd import synth
from gpu_util import bits, dev, guard_intact, mismatches, out_buffer

pytestmark = pytest.mark.gpu

DT = {"fp16": (torch.float16, oracle.FP16), "bf16": (torch.bfloat16, oracle.BF16)}


def codebooks():
    rng = np.random.Generator(np.random.PCG64(77))
    shuffled = synth.e2m1_codebook().copy()
    rng.shuffle(shuffled)
    return {
        "e2m1": synth.e2m1_codebook(),                                   # FP4-style: sign-magnitude order, +0 and -0
        "nf4": oracle.table(),
        "linear": np.linspace(-1.0, 1.0, 16, dtype=np.float32),
        "unsorted_wide": (shuffled * np.float32(3.0e4)).astype(np.float32),   # levels far outside [-1, 1]
    }


@pytest.mark.parametrize("name", ["e2m1", "nf4", "linear", "unsorted_wide"])
@pytest.mark.parametrize("blocksize", [64, 128, 512, 4096])
@pytest.mark.parametrize("dt", ["fp16", "bf16"])
def test_dequantize_codebook_bit_exact(name, blocksize, dt):
    tdt, odt = DT[dt]
    cb = codebooks()[name]
    n = 2048 * 5 + 1234 + (1 if blocksize == 128 else 0)          # several tiles, a ragged end, once an odd n
    packed = synth.random_codes((n + 1) // 2, seed=blocksize + len(name))
    absmax = synth.positive_scales(oracle.nblocks(n, blocksize), seed=7, lo=1e-3, hi=4.0)
    want = oracle.dequantize_codebook(packed, absmax, cb, n, blocksize=blocksize, out_dtype=odt)
    whole, out = out_buffer(n, tdt)
    nf4.nf4_dequantize_codebook(dev(packed), dev(absmax), dev(cb), blocksize, n, out)
    torch.cuda.synchronize()
    assert mismatches(bits(out), want, dt == "bf16") == 0
    assert guard_intact(whole, n)


def test_null_codebook_is_nf4():
    n = 2048 * 3 + 77
    packed = synth.random_codes((n + 1) // 2, seed=1)
    absmax = synth.positive_scales(oracle.nblocks(n), seed=2)
    whole, out = out_buffer(n, torch.float16)
    nf4.nf4_dequantize_codebook(dev(packed), dev(absmax), None, 64, n, out)
    torch.cuda.synchronize()
    assert np.array_equal(bits(out), oracle.dequantize(packed, absmax, n))


@pytest.mark.parametrize("group", [1, 16, 64, 256, 4096])
@pytest.mark.parametrize("blocksize", [64, 256, 2048])
def test_dequantize_dq_codebook_group_sizes_bit_exact(group, blocksize):
    cb = codebooks()["e2m1"]
    n = blocksize * 300 + 2048 * 2 + 99
    w = synth.gaussian_weights(n, 0.02, seed=group + blocksize)
    packed, absmax = oracle.quantize_codebook(w, cb, blocksize=blocksize)
    q8, s2, off, c2 = oracle.dq_encode_group(absmax, group)
    for dt in ("fp16", "bf16"):
        tdt, odt = DT[dt]
        want = oracle.dequantize_dq_codebook(packed, q8, s2, off, c2, group, cb, n, blocksize=blocksize, out_dtype=odt)
        whole, out = out_buffer(n, tdt)
        nf4.nf4_dequantize_dq_codebook(dev(packed), dev(q8), dev(s2), dev(off), dev(c2), group, dev(cb), blocksize, n,
                                       out)
        torch.cuda.synchronize()
        assert mismatches(bits(out), want, dt == "bf16") == 0
        assert guard_intact(whole, n)


@pytest.mark.parametrize("name", ["e2m1", "linear", "unsorted_wide", "nf4"])
@pytest.mark.parametrize("blocksize,group", [(64, 256), (128, 64), (1024, 16), (64, 1)])
def test_quantize_ref_codebook_matches_oracle(name, blocksize, group):
    cb = codebooks()[name]
    n = blocksize * 257 + 31                                        # a partial last block, odd n, > 1 group
    w = synth.gaussian_weights(n, 0.02, seed=3 * blocksize + group)
    w[:blocksize] = 0.0                                             # an all-zero block
    w[blocksize] = 0.0
    p_ref, a_ref = oracle.quantize_codebook(w, cb, blocksize=blocksize)
    q8_ref, s2_ref, off_ref, c2_ref = oracle.dq_encode_group(a_ref, group)
    bufs = nf4.alloc_quantized(n, blocksize=blocksize, dq=True, dq_group=group)
    nf4.nf4_quantize_ref_codebook(dev(w), n, blocksize, dev(cb), group, bufs["packed"], bufs["absmax"],
                                  bufs["absmax_q8"], bufs["scale2"], bufs["offset"], bufs["code2"])
    torch.cuda.synchronize()
    host = {k: v.cpu().numpy() for k, v in bufs.items()}
    assert np.array_equal(host["packed"], p_ref)
    assert np.array_equal(host["absmax"].view(np.uint32), a_ref.view(np.uint32))
    assert np.array_equal(host["offset"].view(np.uint32), off_ref.view(np.uint32))
    assert np.array_equal(host["scale2"].view(np.uint32), s2_ref.view(np.uint32))
    assert np.array_equal(host["absmax_q8"], q8_ref)
    assert np.array_equal(host["code2"].view(np.uint32), c2_ref.view(np.uint32))


def test_round_trip_through_both_directions_on_the_gpu():
    """quantise (codebook, group) -> dequantise on the GPU equals the same two steps in the oracle."""
    cb = codebooks()["e2m1"]
    n, blocksize, group = 4096 * 9 + 640, 128, 64
    w = synth.gaussian_weights(n, 0.015, seed=12)
    bufs = nf4.alloc_quantized(n, blocksize=blocksize, dq=True, dq_group=group)
    dcb = dev(cb)
    nf4.nf4_quantize_ref_codebook(dev(w), n, blocksize, dcb, group, bufs["packed"], bufs["absmax"],
                                  bufs["absmax_q8"], bufs["scale2"], bufs["offset"], bufs["code2"])
    whole, out = out_buffer(n, torch.bfloat16)
    nf4.nf4_dequantize_dq_codebook(bufs["packed"], bufs["absmax_q8"], bufs["scale2"], bufs["offset"], bufs["code2"],
                                   group, dcb, blocksize, n, out)
    torch.cuda.synchronize()
    p, a = oracle.quantize_codebook(w, cb, blocksize=blocksize)
    dq = oracle.dq_encode_group(a, group)
    want = oracle.dequantize_dq_codebook(p, *dq, group, cb, n, blocksize=blocksize, out_dtype=oracle.BF16)
    assert np.array_equal(bits(out), want)
    assert guard_intact(whole, n)
