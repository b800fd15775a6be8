"""GPU parity: nf4_quantize_ref (codes, absmax and the second-level encoding)
against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_02556_amd import binding as nf4
from paper_2604_02556_amd import synth
from gpu_util import dev

pytestmark = pytest.mark.gpu


def quantize_gpu(w, blocksize=64, dq=False):
    n = w.size
    bufs = nf4.alloc_quantized(n, blocksize, dq)
    for t in bufs.values():
        t.view(torch.uint8).fill_(0xCD)
    if dq:
        nf4.nf4_quantize_ref(dev(w), n, blocksize, bufs["packed"], bufs["absmax"], bufs["absmax_q8"],
                             bufs["scale2"], bufs["offset"], bufs["code2"])
    else:
        nf4.nf4_quantize_ref(dev(w), n, blocksize, bufs["packed"], bufs["absmax"])
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in bufs.items()}


@pytest.mark.parametrize("n,seed", [(1024 * 1024, 0), (1, 1), (2, 2), (63, 3), (65, 4), (4097, 5), (1_000_003, 6)])
def test_codes_and_absmax_match(n, seed):
    w = synth.gaussian_weights(n, 0.02, seed, outlier_p=0.001)
    p, a = oracle.quantize(w)
    g = quantize_gpu(w)
    assert np.array_equal(g["absmax"][:a.size], a)
    assert np.array_equal(g["packed"][:p.size], p)


def test_zero_blocks_midpoints_and_other_blocksizes():
    t = oracle.table().astype(np.float64)
    mids = ((t[:-1] + t[1:]) / 2).astype(np.float32)
    w = synth.gaussian_weights(64 * 64, 0.02, 9)
    w[64:128] = 0.0                                    # an all-zero block
    w[128] = 1.0
    w[129:129 + mids.size] = mids                      # exact midpoints where representable
    for bs in (64, 128, 4096):
        p, a = oracle.quantize(w, bs)
        g = quantize_gpu(w, bs)
        assert np.array_equal(g["absmax"][:a.size], a) and np.array_equal(g["packed"][:p.size], p)


@pytest.mark.parametrize("n", [64 * 300, 1_000_003, 64 * 256 * 9 + 64])
def test_double_quant_outputs_match(n):
    w = synth.gaussian_weights(n, 0.02, seed=n % 1000)
    p, a = oracle.quantize(w)
    q8, s2, off, c2 = oracle.dq_encode(a)
    g = quantize_gpu(w, dq=True)
    assert np.array_equal(g["packed"][:p.size], p) and np.array_equal(g["absmax"][:a.size], a)
    assert np.array_equal(g["code2"], c2)
    assert g["offset"][0] == off[0]
    assert np.array_equal(g["scale2"][:s2.size], s2)
    assert np.array_equal(g["absmax_q8"][:q8.size], q8)


@pytest.mark.parametrize("nb", [256 * 37 + 19, 70_001])      # one workgroup / slices summed by many workgroups
@pytest.mark.parametrize("kind", ["narrow", "wide", "tiny_and_huge", "subnormal", "zeros", "inexact_sum"])
def test_mean_offset_equals_the_sequential_double_sum_for_any_spread_of_scales(kind, nb):
    """The offset is float(sum / nb) with the sum a double-precision sum in index order.  The kernel adds in
    parallel when it can prove that every order gives the same (exact) sum, and in index order otherwise; either
    way the bits must be the oracle's.  Scales that span few binades (exact), span 2^100 (inexact: the order
    matters), are subnormal, are all zero, or are chosen so that rounding in the sum really happens."""
    rng = np.random.Generator(np.random.PCG64(11))
    if kind == "narrow":                                # the usual case: every order of summation is exact
        mag = rng.uniform(0.03, 0.09, nb).astype(np.float32)
    elif kind == "wide":
        mag = np.exp2(rng.uniform(-60, 40, nb)).astype(np.float32)
    elif kind == "tiny_and_huge":
        mag = np.where(rng.random(nb) < 0.5, np.float32(1e-30), np.float32(3e8)).astype(np.float32)
        mag *= rng.uniform(1, 2, nb).astype(np.float32)
    elif kind == "subnormal":
        mag = (rng.integers(1, 1 << 20, nb).astype(np.uint32)).view(np.float32)      # subnormal FP32 values
    elif kind == "zeros":
        mag = np.zeros(nb, np.float32)
    else:                                               # 2^30 next to values with all 24 bits set around 1
        mag = rng.uniform(0.5, 2.0, nb).astype(np.float32)
        mag[::97] = np.float32(2.0 ** 31)
    w = np.zeros(nb * 64, np.float32)
    w[::64] = mag * rng.choice([-1.0, 1.0], nb).astype(np.float32)                   # block i has absmax mag[i]
    p, a = oracle.quantize(w)
    assert np.array_equal(a, mag)
    q8, s2, off, c2 = oracle.dq_encode(a)
    # the oracle's offset is the plain sequential sum (pinned here against numpy's own sequential accumulate)
    seq = np.float32(np.add.accumulate(mag.astype(np.float64))[-1] / nb) if nb else np.float32(0)
    assert off[0] == seq
    g = quantize_gpu(w, dq=True)
    assert g["offset"].view(np.uint32)[0] == off.view(np.uint32)[0]
    assert np.array_equal(g["scale2"][:s2.size].view(np.uint32), s2.view(np.uint32))
    assert np.array_equal(g["absmax_q8"][:q8.size], q8)
