"""GPU parity: the tuned quantiser nf4_quantize against the CPU oracle, bit for
bit, with inputs aimed at its threshold table (values within a few ulps of every
decision boundary, found here by bisection with the oracle itself)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_02556_amd import binding as nf4
from paper_2604_02556_amd import synth
from gpu_util import dev

pytestmark = pytest.mark.gpu


def quantize_gpu(w, blocksize=64):
    n = w.size
    bufs = nf4.alloc_quantized(n, blocksize)
    for t in bufs.values():
        t.view(torch.uint8).fill_(0xCD)
    nf4.nf4_quantize(dev(w), n, blocksize, bufs["packed"], bufs["absmax"])
    torch.cuda.synchronize()
    return bufs["packed"].cpu().numpy()[:(n + 1) // 2], bufs["absmax"].cpu().numpy()[:oracle.nblocks(n, blocksize)]


def oracle_code_of(xn):
    """Code the oracle gives a value in a block whose absmax is exactly 1."""
    blk = np.zeros(64, np.float32)
    blk[0] = 1.0
    blk[1] = xn
    p, a = oracle.quantize(blk)
    assert a[0] == 1.0
    return int(p[0] & 15)


def decision_boundaries():
    """For each pair of adjacent levels the smallest float32 the oracle maps to the upper one."""
    t = oracle.table()

    def key(f):
        u = int(np.float32(f).view(np.uint32))
        return -(u & 0x7FFFFFFF) if u >> 31 else u

    def unkey(k):
        u = (0x80000000 | -k) if k < 0 else k
        return np.uint32(u).view(np.float32)

    out = []
    for k in range(15):
        lo, hi = key(t[k]), key(t[k + 1])
        while hi - lo > 1:
            mid = (lo + hi) // 2
            if oracle_code_of(unkey(mid)) >= k + 1:
                hi = mid
            else:
                lo = mid
        out.append(unkey(hi))
    return np.array(out, dtype=np.float32)


@pytest.mark.parametrize("n,seed", [(1024 * 1024, 0), (2048, 1), (2047, 2), (2049, 3), (64, 4), (65, 5), (1, 6),
                                    (1_000_003, 7), (64 * 1024 * 1024, 8)])
def test_codes_and_absmax_match_the_oracle(n, seed):
    w = synth.gaussian_weights(n, 0.02, seed, outlier_p=0.001)
    p, a = oracle.quantize(w)
    gp, ga = quantize_gpu(w)
    assert np.array_equal(ga, a)
    assert np.array_equal(gp, p)


def test_values_around_every_decision_boundary():
    theta = decision_boundaries()
    near = []
    for th in theta:
        v = np.float32(th)
        for _ in range(3):
            v = np.nextafter(v, np.float32(-2))
        for _ in range(7):
            near.append(v)
            v = np.nextafter(v, np.float32(2))
    near = np.array(near, dtype=np.float32)                       # 105 values, within 3 ulps of a boundary
    # blocks with absmax exactly 1, then the same normalised values under other scales
    blocks = []
    for scale in (1.0, 0.5, 0.37, 3.0, 1e-3, 0.0152587890625, 123.456):
        vals = (near.astype(np.float64) * scale).astype(np.float32)
        for s in range(0, vals.size, 63):
            blk = np.zeros(64, np.float32)
            blk[0] = np.float32(scale)
            chunk = vals[s:s + 63]
            blk[1:1 + chunk.size] = chunk
            blocks.append(blk)
    w = np.concatenate(blocks * 40)                               # > one 2048-element tile, many times over
    p, a = oracle.quantize(w)
    gp, ga = quantize_gpu(w)
    assert np.array_equal(ga, a) and np.array_equal(gp, p)


def test_zero_blocks_exact_levels_and_extremes():
    t = oracle.table()
    w = synth.gaussian_weights(2048 * 6, 0.02, 11)
    w[64:192] = 0.0                                               # all-zero blocks -> absmax 0, code 7
    w[2048:2048 + 16] = t                                         # the levels themselves, absmax 1
    w[4096] = 3e38
    w[4096 + 64] = 1e-38
    w[4096 + 128:4096 + 192] = -7.0                               # constant block: every code 0
    p, a = oracle.quantize(w)
    gp, ga = quantize_gpu(w)
    assert np.array_equal(ga, a) and np.array_equal(gp, p)


@pytest.mark.parametrize("blocksize", [128, 4096])
def test_other_blocksizes_with_a_ragged_end(blocksize):
    w = synth.gaussian_weights(4096 * 5 + 300, 0.02, blocksize)
    p, a = oracle.quantize(w, blocksize)
    gp, ga = quantize_gpu(w, blocksize)
    assert np.array_equal(ga, a) and np.array_equal(gp, p)


def test_tuned_equals_reference_on_a_70b_gate_projection():
    n = synth.numel(synth.LLAMA33_70B["gate"])
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    w = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, synth.LLAMA33_70B_SIGMA, generator=g)
    ref = nf4.alloc_quantized(n)
    tuned = nf4.alloc_quantized(n)
    nf4.nf4_quantize_ref(w, n, 64, ref["packed"], ref["absmax"])
    nf4.nf4_quantize(w, n, 64, tuned["packed"], tuned["absmax"])
    torch.cuda.synchronize()
    assert torch.equal(ref["absmax"], tuned["absmax"])
    assert torch.equal(ref["packed"], tuned["packed"])


@pytest.mark.parametrize("blocksize", [128, 256, 512, 1024, 2048, 4096])
@pytest.mark.parametrize("n", [2048 * 37, 2048 * 5 + 4096 + 17, 2048, 100])
def test_other_block_sizes_match_the_oracle(blocksize, n):
    """Blocks of 128 to 4096 in the tuned kernel (cross-row, cross-load and, for 4096, cross-wave maxima), ragged
    ends included; codes and scales are the oracle's."""
    w = synth.gaussian_weights(n, 0.02, seed=blocksize + n % 101, outlier_p=0.002)
    w[2048:2048 + 64] = 0.0                                  # zeros inside a larger block
    if n >= 2048 * 5:
        w[4096:4096 + blocksize] = 0.0                       # an all-zero block
        w[3 * 2048 - 1] = 7.5                                # the maximum as the last element of a tile
        w[2 * 2048] = -9.25                                  # ... and as the first, negative
    p, a = oracle.quantize(w, blocksize)
    gp, ga = quantize_gpu(w, blocksize)
    assert np.array_equal(ga.view(np.uint32), a.view(np.uint32))
    assert np.array_equal(gp, p)


@pytest.mark.parametrize("group", [256, 64, 1])
@pytest.mark.parametrize("n", [64 * 256 * 5 + 64 * 7, 1_000_003])
def test_tuned_quantiser_followed_by_the_second_level_equals_the_oracle(n, group):
    """nf4_quantize + nf4_dq_encode: the tuned first level and the second level as separate calls give the
    oracle's codes, scale codes, second-level scales, offset and map bit for bit."""
    w = synth.gaussian_weights(n, 0.02, seed=n % 977)
    p, a = oracle.quantize(w)
    q8, s2, off, c2 = oracle.dq_encode_group(a, group)
    bufs = nf4.alloc_quantized(n, 64, dq=True, dq_group=group)
    for t in bufs.values():
        t.view(torch.uint8).fill_(0xCD)
    nf4.nf4_quantize(dev(w), n, 64, bufs["packed"], bufs["absmax"])
    nf4.nf4_dq_encode(bufs["absmax"], a.size, group, bufs["absmax_q8"], bufs["scale2"], bufs["offset"], bufs["code2"])
    torch.cuda.synchronize()
    g = {k: v.cpu().numpy() for k, v in bufs.items()}
    assert np.array_equal(g["packed"][:p.size], p) and np.array_equal(g["absmax"][:a.size], a)
    assert np.array_equal(g["absmax_q8"][:q8.size], q8)
    assert np.array_equal(g["scale2"][:s2.size].view(np.uint32), s2.view(np.uint32))
    assert g["offset"].view(np.uint32)[0] == off.view(np.uint32)[0]
    assert np.array_equal(g["code2"].view(np.uint32), c2.view(np.uint32))


@pytest.mark.parametrize("blocksize", [64, 128, 256, 512, 1024, 2048, 4096])
@pytest.mark.parametrize("n", [1, 2, 3, 63, 65, 127, 2047, 2049, 4095, 4097, 6143, 8191, 8193, 2048 * 9 + 1031, 1_000_003])
def test_ragged_sizes_write_nothing_past_the_end(n, blocksize):
    """Sizes that do not fill a tile (Sec. V-A), for every block size: the predicated tile of the tuned kernel
    gives the oracle's codes and scales -- a partial last block takes the maximum of the elements present, the
    unused nibble of an odd n the zero level's code -- and leaves the bytes after packed[ceil(n/2) - 1] and
    absmax[nb - 1] alone."""
    w = synth.gaussian_weights(n, 0.02, seed=n + blocksize, outlier_p=0.002)
    p, a = oracle.quantize(w, blocksize)
    guard = 256
    packed = torch.full((p.size + guard,), 0xCD, dtype=torch.uint8, device="cuda")
    absmax = torch.full((a.size + guard,), -123.0, dtype=torch.float32, device="cuda")
    nf4.nf4_quantize(dev(w), n, blocksize, packed, absmax)
    torch.cuda.synchronize()
    gp, ga = packed.cpu().numpy(), absmax.cpu().numpy()
    assert np.array_equal(ga[:a.size].view(np.uint32), a.view(np.uint32))
    assert np.array_equal(gp[:p.size], p)
    assert np.all(gp[p.size:] == 0xCD) and np.all(ga[a.size:] == -123.0)
