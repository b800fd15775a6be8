"""GPU parity: nf4_quantize_codebook -- the tuned quantiser for any 16 levels, whose decision thresholds are found on
the device -- against the CPU oracle's quantize_codebook, bit for bit: FP4-style E2M1 in sign-magnitude order (levels
out of order, +0 and -0), NF4 passed as a table (must equal nf4_quantize), evenly spaced levels (a threshold a few
ulps from zero), a shuffled table, tables the tuned kernel must hand to the reference kernel inside the same call
(levels too close, far outside [-1, 1] with wide gaps is fine, a non-finite level), every block size, ragged sizes
with guard bytes, NaN and infinite inputs, and values within a few ulps of every decision boundary of the table
(found here by bisection with the oracle itself)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_02556_amd import binding as nf4
from paper_2604_02556_amd import synth
from gpu_util import dev

pytestmark = pytest.mark.gpu


def tables():
    rng = np.random.Generator(np.random.PCG64(5))
    shuffled = oracle.table().copy()
    rng.shuffle(shuffled)
    close = np.linspace(-1.0, 1.0, 16, dtype=np.float32)
    close[8] = close[7] + np.float32(2.0 ** -12)                     # two levels 2^-12 apart: reference kernel
    crowded = np.array([-1, -0.7, -0.5, -0.3, -0.2, -0.1, 0.0, 0.02, 0.045, 0.07, 0.1, 0.2, 0.4, 0.6, 0.8, 1.0],
                       np.float32)                                   # two thresholds in one interval of 1/32: reference kernel
    return {
        "e2m1": synth.e2m1_codebook(),                               # sign-magnitude order, +0 and -0
        "nf4": oracle.table(),
        "linear": np.linspace(-1.0, 1.0, 16, dtype=np.float32),      # the threshold between -1/15 and 1/15 is 2^-28
        "shuffled_nf4": shuffled,
        "wide": (synth.e2m1_codebook() * np.float32(3.0)).astype(np.float32),   # half the levels are never reached
        "close": close,
        "crowded": crowded,
    }


def quantize_gpu(w, table, blocksize=64, guard=64):
    n = w.size
    nbytes, nb = (n + 1) // 2, oracle.nblocks(n, blocksize)
    packed = torch.full((nbytes + guard,), 0xCD, dtype=torch.uint8, device="cuda")
    absmax = torch.full((nb + guard,), -123.0, dtype=torch.float32, device="cuda")
    ws = torch.full((nf4.QUANTIZE_CODEBOOK_WORKSPACE_BYTES,), 0xFF, dtype=torch.uint8, device="cuda")
    nf4.nf4_quantize_codebook(dev(w), n, blocksize, dev(table), packed, absmax, ws)
    torch.cuda.synchronize()
    hp, ha = packed.cpu().numpy(), absmax.cpu().numpy()
    assert np.all(hp[nbytes:] == 0xCD) and np.all(ha[nb:] == -123.0)   # nothing written past the end
    usable = int(ws[520:524].cpu().numpy().view(np.int32)[0])          # the flag behind the 65 + 65 words of bins
    return hp[:nbytes], ha[:nb], usable


@pytest.mark.parametrize("name", ["e2m1", "nf4", "linear", "shuffled_nf4", "wide", "close", "crowded"])
@pytest.mark.parametrize("blocksize", [64, 256, 4096])
def test_codes_and_absmax_match_the_oracle(name, blocksize):
    table = tables()[name]
    n = 2048 * 21 + 1031
    w = synth.gaussian_weights(n, 0.02, seed=blocksize + len(name), outlier_p=0.001)
    w[:blocksize] = 0.0                                               # an all-zero block
    w[5000:5016] = table                                              # the levels themselves
    p, a = oracle.quantize_codebook(w, table, blocksize=blocksize)
    gp, ga, usable = quantize_gpu(w, table, blocksize)
    assert usable == (0 if name in ("close", "crowded") else 1)       # which kernel did the work
    assert np.array_equal(ga.view(np.uint32), a.view(np.uint32))
    assert np.array_equal(gp, p)


def test_nf4_table_equals_the_nf4_call_and_null_is_nf4():
    n = 1_000_003
    w = synth.gaussian_weights(n, 0.02, seed=9)
    gp, ga, _ = quantize_gpu(w, oracle.table())
    b = nf4.alloc_quantized(n, 64)
    nf4.nf4_quantize(dev(w), n, 64, b["packed"], b["absmax"])
    b2 = nf4.alloc_quantized(n, 64)
    nf4.nf4_quantize_codebook(dev(w), n, 64, None, b2["packed"], b2["absmax"], None)     # NULL table: no workspace needed
    torch.cuda.synchronize()
    assert np.array_equal(gp, b["packed"].cpu().numpy()[:(n + 1) // 2])
    assert np.array_equal(ga, b["absmax"].cpu().numpy()[:oracle.nblocks(n, 64)])
    assert torch.equal(b["packed"], b2["packed"]) and torch.equal(b["absmax"], b2["absmax"])


@pytest.mark.parametrize("name", ["e2m1", "linear", "shuffled_nf4", "wide"])
def test_values_around_every_decision_boundary(name):
    """For every pair of neighbouring values of the table, the smallest float32 that the oracle gives to the upper
    one (bisection over the number line with the oracle), then that value +- 3 ulps in blocks whose absmax is 1 and
    under other scales."""
    table = tables()[name]

    def code_of(xn):
        blk = np.zeros(64, np.float32)
        blk[0] = 1.0
        blk[1] = xn
        p, a = oracle.quantize_codebook(blk, table)
        assert a[0] == 1.0
        return int(p[0] & 15)

    def key(f):
        u = int(np.float32(f).view(np.uint32))
        return -(u & 0x7FFFFFFF) if u >> 31 else u

    def unkey(k):
        u = (0x80000000 | -k) if k < 0 else k
        return np.uint32(u).view(np.float32)

    values = np.unique(table[np.abs(table) <= 1.0])                   # ascending; -0 and +0 are one value
    near = []
    for lo_v, hi_v in zip(values[:-1], values[1:]):
        lo, hi = key(lo_v), key(hi_v)
        c_hi = code_of(hi_v)
        assert code_of(lo_v) != c_hi
        while hi - lo > 1:
            mid = (lo + hi) // 2
            if code_of(unkey(mid)) == c_hi:
                hi = mid
            else:
                lo = mid
        v = unkey(hi)
        for _ in range(3):
            v = np.nextafter(v, np.float32(-2))
        for _ in range(7):
            near.append(v)
            v = np.nextafter(v, np.float32(2))
    near = np.array(near, dtype=np.float32)
    blocks = []
    for scale in (1.0, 0.5, 0.37, 3.0, 1e-3, 0.0152587890625, 123.456):
        vals = (near.astype(np.float64) * scale).astype(np.float32)
        for s in range(0, vals.size, 63):
            blk = np.zeros(64, np.float32)
            blk[0] = np.float32(scale)
            chunk = vals[s:s + 63]
            blk[1:1 + chunk.size] = chunk
            blocks.append(blk)
    w = np.concatenate(blocks * 40)
    p, a = oracle.quantize_codebook(w, table)
    gp, ga, usable = quantize_gpu(w, table)
    assert usable == 1
    assert np.array_equal(ga.view(np.uint32), a.view(np.uint32)) and np.array_equal(gp, p)


@pytest.mark.parametrize("name", ["e2m1", "shuffled_nf4"])
def test_nan_infinite_and_extreme_inputs(name):
    table = tables()[name]
    w = synth.gaussian_weights(2048 * 4, 0.02, 13)
    w[3] = np.nan                                                     # NaN in a block: absmax ignores it, its code is 0
    w[64 * 5 + 1] = np.inf                                            # infinite absmax: finite x / inf = 0, inf / inf = NaN
    w[64 * 9:64 * 10] = -7.0                                          # constant block
    w[64 * 12] = 3e38
    w[64 * 13] = 1e-38
    w[64 * 14:64 * 15] = 1e-41                                        # subnormal block: the generic division
    p, a = oracle.quantize_codebook(w, table)
    gp, ga, usable = quantize_gpu(w, table)
    assert usable == 1
    assert np.array_equal(ga.view(np.uint32), a.view(np.uint32)) and np.array_equal(gp, p)


def test_non_finite_level_goes_to_the_reference_kernel():
    table = tables()["linear"].copy()
    table[4] = np.inf
    w = synth.gaussian_weights(2048 * 3 + 77, 0.02, 14)
    p, a = oracle.quantize_codebook(w, table)
    gp, ga, usable = quantize_gpu(w, table)
    assert usable == 0
    assert np.array_equal(ga.view(np.uint32), a.view(np.uint32)) and np.array_equal(gp, p)


@pytest.mark.parametrize("blocksize", [64, 128, 512, 1024, 2048, 4096])
@pytest.mark.parametrize("n", [1, 2, 63, 65, 2047, 2049, 8193, 2048 * 9 + 1031])
def test_ragged_sizes(n, blocksize):
    table = tables()["e2m1"]
    w = synth.gaussian_weights(n, 0.02, seed=n + blocksize)
    p, a = oracle.quantize_codebook(w, table, blocksize=blocksize)
    gp, ga, usable = quantize_gpu(w, table, blocksize)
    assert usable == 1
    assert np.array_equal(ga.view(np.uint32), a.view(np.uint32)) and np.array_equal(gp, p)


def test_workspace_checks():
    w = dev(synth.gaussian_weights(4096, 0.02, 1))
    b = nf4.alloc_quantized(4096, 64)
    t = dev(tables()["e2m1"])
    small = torch.empty(512, dtype=torch.uint8, device="cuda")
    with pytest.raises(nf4.NF4Error) as e:
        nf4.nf4_quantize_codebook(w, 4096, 64, t, b["packed"], b["absmax"], small)
    assert e.value.status == 2                                        # NF4_ERR_SIZE
    with pytest.raises(nf4.NF4Error) as e:
        nf4.nf4_quantize_codebook(w, 4096, 64, t, b["packed"], b["absmax"], None)
    assert e.value.status == 1                                        # NF4_ERR_NULL


def test_tuned_equals_reference_on_a_70b_gate_projection_with_e2m1():
    n = synth.numel(synth.LLAMA33_70B["gate"])
    g = torch.Generator(device="cuda")
    g.manual_seed(78)
    w = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, synth.LLAMA33_70B_SIGMA, generator=g)
    t = dev(tables()["e2m1"])
    ref = nf4.alloc_quantized(n)
    tuned = nf4.alloc_quantized(n)
    ws = torch.empty(nf4.QUANTIZE_CODEBOOK_WORKSPACE_BYTES, dtype=torch.uint8, device="cuda")
    nf4.nf4_quantize_ref_codebook(w, n, 64, t, 256, ref["packed"], ref["absmax"])
    nf4.nf4_quantize_codebook(w, n, 64, t, tuned["packed"], tuned["absmax"], ws)
    torch.cuda.synchronize()
    assert torch.equal(ref["absmax"], tuned["absmax"])
    assert torch.equal(ref["packed"], tuned["packed"])
