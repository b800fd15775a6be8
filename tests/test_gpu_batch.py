"""GPU parity of the batched entry point: several tensors in one launch must give,
tensor by tensor, exactly what the CPU oracle gives (and so exactly what the
one-tensor entry points give), for full tiles, ragged ends, empty tensors, both
kinds of scales and both output types; nothing is written outside an output."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_02556_amd import binding as nf4
from paper_2604_02556_amd import synth
from gpu_util import dev, out_buffer, bits, guard_intact, mismatches

pytestmark = pytest.mark.gpu

SIZES = [2048 * 3 + 77, 1, 0, 2048, 63, 2048 * 40, 65, 1_000_003]      # ragged, tiny, empty, exact tiles


@pytest.mark.parametrize("dt", ["fp16", "bf16"])
@pytest.mark.parametrize("dq", [False, True])
def test_batch_of_ragged_tensors_matches_the_oracle(dt, dq):
    tdt, odt = (torch.float16, oracle.FP16) if dt == "fp16" else (torch.bfloat16, oracle.BF16)
    items, keep = [], []
    for i, n in enumerate(SIZES):
        w = synth.gaussian_weights(max(n, 1), 0.02, seed=100 + i)[:n]
        p, a = oracle.quantize(w) if n else (np.zeros(0, np.uint8), np.zeros(0, np.float32))
        whole, out = out_buffer(n, tdt)
        if dq and n:
            q8, s2, off, c2 = oracle.dq_encode(a)
            want = oracle.dequantize_dq(p, q8, s2, off, c2, n, out_dtype=odt)
            t = dict(packed=dev(p), absmax_q8=dev(q8), scale2=dev(s2), offset=dev(off), code2=dev(c2), out=out, n=n)
        else:
            want = oracle.dequantize(p, a, n, out_dtype=odt) if n else np.zeros(0, np.uint16)
            t = dict(packed=dev(p) if n else None, absmax=dev(a) if n else None, out=out, n=n)
            if dq:                                           # an empty tensor in a double-quantised batch
                t.pop("absmax")
        items.append(t)
        keep.append((whole, out, want, n))
    nf4.nf4_dequantize_batch(items, 64)
    torch.cuda.synchronize()
    for whole, out, want, n in keep:
        assert guard_intact(whole, n)
        assert mismatches(bits(out), want, dt == "bf16") == 0


def test_batch_equals_single_calls_on_a_decoder_layer_shape():
    """The seven projections of a (scaled-down) decoder layer in one launch, against seven launches."""
    shapes = [(1024, 1024), (1024, 128), (1024, 128), (1024, 1024), (1024, 3584), (1024, 3584), (3584, 1024)]
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    items, singles = [], []
    for N, K in shapes:
        n = N * K
        packed = torch.randint(0, 256, (n // 2,), dtype=torch.uint8, device="cuda", generator=g)
        absmax = torch.rand(n // 64, device="cuda", generator=g) * 0.1 + 0.001
        out = torch.zeros(n, dtype=torch.float16, device="cuda")
        ref = torch.zeros(n, dtype=torch.float16, device="cuda")
        nf4.nf4_dequantize(packed, absmax, 64, n, ref)
        items.append(dict(packed=packed, absmax=absmax, out=out, n=n))
        singles.append(ref)
    nf4.nf4_dequantize_batch(items, 64)
    torch.cuda.synchronize()
    for it, ref in zip(items, singles):
        assert torch.equal(it["out"].view(torch.int16), ref.view(torch.int16))


def test_batch_other_blocksize():
    n = 2048 * 5 + 300
    w = synth.gaussian_weights(n, 0.02, seed=3)
    p, a = oracle.quantize(w, 256)
    whole, out = out_buffer(n, torch.float16)
    nf4.nf4_dequantize_batch([dict(packed=dev(p), absmax=dev(a), out=out, n=n)], 256)
    torch.cuda.synchronize()
    assert guard_intact(whole, n)
    assert mismatches(bits(out), oracle.dequantize(p, a, n, blocksize=256)) == 0
