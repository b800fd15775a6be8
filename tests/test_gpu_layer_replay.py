"""GPU parity for the decoder-layer replay that bench.py times (Sec. III-C: a quantised linear layer dequantises
the weight into an FP16 temporary, then multiplies): the seven Qwen3-32B-shaped projections, double-quantised
scales, in the calls and shapes of the bench leg.

  * nf4_dequantize_dq into the reused FP16 temporary: every element against the oracle, bit for bit;
  * nf4_dequant_gemm, both algorithms (single kernel, and split along K with a workspace shared by the seven
    calls as in the bench), at 8 and 64 tokens: sampled rows of every projection against the oracle's
    double-precision sums over FP16-rounded weights (dequant_gemm_rows), to the GEMM's bar."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_02556_amd import binding as nf4
from paper_2604_02556_amd import synth
from gpu_util import oracle_dequantize_threaded

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def layer():
    """The layer as bench.py builds it: N(0, 0.02^2) weights drawn on the GPU, quantised by nf4_quantize_ref."""
    gen = torch.Generator(device="cuda")
    tensors = []
    for ti, (name, (N, K)) in enumerate(synth.QWEN3_32B.items()):
        n = N * K
        gen.manual_seed(8000 + ti)
        w = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, synth.QWEN3_32B_SIGMA, generator=gen)
        b = nf4.alloc_quantized(n, 64, dq=True)
        nf4.nf4_quantize_ref(w, n, 64, b["packed"], b["absmax"], b["absmax_q8"], b["scale2"], b["offset"], b["code2"])
        torch.cuda.synchronize()
        del w
        host = {k: v.cpu().numpy() for k, v in b.items()}
        tensors.append((name, N, K, b, host))
    return tensors


def test_dequantize_dq_into_the_reused_temporary_is_bit_exact(layer):
    wtmp = torch.empty(max(N * K for _, N, K, _, _ in layer), dtype=torch.float16, device="cuda")
    for name, N, K, b, host in layer:
        n = N * K
        nf4.nf4_dequantize_dq(b["packed"], b["absmax_q8"], b["scale2"], b["offset"], b["code2"], 64, n, wtmp)
        torch.cuda.synchronize()
        scales = oracle.dq_decode(host["absmax_q8"], host["scale2"], host["offset"], host["code2"])
        want = oracle_dequantize_threaded(host["packed"], scales, n, out_dtype=oracle.FP16)
        got = wtmp[:n].view(torch.int16).cpu().numpy().view(np.uint16)
        bad = int(np.count_nonzero(got != want))
        assert bad == 0, f"{name}: {bad} of {n} elements differ from the oracle"


@pytest.mark.parametrize("B", [8, 64])
@pytest.mark.parametrize("split", [False, True])
def test_fused_gemm_on_every_projection(layer, B, split):
    xs = {K: synth.activations_fp16(B, K, seed=8100 + B + K % 13) for K in {t[2] for t in layer}}
    ws = None
    if split:
        ws = torch.full((max(nf4.nf4_dequant_gemm_workspace_bytes(N, K, B) for _, N, K, _, _ in layer) // 4,),
                        float("nan"), dtype=torch.float32, device="cuda")
    for name, N, K, b, host in layer:
        x = xs[K]
        y = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
        nf4.nf4_dequant_gemm(b["packed"], b["absmax_q8"], b["scale2"], b["offset"], b["code2"], 64, N, K,
                             torch.from_numpy(x).cuda(), B, y, workspace=ws)
        torch.cuda.synchronize()
        yh = y.cpu().numpy().astype(np.float64)
        assert np.isfinite(yh).all(), name
        rng = np.random.Generator(np.random.PCG64(N + K + B))
        rows = np.unique(np.concatenate([np.arange(3), np.arange(N - 3, N), rng.integers(0, N, 10)]))
        ref = np.empty((B, rows.size))
        for j, r in enumerate(rows):
            _, r64 = oracle.dequant_gemm_rows(host["packed"], host["absmax_q8"], host["scale2"], host["offset"],
                                              host["code2"], N, K, x.view(np.uint16), int(r), 1)
            ref[:, j] = r64[:, 0]
        err = np.abs(yh[:, rows] - ref)
        rms = np.sqrt(np.mean(ref ** 2))
        assert np.all(err <= 1e-2 * np.abs(ref) + 1e-2 * rms), name
        rel = err.max() / np.abs(ref).max()
        print(f"{name} {N}x{K} B={B} split={split}: max err / max |y| = {rel:.2e}")
        assert rel < 2e-3, name
