"""The library only enqueues kernels on the caller's stream (no allocation, no
synchronisation, no memset), so its calls can be captured in a HIP graph -- the
column-layout GEMV kernels, the entry point over the static scratch array and the
three-kernel quantiser for a table in device memory included.  The
graph is replayed several times with eager work and synchronisation between
the replays, and every replay must reproduce the eager results bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_02556_amd import binding as nf4
from paper_2604_02556_amd import synth
from gpu_util import dev

pytestmark = pytest.mark.gpu


def test_captured_calls_replay_bit_exactly():
    n = 64 * 4096 + 1000
    N, K, B = 96, 1024, 20
    w = synth.gaussian_weights(n, 0.02, 1)
    p, a = oracle.quantize(w)
    q8, s2, off, c2 = oracle.dq_encode(a)
    wm = synth.gaussian_weights(N * K, 0.015, 2)
    pm, am = oracle.quantize(wm)
    mq8, ms2, moff, mc2 = oracle.dq_encode(am)
    x = synth.activations_fp16(B, K, 3)

    d = {k: dev(v) for k, v in dict(p=p, a=a, q8=q8, s2=s2, off=off, c2=c2, pm=pm, mq8=mq8, ms2=ms2, moff=moff,
                                    mc2=mc2, x=x, w=w).items()}
    out16 = torch.empty(n, dtype=torch.float16, device="cuda")
    outbf = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    yv = torch.empty((8, N), dtype=torch.float16, device="cuda")
    ym = torch.empty((B, N), dtype=torch.float16, device="cuda")
    qp = torch.empty((n + 1) // 2, dtype=torch.uint8, device="cuda")
    qa = torch.empty((n + 63) // 64, dtype=torch.float32, device="cuda")
    ys = torch.empty((B, N), dtype=torch.float16, device="cuda")           # split-K GEMM: two kernels per call
    ws = torch.empty(nf4.nf4_dequant_gemm_workspace_bytes(N, K, B), dtype=torch.uint8, device="cuda")
    cb = dev(synth.e2m1_codebook())
    outcb = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    b1 = torch.empty(n, dtype=torch.float16, device="cuda")            # one launch for two tensors
    b2 = torch.empty(5000, dtype=torch.float16, device="cuda")
    yw = torch.empty((8, N), dtype=torch.float16, device="cuda")           # GEMV with a workspace: two kernels per call
    wsv = torch.empty(nf4.nf4_dequant_gemv_workspace_bytes(N, K, 8), dtype=torch.uint8, device="cuda")
    # column-layout GEMV kernels (rows of 4096 columns and more): one token, four tokens; the no-allocation entry
    N2, K2 = 70, 4096 + 64
    wm2 = synth.gaussian_weights(N2 * K2, 0.015, 4)
    pm2, am2 = oracle.quantize(wm2)
    m2 = {k: dev(v) for k, v in zip(("q8", "s2", "off", "c2"), oracle.dq_encode(am2))}
    m2["p"] = dev(pm2)
    x2 = dev(synth.activations_fp16(6, K2, 5))
    y1 = torch.empty((1, N2), dtype=torch.float16, device="cuda")
    y4 = torch.empty((4, N2), dtype=torch.float16, device="cuda")
    y6 = torch.empty((6, N2), dtype=torch.float16, device="cuda")
    # tuned quantiser for a table in device memory: three kernels, the decision thresholds in a caller workspace
    qcp = torch.empty((n + 1) // 2, dtype=torch.uint8, device="cuda")
    qca = torch.empty((n + 63) // 64, dtype=torch.float32, device="cuda")
    wsq = torch.empty(nf4.QUANTIZE_CODEBOOK_WORKSPACE_BYTES, dtype=torch.uint8, device="cuda")
    outputs = [out16, outbf, yv, ym, qp, qa, ys, outcb, b1, b2, yw, y1, y4, y6, qcp, qca]

    def run(stream):
        nf4.nf4_dequantize(d["p"], d["a"], 64, n, out16, stream=stream)
        nf4.nf4_dequantize_dq(d["p"], d["q8"], d["s2"], d["off"], d["c2"], 64, n, outbf, stream=stream)
        nf4.nf4_dequant_gemv(d["pm"], d["mq8"], d["ms2"], d["moff"], d["mc2"], 64, N, K, d["x"], 8, yv, stream=stream)
        nf4.nf4_dequant_gemm(d["pm"], d["mq8"], d["ms2"], d["moff"], d["mc2"], 64, N, K, d["x"], B, ym, stream=stream)
        nf4.nf4_quantize(d["w"], n, 64, qp, qa, stream=stream)
        nf4.nf4_dequant_gemm(d["pm"], d["mq8"], d["ms2"], d["moff"], d["mc2"], 64, N, K, d["x"], B, ys, workspace=ws,
                             stream=stream)
        nf4.nf4_dequantize_dq_codebook(d["p"], d["q8"], d["s2"], d["off"], d["c2"], 256, cb, 64, n, outcb, stream=stream)
        nf4.nf4_dequant_gemv_ws(d["pm"], d["mq8"], d["ms2"], d["moff"], d["mc2"], 64, N, K, d["x"], 8, yw, wsv,
                                stream=stream)
        nf4.nf4_dequantize_batch([dict(packed=d["p"], absmax=d["a"], out=b1, n=n),
                                  dict(packed=d["p"], absmax=d["a"], out=b2, n=5000)], 64, stream=stream)
        nf4.nf4_dequant_gemv(m2["p"], m2["q8"], m2["s2"], m2["off"], m2["c2"], 64, N2, K2, x2, 1, y1, stream=stream)
        nf4.nf4_dequant_gemv(m2["p"], m2["q8"], m2["s2"], m2["off"], m2["c2"], 64, N2, K2, x2, 4, y4, stream=stream)
        nf4.nf4_dequant_gemv_static(m2["p"], m2["q8"], m2["s2"], m2["off"], m2["c2"], 64, N2, K2, x2, 6, y6, stream=stream)
        nf4.nf4_quantize_codebook(d["w"], n, 64, cb, qcp, qca, wsq, stream=stream)

    side = torch.cuda.Stream()
    run(side)                                              # eager reference (also warms up lazy initialisation)
    side.synchronize()
    want = [t.clone() for t in outputs]
    assert np.array_equal(want[0].view(torch.int16).cpu().numpy().view(np.uint16), oracle.dequantize(p, a, n))

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(torch.cuda.current_stream())
    for replay in range(4):
        for t in outputs + [ws, wsv, wsq]:                 # eager work between replays: poison outputs and workspaces
            t.view(torch.uint8).fill_(0xA5)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outputs, want):
            assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), f"replay {replay} differs"
