"""The library keeps no per-call state on the host (a thread-local error code, a table built once behind
std::call_once) and none on the device, so calls may be issued from several host threads and on several
streams at once.  Each worker runs its own mix of entry points on its own stream, many times, while the
others run theirs; every result must be the oracle's."""
import threading

import numpy as np
import pytest
import torch

import oracle
from paper_2604_02556_amd import binding as nf4
from paper_2604_02556_amd import synth
from gpu_util import dev

pytestmark = pytest.mark.gpu


def test_four_host_threads_on_four_streams():
    n = 64 * 3000 + 41
    N, K, B = 64, 2048, 12
    cases = []
    for i in range(4):
        w = synth.gaussian_weights(n, 0.02, seed=900 + i)
        p, a = oracle.quantize(w)
        q8, s2, off, c2 = oracle.dq_encode(a)
        wm = synth.gaussian_weights(N * K, 0.015, seed=950 + i)
        pm, am = oracle.quantize(wm)
        mq8, ms2, moff, mc2 = oracle.dq_encode(am)
        x = synth.activations_fp16(B, K, seed=970 + i)
        _, ref_mm = oracle.dequant_gemm_rows(pm, mq8, ms2, moff, mc2, N, K, x.view(np.uint16), 0, N)
        cases.append(dict(w=dev(w), p=p, a=a, want16=oracle.dequantize(p, a, n),
                          wantbf=oracle.dequantize_dq(p, q8, s2, off, c2, n, out_dtype=oracle.BF16),
                          dp=dev(p), da=dev(a), dq8=dev(q8), ds2=dev(s2), doff=dev(off), dc2=dev(c2),
                          m=[dev(v) for v in (pm, mq8, ms2, moff, mc2)], x=dev(x), ref_mm=ref_mm))
    errors = []

    def worker(i):
        try:
            c = cases[i]
            torch.cuda.set_device(0)
            st = torch.cuda.Stream()
            out16 = torch.empty(n, dtype=torch.float16, device="cuda")
            outbf = torch.empty(n, dtype=torch.bfloat16, device="cuda")
            qp = torch.empty((n + 1) // 2, dtype=torch.uint8, device="cuda")
            qa = torch.empty((n + 63) // 64, dtype=torch.float32, device="cuda")
            y = torch.empty((B, N), dtype=torch.float16, device="cuda")
            ws = torch.empty(nf4.nf4_dequant_gemm_workspace_bytes(N, K, B), dtype=torch.uint8, device="cuda")
            for rep in range(25):
                nf4.nf4_quantize(c["w"], n, 64, qp, qa, stream=st)
                nf4.nf4_dequantize(qp, qa, 64, n, out16, stream=st)
                nf4.nf4_dequantize_dq(c["dp"], c["dq8"], c["ds2"], c["doff"], c["dc2"], 64, n, outbf, stream=st)
                nf4.nf4_dequant_gemm(*c["m"], 64, N, K, c["x"], B, y, workspace=ws, stream=st)
                st.synchronize()
                assert np.array_equal(qp.cpu().numpy(), c["p"]) and np.array_equal(qa.cpu().numpy(), c["a"])
                assert np.array_equal(out16.view(torch.int16).cpu().numpy().view(np.uint16), c["want16"])
                assert np.array_equal(outbf.view(torch.int16).cpu().numpy().view(np.uint16), c["wantbf"])
                yy = y.cpu().numpy().astype(np.float64)
                assert np.abs(yy - c["ref_mm"]).max() / np.abs(c["ref_mm"]).max() < 2e-3
        except BaseException as e:                           # noqa: BLE001 - reported by the main thread
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
