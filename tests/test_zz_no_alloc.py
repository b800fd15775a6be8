"""GPU test of nf4_dequant_gemv_static, the entry point that allocates nothing: called through the raw C-ABI
(ctypes on libnf4.so, device addresses as integers), its output must equal nf4_dequant_gemv_ws's bit for bit (the
same kernels in the same order; only the home of the partial sums differs), and both must be inside the GEMV's bar
against the double-precision oracle.  Two calls in a row share the library's static scratch array, the second with
a smaller input, so that whatever the first left behind must not show in the second.  Collected last on purpose."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2604_02556_amd import binding as nf4
from paper_2604_02556_amd import synth
from gpu_util import dev

pytestmark = pytest.mark.gpu

STATIC_SCRATCH_BYTES = 4 << 20                      # NF4_STATIC_SCRATCH_BYTES of include/nf4.h


def make_case(N, K, seed):
    w = synth.gaussian_weights(N * K, 0.015, seed)
    p, a = oracle.quantize(w)
    return (p,) + tuple(oracle.dq_encode(a))


def run_both(L, N, K, B, seed):
    """One call of each entry point on the same inputs, through the C-ABI; returns (static, ws, oracle sums)."""
    case = make_case(N, K, seed)
    x = synth.activations_fp16(B, K, seed=seed + 1)
    d = [dev(a) for a in case]
    dx = dev(x)
    stream = torch.cuda.current_stream().cuda_stream
    y_static = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
    y_ws = torch.full((B, N), float("nan"), dtype=torch.float16, device="cuda")
    ws_bytes = L.nf4_dequant_gemv_workspace_bytes(N, K, B)
    assert 0 < ws_bytes <= STATIC_SCRATCH_BYTES
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    args = [t.data_ptr() for t in d] + [64, N, K, dx.data_ptr(), B]
    rc = L.nf4_dequant_gemv_static(*args, y_static.data_ptr(), stream)
    assert rc == 0, nf4.status_string(rc)
    rc = L.nf4_dequant_gemv_ws(*args, y_ws.data_ptr(), ws.data_ptr(), ws_bytes, stream)
    assert rc == 0, nf4.status_string(rc)
    torch.cuda.synchronize()
    _, ref = oracle.dequant_gemv(*case, N, K, x.view(np.uint16))
    return y_static.cpu().numpy(), y_ws.cpu().numpy(), ref


def check(y_static, y_ws, ref):
    assert np.array_equal(y_static.view(np.uint16), y_ws.view(np.uint16))
    err = np.abs(y_static.astype(np.float64) - ref)
    assert np.all(err <= 1e-2 * np.abs(ref) + 1e-2 * np.sqrt(np.mean(ref ** 2)))
    assert err.max() / np.abs(ref).max() < 2e-3


def test_static_scratch_matches_workspace_on_two_calls_in_a_row():
    L = nf4.lib()
    # first call: K split 16 ways, 16 tokens, ragged N (partial sums fill 16 * 16 * 300 floats of the array)
    check(*run_both(L, N=300, K=8192, B=16, seed=901))
    # second call, smaller: fewer rows, fewer tokens, fewer splits -- it must not see the first call's sums
    check(*run_both(L, N=70, K=2048 + 512, B=5, seed=903))
    # and a token count that runs on the FMA kernels (no partial sums at all)
    check(*run_both(L, N=33, K=1024, B=2, seed=905))


def test_every_accepted_shape_fits_the_static_array_on_this_device():
    """K is split at most as many ways as fill the compute units once, so the partial sums of any shape stay inside
    the array on a part with up to 256 compute units; the size check in the entry point (NF4_ERR_SIZE) is for
    devices with more.  Host arithmetic only: no launch."""
    L = nf4.lib()
    rng = np.random.Generator(np.random.PCG64(77))
    shapes = [(8192, 28672), (28672, 8192), (1, 64), (255, 1 << 20), (256, 1 << 20), (257, 1 << 20), (65536, 65536),
              (65535, 4096), (1 << 22, 64), (2 ** 31 - 1, 64)]
    shapes += [(int(rng.integers(1, 1 << 18)), 64 * int(rng.integers(1, 1 << 12))) for _ in range(2000)]
    worst = 0
    for N, K in shapes:
        for B in (3, 16):
            need = L.nf4_dequant_gemv_workspace_bytes(N, K, B)
            assert 0 < need <= STATIC_SCRATCH_BYTES, (N, K, B, need)
            worst = max(worst, need)
    assert worst == STATIC_SCRATCH_BYTES                 # reached by 8192 x 28672 at 16 tokens
