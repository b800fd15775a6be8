"""Helpers for the GPU parity tests: device buffers from numpy arrays, guard
words after outputs, and bit-level comparison that treats any NaN as NaN."""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

import oracle

from paper_2604_02556_amd import binding as nf4

GUARD = 64                      # 16-bit guard words after the last output element
CANARY = 0x7A5C


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def out_buffer(n, dtype):
    """n outputs followed by GUARD canary words; returns (whole, view of the n outputs)."""
    whole = torch.full((n + GUARD,), CANARY, dtype=torch.int16, device="cuda")
    return whole, whole[:n].view(dtype)


def bits(t):
    """uint16 bit patterns of an fp16/bf16/int16 tensor, on the host."""
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def guard_intact(whole, n):
    return bool((whole[n:] == CANARY).all().item())


def is_nan16(b, bf16):
    b = b.astype(np.uint32)
    if bf16:
        return ((b & 0x7F80) == 0x7F80) & ((b & 0x007F) != 0)
    return ((b & 0x7C00) == 0x7C00) & ((b & 0x03FF) != 0)


def mismatches(got_bits, want_bits, bf16=False):
    """Number of elements whose bits differ, NaNs of any payload counted equal."""
    diff = got_bits != want_bits
    both_nan = is_nan16(got_bits, bf16) & is_nan16(want_bits, bf16)
    return int((diff & ~both_nan).sum())


def dequantize_gpu(packed, absmax, n, dtype, blocksize=64):
    whole, out = out_buffer(n, dtype)
    nf4.nf4_dequantize(dev(packed) if n else None, dev(absmax) if n else None, blocksize, n, out)
    torch.cuda.synchronize()
    return whole, bits(out)


def dequantize_dq_gpu(packed, q8, scale2, offset, code2, n, dtype, blocksize=64):
    whole, out = out_buffer(n, dtype)
    nf4.nf4_dequantize_dq(dev(packed), dev(q8), dev(scale2), dev(offset), dev(code2), blocksize, n, out)
    torch.cuda.synchronize()
    return whole, bits(out)


ORACLE_THREADS = max(1, min(16, os.cpu_count() or 1))


def oracle_dequantize_threaded(packed, absmax, n, out_dtype=oracle.FP16, blocksize=64):
    """oracle.dequantize over the whole tensor, split on block boundaries over host threads (the C routine runs
    without the interpreter lock): every element of a full-size tensor in well under a second."""
    out = np.empty(n, dtype=np.uint16)
    nb = (n + blocksize - 1) // blocksize
    per = (nb + ORACLE_THREADS - 1) // ORACLE_THREADS * blocksize        # whole quantisation blocks per thread
    with ThreadPoolExecutor(max_workers=ORACLE_THREADS) as pool:
        jobs = [pool.submit(oracle.dequantize_range, packed, absmax, lo, min(per, n - lo), out, blocksize, out_dtype)
                for lo in range(0, n, per)]
        for j in jobs:
            j.result()
    return out


def oracle_rows_threaded(fn, host, N, K, x_bits, rows_per_job=64):
    """fn = oracle.dequant_gemv_rows or oracle.dequant_gemm_rows over ALL rows of the matrix, a slice of rows per
    job on the host threads.  Returns the double-precision sums, float64[B][N]."""
    B = x_bits.size // K
    ref = np.empty((B, N), dtype=np.float64)

    def job(r0):
        cnt = min(rows_per_job, N - r0)
        _, y64 = fn(host["packed"], host["absmax_q8"], host["scale2"], host["offset"], host["code2"], N, K, x_bits,
                    int(r0), int(cnt))
        ref[:, r0:r0 + cnt] = y64

    with ThreadPoolExecutor(max_workers=ORACLE_THREADS) as pool:
        for j in [pool.submit(job, r0) for r0 in range(0, N, rows_per_job)]:
            j.result()
    return ref
