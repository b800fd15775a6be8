"""Helpers for the GPU parity tests: device buffers from numpy arrays, guard
words after outputs, and bit-level comparison that treats any NaN as NaN."""
import numpy as np
import torch

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
