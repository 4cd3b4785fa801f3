"""Helpers for the GPU parity tests: fp16 ulp distance and host<->device marshalling."""
import numpy as np


def ordered_f16(bits):
    """Monotone integer image of fp16 bit patterns (+0 and -0 both map to 0)."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.int32)
    mag = b & 0x7FFF
    return np.where(b & 0x8000, -mag, mag)


def ulp_distance(bits_a, bits_b):
    return np.abs(ordered_f16(bits_a) - ordered_f16(bits_b))


def to_dev(arr, torch, dtype=None):
    """numpy -> cuda tensor; uint16/uint32 travel as the same-width signed/fp16 views."""
    a = np.ascontiguousarray(arr)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    if a.dtype == np.uint16:
        a = a.view(np.float16)
    t = torch.from_numpy(a).cuda()
    return t


def f16_bits(t):
    """cuda fp16 tensor -> numpy uint16 bit patterns."""
    return t.detach().cpu().numpy().view(np.uint16)
