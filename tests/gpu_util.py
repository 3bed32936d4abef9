"""Helpers shared by the GPU parity tests: device buffers through torch, bf16 packing, comparisons."""
import numpy as np

from paper_2102_10485_amd import synth


def torch_mod():
    import torch
    return torch


def dev(a):
    """numpy array -> device tensor (same bits)."""
    torch = torch_mod()
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


def to_bf16_bits(a):
    """fp32 -> bf16 bits, round to nearest even (the format's published definition)."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def from_bf16_bits(b):
    return (np.ascontiguousarray(b).astype(np.uint32) << 16).view(np.float32)


def round_to(a, bf16):
    return from_bf16_bits(to_bf16_bits(a)) if bf16 else np.asarray(a, np.float32)


def pack(a, bf16):
    return to_bf16_bits(a) if bf16 else np.ascontiguousarray(a, np.float32)


def unpack(t, bf16, shape):
    a = t.cpu().numpy()
    if bf16:
        return from_bf16_bits(a.view(np.uint16)).reshape(shape)
    return a.reshape(shape)


def rel_l2(a, b, floor=0.0):
    a, b = np.asarray(a, np.float64).ravel(), np.asarray(b, np.float64).ravel()
    den = max(np.linalg.norm(b), floor)
    return np.linalg.norm(a - b) / den if den > 0 else np.linalg.norm(a - b)
