"""Plumbing for the GPU parity tests: host <-> device conversion only (no method arithmetic)."""
import numpy as np
import torch

from oracle import l2l_oracle as O


def to_dev(a, dtype):
    """numpy array -> device tensor in 'fp32', 'bf16' or 'fp16' (the 16-bit ones by the oracle's own rounding)."""
    a = np.ascontiguousarray(a, np.float32)
    if dtype == "fp32":
        return torch.from_numpy(a).cuda()
    if dtype == "fp16":
        bits = O.fp16_bits(a).view(np.int16).reshape(a.shape)
        return torch.from_numpy(bits).cuda().view(torch.float16)
    bits = O.bf16_bits(a).astype(np.int16).reshape(a.shape)
    return torch.from_numpy(bits).cuda().view(torch.bfloat16)


def to_host(t):
    """device tensor -> float64 numpy."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def rounded(a, dtype):
    """The values the device will actually hold, as float64."""
    a = np.asarray(a, np.float32)
    if dtype == "fp16":
        return O.fp16_round(a).astype(np.float64)
    return (O.bf16_round(a) if dtype == "bf16" else a).astype(np.float64)


def pinned(a):
    t = torch.from_numpy(np.ascontiguousarray(a)).pin_memory()
    return t
