"""Seeded tensor values.  Input generation only: what the reshard moves, not how.

Tensors travel between torch (device memory, generation) and the numpy oracle
as raw bit patterns: uint16 for bf16, uint32 for fp32.
"""
import numpy as np
import torch

_TORCH_DTYPE = {"bf16": torch.bfloat16, "f32": torch.float32}
_BITS_DTYPE = {"bf16": (torch.int16, np.uint16), "f32": (torch.int32, np.uint32)}


def _gen(seed, index, device):
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1_000_003 + int(index)) & 0x7FFFFFFFFFFF)
    return g


def weight_values(n_elems, dtype, seed, index, device="cpu", is_norm=False):
    """Values of one registered tensor: weights ~ N(0, 0.02) drawn in fp32 and
    stored in `dtype`; normalisation weights are ones."""
    td = _TORCH_DTYPE[dtype]
    if is_norm:
        return torch.ones(n_elems, dtype=td, device=device)
    g = _gen(seed, index, device)
    out = torch.empty(n_elems, dtype=td, device=device)
    step = 1 << 26
    for lo in range(0, n_elems, step):
        hi = min(n_elems, lo + step)
        out[lo:hi] = (torch.randn(hi - lo, dtype=torch.float32, device=device, generator=g) * 0.02).to(td)
    return out


def id_pattern_values(n_elems, dtype, index, device="cpu"):
    """Debug pattern: bits are a hash of (tensor index, element index), so a
    misplaced element is visible.  NaN/Inf patterns included on purpose."""
    i = torch.arange(n_elems, dtype=torch.int64, device=device)
    h = (i * 2654435761 + (index + 1) * 40503 + (i >> 13) * 97) & 0xFFFFFFFF
    if dtype == "bf16":
        return (h & 0xFFFF).to(torch.int32).to(torch.int16).view(torch.bfloat16)
    return (h - ((h >> 31) << 32)).to(torch.int32).view(torch.float32)


def to_bits(t):
    """torch tensor (any device) -> flat numpy array of its bit patterns."""
    t = t.detach().reshape(-1)
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.view(torch.int32).cpu().numpy().view(np.uint32)
    if t.dtype == torch.uint8:
        return t.cpu().numpy()
    raise TypeError(t.dtype)


def from_bits(a, device="cpu"):
    """flat numpy bit-pattern array -> torch tensor of the float dtype."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).to(device).view(torch.float32)
    raise TypeError(a.dtype)
