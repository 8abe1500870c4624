"""The scattered-tensor sweep: many fp32 master tensors of skewed sizes, each
contributing one 2-D strided sub-slice, listed in a random wire order.

The literal recipe (100,000 sizes log-uniform on [4 KiB, 64 MiB]) averages
6.9 MB per tensor, i.e. ~690 GB, which contradicts its own "~40 GB" and exceeds
one GPU's memory.  Sizes are therefore drawn from the tilted density
p(s) ~ s^-(1+alpha) on the same interval; alpha = 0.55 gives a mean of ~391 KB
(~39 GB for 100,000 tensors).  alpha = 0 is the literal log-uniform.

What is returned is an *input description*: a list of caller-defined segments
(tensor, element offset, row stride, rows, row length) in wire order, exactly
what a caller hands to the library's explicit-segment entry point and to the
oracle.  No wire offsets, no chunking, no narrowing here.
"""
import numpy as np
import torch


def _tilted_sizes(rng, n, lo, hi, alpha):
    u = rng.random(n)
    if alpha == 0.0:
        s = lo * (hi / lo) ** u
    else:
        s = (lo ** -alpha - u * (lo ** -alpha - hi ** -alpha)) ** (-1.0 / alpha)
    s = (np.floor(s / 4.0).astype(np.int64)) * 4
    return np.clip(s, int(lo), int(hi)).astype(np.int64)


def scatter_description(n_tensors, seed, min_bytes=4096, max_bytes=64 << 20, alpha=0.55):
    """Returns a dict of int64 arrays.

    Per tensor i (index order = allocation order in the source pool):
      n_elems[i]            fp32 elements of the tensor (tensor bytes / 4)
      row_stride[i]         S_i, the row stride in elements of the matrix the storage holds
      r0, nr, c0, nc        the sub-slice: rows [r0, r0+nr), cols [c0, c0+nc)
    Wire order:
      perm[k]               the tensor whose slice is k-th on the wire
    Destination arena (one dense bf16 tensor, slices in index order, no padding):
      arena_off[i]          element offset of slice i; arena_elems = total
    Segment list in wire order (k = 0..n-1), ready for the explicit-segment API:
      seg_src_tensor, seg_src_off, seg_src_stride, seg_dst_off, seg_dst_stride,
      seg_nrows, seg_row_len
    """
    rng = np.random.default_rng(seed)
    size_bytes = _tilted_sizes(rng, n_tensors, float(min_bytes), float(max_bytes), alpha)
    n = size_bytes // 4
    # row stride: log-uniform integer in [16, min(n, 16384)], not forced to a multiple of 4
    s_hi = np.minimum(n, 16384).astype(np.float64)
    S = np.floor(16.0 * (s_hi / 16.0) ** rng.random(n_tensors)).astype(np.int64)
    S = np.clip(S, 16, np.minimum(n, 16384))
    R = n // S
    nr = rng.integers((R + 1) // 2, R + 1)
    nc = rng.integers((S + 1) // 2, S + 1)
    r0 = rng.integers(0, R - nr + 1)
    c0 = rng.integers(0, S - nc + 1)
    perm = rng.permutation(n_tensors).astype(np.int64)
    slice_elems = nr * nc
    arena_off = np.concatenate(([0], np.cumsum(slice_elems)[:-1])).astype(np.int64)
    d = dict(n_elems=n, row_stride=S, r0=r0, nr=nr, c0=c0, nc=nc, perm=perm,
             arena_off=arena_off, arena_elems=int(slice_elems.sum()),
             pool_off=np.concatenate(([0], np.cumsum(n)[:-1])).astype(np.int64),
             pool_elems=int(n.sum()))
    d["seg_src_tensor"] = perm.copy()
    d["seg_src_off"] = (r0 * S + c0)[perm]
    d["seg_src_stride"] = S[perm]
    d["seg_dst_off"] = arena_off[perm]
    d["seg_dst_stride"] = nc[perm]
    d["seg_nrows"] = nr[perm]
    d["seg_row_len"] = nc[perm]
    return d


def scatter_values(n_elems, seed, device="cpu", special_rate=0.01):
    """fp32 N(0,1) pool with `special_rate` of the elements replaced by edge
    bit patterns: +-Inf, NaNs (quiet, signalling, payload only in the low half),
    subnormals, bf16 rounding midpoints and their neighbours, values next to
    FLT_MAX.  Returned as a float32 torch tensor on `device`."""
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 7919 + 17)
    out = torch.empty(n_elems, dtype=torch.float32, device=device)
    bits = out.view(torch.int32)
    step = 1 << 26
    for lo in range(0, n_elems, step):
        m = min(n_elems, lo + step) - lo
        out[lo:lo + m] = torch.randn(m, dtype=torch.float32, device=device, generator=g)
        sel = torch.rand(m, device=device, generator=g) < special_rate
        kind = torch.randint(0, 10, (m,), device=device, generator=g)
        r = torch.randint(0, 1 << 31, (m,), device=device, generator=g, dtype=torch.int64)
        r = r | (torch.randint(0, 2, (m,), device=device, generator=g, dtype=torch.int64) << 31)
        hi16 = r & 0xFFFF0000
        sign = r & 0x80000000
        pat = torch.zeros(m, dtype=torch.int64, device=device)
        pat = torch.where(kind == 0, sign | 0x7F800000, pat)                           # +-Inf
        pat = torch.where(kind == 1, sign | 0x7FC00000 | (r & 0x003FFFFF), pat)        # quiet NaN, random payload
        pat = torch.where(kind == 2, sign | 0x7F800000 | ((r & 0x003FFFFF) | 1), pat)  # signalling NaN
        pat = torch.where(kind == 3, sign | 0x7F800000 | ((r & 0xFFFF) | 1), pat)      # NaN, payload in low half only
        pat = torch.where(kind == 4, sign | (r & 0x007FFFFF), pat)                     # subnormal (or zero)
        pat = torch.where(kind == 5, hi16 | 0x8000, pat)                               # exact midpoint
        pat = torch.where(kind == 6, hi16 | 0x7FFF, pat)                               # just below midpoint
        pat = torch.where(kind == 7, hi16 | 0x8001, pat)                               # just above midpoint
        pat = torch.where(kind == 8, sign | 0x7F7FFFFF - (r & 0x3), pat)               # next to FLT_MAX
        pat = torch.where(kind == 9, sign | 0x7F7F0000 | (r & 0xFFFF), pat)            # rounds to max finite or Inf
        pat = pat & 0xFFFFFFFF
        pat32 = (pat - ((pat >> 31) << 32)).to(torch.int32)
        chunk = bits[lo:lo + m]
        chunk[sel] = pat32[sel]
    return out
