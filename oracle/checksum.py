"""Oracle: per-tensor checksum of a (holder -> reader) wire stream.

The paper attaches a checksum of each tensor to the published reference and
validates it after transfer; it is computed on the GPU and overlapped with the
transfer (Sec. 4.6).  It does not say which function.  The reading used here is
a position-weighted pair of 64-bit sums over the tensor's run on the wire, chosen
because every term depends only on (position, value), so any number of workers
can add their terms in any order:

    the run of holder tensor t = its payload bytes on the wire (gap excluded),
    read as little-endian 16-bit units h_0 .. h_{n-1};
        A_t = sum_k h_k                 (mod 2^64)
        B_t = sum_k (k + 1) * h_k       (mod 2^64)

Holder tensors that send nothing have A = B = 0.  The pack side computes the pair
from what it writes, the unpack side from what it reads; equal pairs mean the run
arrived intact and in order.  Test infrastructure only.
"""
import numpy as np

from . import reshard

MASK = (1 << 64) - 1


def run_checksum(run_bytes):
    """(A, B) of one run given as a uint8 array of even length."""
    h = np.ascontiguousarray(run_bytes).view("<u2").astype(np.uint64)
    k1 = np.arange(1, len(h) + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        a = int(h.sum(dtype=np.uint64))
        b = int((h * k1).sum(dtype=np.uint64))
    return a & MASK, b & MASK


def model_checksums(model, src, dst, wire, n_src_tensors, narrow_at="pack"):
    """(A, B) per holder tensor for the stream `wire` of the pair (src, dst)."""
    out = np.zeros((n_src_tensors, 2), dtype=np.uint64)
    spans = {}
    for it in reshard.plan_items(model, src, dst, narrow_at):
        n = len(it["src_r"]) * len(it["src_c"]) * reshard.ESIZE[it["wire_dtype"]]
        lo, hi = spans.get(it["src_id"], (it["wire_off"], it["wire_off"]))
        spans[it["src_id"]] = (min(lo, it["wire_off"]), max(hi, it["wire_off"] + n))
    for t, (lo, hi) in spans.items():
        out[t] = run_checksum(wire[lo:hi])
    return out


def segment_checksums(segs, offs, dst_dtype, wire, n_src_tensors):
    """Same for an explicit-segment plan; offs = per-segment wire offsets.  A tensor's run is the
    consecutive segments that name it (segments of one tensor that are not adjacent in wire order
    form separate runs whose sums add up, each counted from its own start)."""
    es = {"bf16": 2, "f32": 4}
    out = np.zeros((n_src_tensors, 2), dtype=np.uint64)
    k, n = 0, len(offs)
    while k < n:
        t = int(segs["src_tensor"][k])
        lo = int(offs[k])
        hi = lo
        while k < n and int(segs["src_tensor"][k]) == t:
            d = dst_dtype if isinstance(dst_dtype, str) else dst_dtype[k]
            hi = int(offs[k]) + int(segs["nrows"][k]) * int(segs["row_len"][k]) * es[d]
            k += 1
        a, b = run_checksum(wire[lo:hi])
        with np.errstate(over="ignore"):
            out[t, 0] += np.uint64(a)
            out[t, 1] += np.uint64(b)
    return out
