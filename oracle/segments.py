"""Oracle for caller-defined segment lists (the scattered-tensor sweep).

A segment names a 2-D strided slice of a source tensor and of a destination
tensor: nrows rows of row_len elements, row r starting at element
off + r*row_stride on either side.  Segments are given in wire order.  On the
wire every segment is dense (row after row) and already in the destination
dtype; a segment whose source tensor differs from the previous segment's starts
at the next 16-byte boundary, the gap being zero.  Chunking as for model plans.
With narrow_at="unpack" the wire carries the source dtype and the reader converts
(pass the source dtype as the wire dtype to wire_offsets).
Test infrastructure only.
"""
import numpy as np

from . import rne

ESIZE = {"bf16": 2, "f32": 4}
NPBITS = {"bf16": np.uint16, "f32": np.uint32}


def _dt(d, k):
    """dtype of segment k: one name for all segments, or one per segment."""
    return d if isinstance(d, str) else d[k]


def wire_offsets(segs, dst_dtype):
    """Byte offset of each segment on the wire, and the stream length (dst_dtype: the wire's dtype)."""
    off = 0
    offs = np.zeros(len(segs["src_tensor"]), dtype=np.int64)
    prev = None
    for k in range(len(offs)):
        t = int(segs["src_tensor"][k])
        if t != prev:
            off = (off + 15) // 16 * 16
            prev = t
        offs[k] = off
        off += int(segs["nrows"][k]) * int(segs["row_len"][k]) * ESIZE[_dt(dst_dtype, k)]
    return offs, off


def _gather_index(off, stride, nrows, row_len):
    return (off + np.arange(nrows, dtype=np.int64)[:, None] * stride
            + np.arange(row_len, dtype=np.int64)[None, :])


def segment_wire(segs, k, src_tensors, src_dtype, dst_dtype):
    """Elements of segment k as they appear on the wire (dst_dtype: the wire's dtype)."""
    idx = _gather_index(int(segs["src_off"][k]), int(segs["src_stride"][k]),
                        int(segs["nrows"][k]), int(segs["row_len"][k]))
    vals = src_tensors[int(segs["src_tensor"][k])][idx]
    return rne.convert(vals, _dt(src_dtype, k), _dt(dst_dtype, k)).reshape(-1)


def pack(segs, src_tensors, src_dtype, dst_dtype, narrow_at="pack"):
    wire_dtype = dst_dtype if narrow_at == "pack" else src_dtype
    offs, total = wire_offsets(segs, wire_dtype)
    wire = np.zeros(total, dtype=np.uint8)
    for k in range(len(offs)):
        w = segment_wire(segs, k, src_tensors, src_dtype, wire_dtype)
        wire[offs[k]:offs[k] + w.nbytes] = w.view(np.uint8)
    return wire


def unpack(segs, wire, dst_tensors, dst_dtype, counts=None, wire_dtype=None):
    """wire_dtype: dtype(s) the wire carries if not the destination's (narrowing at unpack)."""
    wdt_all = dst_dtype if wire_dtype is None else wire_dtype
    offs, _ = wire_offsets(segs, wdt_all)
    for k in range(len(offs)):
        nr, nc = int(segs["nrows"][k]), int(segs["row_len"][k])
        dt, wdt = _dt(dst_dtype, k), _dt(wdt_all, k)
        vals = wire[offs[k]:offs[k] + nr * nc * ESIZE[wdt]].view(NPBITS[wdt])
        vals = rne.convert(vals, wdt, dt)
        idx = _gather_index(int(segs["dst_off"][k]), int(segs["dst_stride"][k]), nr, nc)
        t = dst_tensors[int(segs["dst_tensor"][k])]
        t[idx.reshape(-1)] = vals
        if counts is not None:
            np.add.at(counts[int(segs["dst_tensor"][k])], idx.reshape(-1), 1)
