"""Oracle: the reshard itself - destination shard, wire stream, chunks.

Result (definition).  For reader rank d, every element (i, j) of every
destination tensor maps through the reader's shard index to a global element
(I, J) of a logical weight; the one holder whose shard index contains (I, J)
supplies it:   dst[i, j] = convert(src[i', j']).

Wire (a reading motivated by the compaction of small tensors into contiguous
staging buffers and by the tensor-ordered prefix a reader may fetch, Sec. 4.3.2
/ 4.3.3).  For one
(holder, reader) pair the stream is, for each of the holder's registered
tensors in registration order, the elements of that tensor the reader needs,
in the tensor's row-major order, already converted to the reader's dtype
(narrow_at="pack", the default: the wire carries the narrow type) or still in
the holder's dtype (narrow_at="unpack": the reader converts).  Each tensor's run
starts at the next 16-byte boundary, the gap is zero bytes, tensors that
contribute nothing take no space.  Chunk c is stream bytes
[c*CB, min((c+1)*CB, total)).

Everything is done with index vectors and numpy fancy indexing: membership of
a global row/column in the reader's index vector decides what is sent.
Test infrastructure only.
"""
import numpy as np

from . import layouts, rne

ESIZE = {"bf16": 2, "f32": 4}
NPBITS = {"bf16": np.uint16, "f32": np.uint32}


def _align16(n):
    return (n + 15) // 16 * 16


def plan_items(model, src, dst, narrow_at="pack"):
    """What moves for the pair (holder layout src, reader layout dst).

    Yields, in wire order, one item per (holder tensor, logical tensor in it)
    that the reader needs anything of:
      src_id, dst_id        registered-tensor indices on either side
      src_r, src_c          local row / col indices (holder tensor) of the needed
                            elements; needed set = src_r x src_c, row-major
      dst_r, dst_c          local row / col indices (reader tensor) where they land
      src_dtype, dst_dtype, wire_dtype
      wire_off              byte offset of the item's first element in the stream
    and finally the total stream length via StopIteration-free helper wire_bytes().
    """
    lts = layouts.logical_tensors(model)
    src_regs = layouts.registered_tensors(model, src)
    dst_regs = layouts.registered_tensors(model, dst)
    where_dst = {}
    for did, t in enumerate(dst_regs):
        for li, row0 in t["parts"]:
            where_dst[li] = (did, row0)
    off = 0
    for sid, t in enumerate(src_regs):
        first_of_tensor = True
        for li, srow0 in t["parts"]:
            lt = lts[li]
            if li not in where_dst or not layouts.supplies(model, lt, src, dst):
                continue
            did, drow0 = where_dst[li]
            s_rows, s_cols = layouts.shard_index(model, lt, src)
            d_rows, d_cols = layouts.shard_index(model, lt, dst)
            r_need = np.isin(s_rows, d_rows) & layouts.row_supply_mask(model, lt, src, dst)
            c_need = np.isin(s_cols, d_cols)
            if not r_need.any() or not c_need.any():
                continue
            # position of a global row / col inside the reader's shard
            pos_r = np.full(lt["rows"], -1, dtype=np.int64)
            pos_r[d_rows] = np.arange(len(d_rows))
            pos_c = np.full(lt["cols"], -1, dtype=np.int64)
            pos_c[d_cols] = np.arange(len(d_cols))
            ddt = dst_regs[did]["dtype"]
            wdt = ddt if narrow_at == "pack" else t["dtype"]
            if first_of_tensor:
                off = _align16(off)
                first_of_tensor = False
            item = dict(src_id=sid, dst_id=did,
                        src_r=srow0 + np.nonzero(r_need)[0], src_c=np.nonzero(c_need)[0],
                        dst_r=drow0 + pos_r[s_rows[r_need]], dst_c=pos_c[s_cols[c_need]],
                        src_dtype=t["dtype"], dst_dtype=ddt, wire_dtype=wdt, wire_off=off, logical=li)
            off += len(item["src_r"]) * len(item["src_c"]) * ESIZE[wdt]
            yield item


def wire_bytes(model, src, dst, narrow_at="pack"):
    total = 0
    for it in plan_items(model, src, dst, narrow_at):
        total = it["wire_off"] + len(it["src_r"]) * len(it["src_c"]) * ESIZE[it["wire_dtype"]]
    return total


def item_wire(it, src_tensor):
    """The item's elements as they appear on the wire (1-D bit-pattern array)."""
    sel = src_tensor[np.ix_(it["src_r"], it["src_c"])]
    return rne.convert(sel, it["src_dtype"], it["wire_dtype"]).reshape(-1)


def pack(model, src, dst, src_tensors, narrow_at="pack"):
    """Wire stream (uint8 array) of holder `src` for reader `dst`.
    src_tensors: the holder's registered tensors as 2-D bit-pattern arrays."""
    items = list(plan_items(model, src, dst, narrow_at))
    total = 0
    for it in items:
        total = it["wire_off"] + len(it["src_r"]) * len(it["src_c"]) * ESIZE[it["wire_dtype"]]
    wire = np.zeros(total, dtype=np.uint8)
    for it in items:
        w = item_wire(it, src_tensors[it["src_id"]])
        wire[it["wire_off"]:it["wire_off"] + w.nbytes] = w.view(np.uint8)
    return wire


def unpack(model, src, dst, wire, dst_tensors, counts=None, narrow_at="pack"):
    """Scatter a received stream into the reader's registered tensors (in place).
    counts (optional, same shapes, integer): incremented once per written element."""
    for it in plan_items(model, src, dst, narrow_at):
        nr, nc = len(it["src_r"]), len(it["src_c"])
        nb = nr * nc * ESIZE[it["wire_dtype"]]
        vals = wire[it["wire_off"]:it["wire_off"] + nb].view(NPBITS[it["wire_dtype"]]).reshape(nr, nc)
        vals = rne.convert(vals, it["wire_dtype"], it["dst_dtype"])
        ix = np.ix_(it["dst_r"], it["dst_c"])
        dst_tensors[it["dst_id"]][ix] = vals
        if counts is not None:
            counts[it["dst_id"]][ix] += 1


def chunks(wire, chunk_bytes):
    """Cut the stream into wire chunks; the last one is short."""
    if chunk_bytes <= 0 or chunk_bytes % 16:
        raise ValueError("chunk size must be a positive multiple of 16")
    return [wire[o:o + chunk_bytes] for o in range(0, len(wire), chunk_bytes)]


def empty_tensors(model, lay, fill=0):
    return [np.full((t["rows"], t["cols"]), fill, dtype=NPBITS[t["dtype"]])
            for t in layouts.registered_tensors(model, lay)]


def _find_part(regs, li):
    for sid, st in enumerate(regs):
        for sli, srow0 in st["parts"]:
            if sli == li:
                return sid, srow0, st["dtype"]
    return None


def reshard_by_definition(model, holders, holder_tensors, dst):
    """The result definition, with no wire in between: assemble every logical
    weight from the holders' shards, then cut the reader's shard out of it.

    holders / holder_tensors: layouts and registered tensors (2-D bit-pattern
    arrays) of the ranks the reader pulls from.  Replicated data is taken from
    the primary holder only.  Reader elements that none of the listed holders
    keeps (experts of absent expert-parallel ranks) are left at zero and
    reported in the returned mask list as False.
    Returns (reader tensors, written masks)."""
    lts = layouts.logical_tensors(model)
    out = empty_tensors(model, dst)
    written = [np.zeros(t.shape, dtype=bool) for t in out]
    for did, t in enumerate(layouts.registered_tensors(model, dst)):
        for li, drow0 in t["parts"]:
            lt = lts[li]
            full, have, sdt = None, np.zeros((lt["rows"], lt["cols"]), dtype=np.int32), None
            for lay, tensors in zip(holders, holder_tensors):
                if not layouts.holds(model, lt, lay) or not layouts.supplies(model, lt, lay, dst):
                    continue
                sid, srow0, sdt = _find_part(layouts.registered_tensors(model, lay), li)
                rows, cols = layouts.shard_index(model, lt, lay)
                sends = layouts.row_supply_mask(model, lt, lay, dst)  # partly replicated rows: one sender
                if full is None:
                    full = np.zeros((lt["rows"], lt["cols"]), dtype=NPBITS[sdt])
                full[np.ix_(rows[sends], cols)] = tensors[sid][srow0:srow0 + len(rows), :][sends]
                have[np.ix_(rows[sends], cols)] += 1
            if full is None:
                continue
            assert have.max() <= 1, "two holders supplied the same element"
            rows, cols = layouts.shard_index(model, lt, dst)
            got = have[np.ix_(rows, cols)] > 0
            piece = rne.convert(full[np.ix_(rows, cols)], sdt, t["dtype"])
            out[did][drow0:drow0 + len(rows), :][got] = piece[got]
            written[did][drow0:drow0 + len(rows), :][got] = True
    return out, written
