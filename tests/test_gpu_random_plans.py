"""Randomised explicit-segment plans on the GPU against the segment oracle.

Each seed draws one plan: dtype pair, alignment regime (everything a multiple of 16 bytes, so the
vector path runs, or element-aligned offsets with misaligned base pointers), segment shapes from
single elements to rows of a few thousand, strided or dense destinations, chunk and tile sizes,
checksums on or off, narrowing at pack or at unpack.  Checked bit for bit: the wire, the destination tensors (with sentinels in
every byte the plan does not own), both checksum arrays, and th_reshard into a second copy.
"""
import numpy as np
import pytest
import torch

import synth
import paper_2604_09107_amd as th
from paper_2604_09107_amd import device as dev
from oracle import checksum, segments
from helpers import tile_sizes

pytestmark = pytest.mark.gpu

NP = {"bf16": np.uint16, "f32": np.uint32}
TH = {"bf16": th.TH_BF16, "f32": th.TH_F32}
SENT = {"bf16": 0x7777, "f32": 0x77777777}


def draw_plan(rng, big=False):
    """big: rows of up to 400,000 elements in tensors of up to 8M (rows longer than any tile, thousands of
    rows per segment, chunks of up to 16 MiB) instead of rows of up to 3000 in tensors of up to 256K."""
    src_dt, dst_dt = [("f32", "bf16"), ("bf16", "bf16"), ("f32", "f32")][int(rng.integers(0, 3))]
    aligned = bool(rng.integers(0, 2))
    es_s, es_d = (4 if src_dt == "f32" else 2), (4 if dst_dt == "f32" else 2)
    # in the aligned regime every element count is a multiple of `q` (16 bytes on both sides)
    q = 16 // min(es_s, es_d) if aligned else 1
    n_src = int(rng.integers(1, 4 if big else 6))
    n_dst = int(rng.integers(1, 3 if big else 4))
    lo, hi = (1 << 18, 1 << 23) if big else (1 << 12, 1 << 18)
    src_len = [int(rng.integers(lo, hi)) // 8 * 8 for _ in range(n_src)]
    n_seg = int(rng.integers(1, 12 if big else 60))
    keys = ("src_tensor", "dst_tensor", "src_off", "src_stride", "dst_off", "dst_stride", "nrows", "row_len")
    segs = {k: np.zeros(n_seg, dtype=np.int64) for k in keys}
    dst_fill = [int(rng.integers(0, 5)) * q for _ in range(n_dst)]
    src_t = np.sort(rng.integers(0, n_src, size=n_seg)) if rng.integers(0, 2) else rng.integers(0, n_src, size=n_seg)
    for k in range(n_seg):
        t = int(src_t[k])
        if big:
            shape = int(rng.integers(0, 5))
            row_len = [int(rng.integers(1, 9)), int(rng.integers(1000, 9000)), int(rng.integers(9000, 200000)),
                       int(rng.integers(1, 400000)), int(rng.integers(4000, 7000))][shape]
            nrows = [int(rng.integers(1000, 40000)), int(rng.integers(1, 300)), int(rng.integers(1, 30)), 1,
                     int(rng.integers(100, 700))][shape]
        else:
            shape = int(rng.integers(0, 4))
            row_len = [int(rng.integers(1, 9)), int(rng.integers(1, 200)), int(rng.integers(200, 3000)),
                       int(rng.integers(1, 40))][shape]
            nrows = [int(rng.integers(1, 400)), int(rng.integers(1, 60)), int(rng.integers(1, 12)), 1][shape]
        row_len = max(q, row_len // q * q)
        s_stride = row_len + int(rng.integers(0, 5000 if big else 40)) // q * q
        while (nrows - 1) * s_stride + row_len > src_len[t]:
            nrows = max(1, nrows // 2)
            if nrows == 1 and row_len > src_len[t]:
                row_len = src_len[t] // q * q
        span = (nrows - 1) * s_stride + row_len
        s_off = int(rng.integers(0, src_len[t] - span + 1)) // q * q
        d = int(rng.integers(0, n_dst))
        d_stride = row_len if rng.integers(0, 2) else row_len + int(rng.integers(1, 3000 if big else 24)) // q * q
        d_stride = max(d_stride, row_len)
        for key, v in (("src_tensor", t), ("dst_tensor", d), ("src_off", s_off), ("src_stride", s_stride),
                       ("dst_off", dst_fill[d]), ("dst_stride", d_stride), ("nrows", nrows), ("row_len", row_len)):
            segs[key][k] = v
        dst_fill[d] += (nrows - 1) * d_stride + row_len + int(rng.integers(0, 6)) * q
    dst_len = [max(8, f + 8) for f in dst_fill]
    chunks = [4096, 65536, 1 << 20, 16 << 20] if big else [256, 4096, 65536, 1 << 20]
    return dict(src_dt=src_dt, dst_dt=dst_dt, aligned=aligned, segs=segs, src_len=src_len, dst_len=dst_len,
                chunk_bytes=int(chunks[int(rng.integers(0, 4))]),
                tile_bytes=int([4096, 8192, 16384, 32768, 131072][int(rng.integers(0, 5))]),
                checksum=bool(rng.integers(0, 2)),
                narrow_at_unpack=bool(rng.integers(0, 2)) and src_dt != dst_dt)


def device_tensor(bits, shift_elems):
    """The bit pattern in device memory, starting shift_elems elements into an allocation."""
    store = synth.from_bits(np.concatenate([np.zeros(shift_elems, dtype=bits.dtype), bits]), "cuda")
    return store, store.data_ptr() + shift_elems * bits.dtype.itemsize


BIG = 1_000_000  # seeds from here on draw the larger shapes


@pytest.mark.parametrize("seed", list(range(400)) + list(range(BIG, BIG + 40)))
def test_random_segment_plan(seed):
    rng = np.random.default_rng(9000 + seed)
    p = draw_plan(rng, big=seed >= BIG)
    segs, src_dt, dst_dt = p["segs"], p["src_dt"], p["dst_dt"]
    n_seg = len(segs["nrows"])
    if src_dt == "f32":
        srcs = [synth.to_bits(synth.scatter_values(n, 100 * seed + i, special_rate=0.05))
                for i, n in enumerate(p["src_len"])]
    else:
        srcs = [rng.integers(0, 1 << 16, size=n).astype(np.uint16) for n in p["src_len"]]
    late = p["narrow_at_unpack"]  # the wire carries the source dtype and th_unpack narrows
    wire_dt = src_dt if late else dst_dt
    wire = segments.pack(segs, srcs, src_dt, dst_dt, narrow_at="unpack" if late else "pack")
    want = [np.full(n, SENT[dst_dt], dtype=NP[dst_dt]) for n in p["dst_len"]]
    segments.unpack(segs, wire, want, dst_dt, wire_dtype=wire_dt)
    offs, _ = segments.wire_offsets(segs, wire_dt)
    want_sums = checksum.segment_checksums(segs, offs, wire_dt, wire, len(srcs))

    S = th.binding.SEGMENT_NP
    csegs = np.zeros(n_seg, dtype=S)
    csegs["src_tensor"], csegs["dst_tensor"] = segs["src_tensor"], segs["dst_tensor"]
    csegs["src_elem_off"], csegs["src_row_stride"] = segs["src_off"], segs["src_stride"]
    csegs["dst_elem_off"], csegs["dst_row_stride"] = segs["dst_off"], segs["dst_stride"]
    csegs["nrows"], csegs["row_len"] = segs["nrows"], segs["row_len"]
    csegs["src_dtype"], csegs["dst_dtype"] = TH[src_dt], TH[dst_dt]
    flags = ((th.TH_FLAG_CHECKSUM if p["checksum"] else 0) | (th.TH_FLAG_PTRS_ALIGNED16 if p["aligned"] else 0) |
             (th.TH_FLAG_NARROW_AT_UNPACK if late else 0))
    with tile_sizes(p["tile_bytes"]):
        plan = th.th_plan_create_from_segments(csegs, p["src_len"], p["dst_len"], p["chunk_bytes"], flags)
    assert plan.wire_bytes == len(wire)

    es_s, es_d = NP[src_dt]().itemsize, NP[dst_dt]().itemsize
    shift = (lambda es: 0) if p["aligned"] else (lambda es: int(rng.integers(0, 16 // es)))
    src_keep, src_ptrs = zip(*[device_tensor(s, shift(es_s)) for s in srcs])
    sent = [np.full(n, SENT[dst_dt], dtype=NP[dst_dt]) for n in p["dst_len"]]
    dst_shift = [shift(es_d) for _ in sent]
    dst_keep, dst_ptrs = zip(*[device_tensor(s, k) for s, k in zip(sent, dst_shift)])
    dir_keep, dir_ptrs = zip(*[device_tensor(s, k) for s, k in zip(sent, dst_shift)])
    wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=0xEE)
    stream = dev.current_stream()
    n = plan.num_chunks
    ps = torch.zeros(2 * len(srcs), dtype=torch.int64, device="cuda")
    us = torch.zeros_like(ps)
    src_ptrs, dst_ptrs, dir_ptrs = list(src_ptrs), list(dst_ptrs), list(dir_ptrs)
    if p["checksum"]:
        th.th_pack_checksum(plan, src_ptrs, wptrs, 0, n, ps.data_ptr(), stream)
    else:
        th.th_pack(plan, src_ptrs, wptrs, 0, n, stream)
    # unpack in pieces of one to nine chunks, taken in a random order
    cuts, c = [], 0
    while c < n:
        k = min(n - c, int(rng.integers(1, 10)))
        cuts.append((c, k))
        c += k
    for i in rng.permutation(len(cuts)):
        c, k = cuts[i]
        if p["checksum"]:
            th.th_unpack_checksum(plan, wptrs[c:c + k], c, k, dst_ptrs, us.data_ptr(), stream)
        else:
            th.th_unpack(plan, wptrs[c:c + k], c, k, dst_ptrs, stream)
    th.th_reshard(plan, src_ptrs, dir_ptrs, stream)
    torch.cuda.synchronize()

    what = "seed %d: %s" % (seed, {k: p[k] for k in ("src_dt", "dst_dt", "aligned", "chunk_bytes", "tile_bytes", "checksum",
                                                        "narrow_at_unpack")})
    got_wire = wire_dev.cpu().numpy()[:plan.wire_bytes]
    bad = np.nonzero(got_wire != wire)[0]
    assert bad.size == 0, "%s: wire differs first at byte %d (%d differ)" % (what, bad[0], bad.size)
    for name, keep in (("th_unpack", dst_keep), ("th_reshard", dir_keep)):
        for t, (g, w, k) in enumerate(zip(keep, want, dst_shift)):
            gb = synth.to_bits(g)
            assert np.all(gb[:k] == 0), "%s: %s wrote before destination tensor %d" % (what, name, t)
            bad = np.nonzero(gb[k:] != w)[0]
            assert bad.size == 0, "%s: %s destination tensor %d differs first at element %d (%d differ)" % (
                what, name, t, bad[0], bad.size)
    if p["checksum"]:
        assert np.array_equal(ps.cpu().numpy().view(np.uint64).reshape(-1, 2), want_sums), what + ": pack sums"
        assert np.array_equal(us.cpu().numpy().view(np.uint64).reshape(-1, 2), want_sums), what + ": unpack sums"
    plan.destroy()


@pytest.mark.parametrize("seed", list(range(150)) + list(range(BIG, BIG + 30)))
def test_random_segment_plan_with_progress_and_without_allocation(seed):
    """The same generator through the launches that publish progress (every store written through, one
    list in chunk order) and through th_pack_noalloc: wire and destination tensors bit for bit, the
    caller's counter equal to the range's length after each call."""
    rng = np.random.default_rng(500000 + seed)
    p = draw_plan(rng, big=seed >= BIG)
    segs, src_dt, dst_dt = p["segs"], p["src_dt"], p["dst_dt"]
    if src_dt == "f32":
        srcs = [synth.to_bits(synth.scatter_values(n, 77 * seed + i, special_rate=0.05))
                for i, n in enumerate(p["src_len"])]
    else:
        srcs = [rng.integers(0, 1 << 16, size=n).astype(np.uint16) for n in p["src_len"]]
    late = p["narrow_at_unpack"]
    wire_dt = src_dt if late else dst_dt
    wire = segments.pack(segs, srcs, src_dt, dst_dt, narrow_at="unpack" if late else "pack")
    want = [np.full(n, SENT[dst_dt], dtype=NP[dst_dt]) for n in p["dst_len"]]
    segments.unpack(segs, wire, want, dst_dt, wire_dtype=wire_dt)

    csegs = np.zeros(len(segs["nrows"]), dtype=th.binding.SEGMENT_NP)
    csegs["src_tensor"], csegs["dst_tensor"] = segs["src_tensor"], segs["dst_tensor"]
    csegs["src_elem_off"], csegs["src_row_stride"] = segs["src_off"], segs["src_stride"]
    csegs["dst_elem_off"], csegs["dst_row_stride"] = segs["dst_off"], segs["dst_stride"]
    csegs["nrows"], csegs["row_len"] = segs["nrows"], segs["row_len"]
    csegs["src_dtype"], csegs["dst_dtype"] = TH[src_dt], TH[dst_dt]
    flags = (th.TH_FLAG_PROGRESS | (th.TH_FLAG_PTRS_ALIGNED16 if p["aligned"] else 0) |
             (th.TH_FLAG_NARROW_AT_UNPACK if late else 0))
    with tile_sizes(p["tile_bytes"]):
        plan = th.th_plan_create_from_segments(csegs, p["src_len"], p["dst_len"], p["chunk_bytes"], flags)
    assert plan.wire_bytes == len(wire)
    es_s, es_d = NP[src_dt]().itemsize, NP[dst_dt]().itemsize
    shift = (lambda es: 0) if p["aligned"] else (lambda es: int(rng.integers(0, 16 // es)))
    src_keep, src_ptrs = zip(*[device_tensor(s, shift(es_s)) for s in srcs])
    sent = [np.full(n, SENT[dst_dt], dtype=NP[dst_dt]) for n in p["dst_len"]]
    dst_shift = [shift(es_d) for _ in sent]
    dst_keep, dst_ptrs = zip(*[device_tensor(s, k) for s, k in zip(sent, dst_shift)])
    src_ptrs, dst_ptrs = list(src_ptrs), list(dst_ptrs)
    wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=0xEE)
    wire_na, wptrs_na = dev.alloc_wire(plan, fill_byte=0xEE)
    stream = dev.current_stream()
    n = plan.num_chunks
    flag = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    what = "seed %d: %s" % (seed, {k: p[k] for k in ("src_dt", "dst_dt", "aligned", "chunk_bytes", "tile_bytes",
                                                        "narrow_at_unpack")})
    # pack in two ranges, each with a counter of its own
    cut = int(rng.integers(0, n + 1))
    th.th_pack_progress(plan, src_ptrs, wptrs[:cut], 0, cut, flag[0:].data_ptr(), stream)
    th.th_pack_progress(plan, src_ptrs, wptrs[cut:], cut, n - cut, flag[1:].data_ptr(), stream)
    for c in range(0, n, 4096):  # th_pack_noalloc takes at most 4096 chunks per call
        k = min(4096, n - c)
        th.th_pack_noalloc(plan, src_ptrs, wptrs_na[c:c + k], c, k, stream)
    torch.cuda.synchronize()
    assert flag.tolist() == [cut, n - cut], what
    for name, w in (("th_pack_progress", wire_dev), ("th_pack_noalloc", wire_na)):
        got = w.cpu().numpy()[:plan.wire_bytes]
        bad = np.nonzero(got != wire)[0]
        assert bad.size == 0, "%s: %s wire differs first at byte %d (%d differ)" % (what, name, bad[0], bad.size)
    th.th_unpack_progress(plan, wptrs, 0, n, dst_ptrs, flag[0:].data_ptr(), stream)
    torch.cuda.synchronize()
    assert int(flag[0]) == n, what
    for t, (g, w, k) in enumerate(zip(dst_keep, want, dst_shift)):
        gb = synth.to_bits(g)
        assert np.all(gb[:k] == 0), "%s: wrote before destination tensor %d" % (what, t)
        bad = np.nonzero(gb[k:] != w)[0]
        assert bad.size == 0, "%s: destination tensor %d differs first at element %d (%d differ)" % (
            what, t, bad[0], bad.size)
    plan.destroy()
