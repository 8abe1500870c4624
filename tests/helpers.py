"""Shared test helpers: build oracle-side inputs for a workload and run a plan's
manifest on the CPU with numpy (a test-only executor of the host planner's
output; the product path has no CPU route)."""
import contextlib

import numpy as np

import synth
from oracle import layouts, reshard, rne

NPBITS = {"bf16": np.uint16, "f32": np.uint32}
ES = {"bf16": 2, "f32": 4}


def holder_tensors_cpu(model, lay, seed, pattern=False):
    """Registered tensors of a holder as 2-D bit arrays (seeded values, norms = 1.0)."""
    lts = layouts.logical_tensors(model)
    out = []
    for i, t in enumerate(layouts.registered_tensors(model, lay)):
        n = t["rows"] * t["cols"]
        is_norm = lts[t["parts"][0][0]]["role"] == "norm"
        if pattern:
            v = synth.id_pattern_values(n, t["dtype"], i)
        else:
            v = synth.weight_values(n, t["dtype"], seed * 100 + lay["tp_rank"] * 10 + lay["ep_rank"], i, is_norm=is_norm)
        out.append(synth.to_bits(v).reshape(t["rows"], t["cols"]))
    return out


def narrow_bytes(src_bytes):
    return rne.narrow(src_bytes.view(np.uint32)).view(np.uint8)


def exec_copy(src, dst, soff, sstride, doff, dstride, nrows, ncols, es_s, es_d, pad=0):
    """Row-by-row byte copy of an nrows x ncols element rectangle, narrowing if es_s=4, es_d=2."""
    for r in range(int(nrows)):
        s = src[soff + r * sstride: soff + r * sstride + ncols * es_s]
        assert len(s) == ncols * es_s, "source read out of bounds"
        if es_s != es_d:
            assert (es_s, es_d) == (4, 2)
            s = narrow_bytes(np.ascontiguousarray(s))
        a = doff + r * dstride
        assert a + len(s) <= len(dst), "destination write out of bounds"
        dst[a:a + len(s)] = s
    if pad:
        end = doff + (nrows - 1) * dstride + ncols * es_d
        dst[end:end + pad] = 0


def exec_runs_pack(plan, src_flat, fill=0xEE):
    """Run the manifest's runs on the CPU: source tensors (flat uint8 views) -> list of chunk buffers."""
    chunks = [np.full(plan.chunk_bytes(c), fill, dtype=np.uint8) for c in range(plan.num_chunks)]
    for i in range(plan.num_runs):
        r = plan.run(i)
        exec_copy(src_flat[r.src_tensor], chunks[r.chunk], r.src_byte_off, r.src_byte_stride,
                  r.chunk_byte_off, r.wire_byte_stride, r.nrows, r.row_len,
                  4 if r.src_dtype == 2 else 2, 4 if r.wire_dtype == 2 else 2, r.pad_bytes)
    return chunks


def exec_runs_unpack(plan, chunks, dst_flat):
    for i in range(plan.num_runs):
        r = plan.run(i)
        exec_copy(chunks[r.chunk], dst_flat[r.dst_tensor], r.chunk_byte_off, r.wire_byte_stride,
                  r.dst_byte_off, r.dst_byte_stride, r.nrows, r.row_len,
                  4 if r.wire_dtype == 2 else 2, 4 if r.dst_dtype == 2 else 2)


def exec_tiles(plan, side, src_bufs, dst_bufs, chunk_range=None):
    """Run the device work list of one direction on the CPU."""
    if chunk_range is None:
        todo = range(plan.num_tiles(side))
    else:  # a chunk range is one tile range per path class (vector path, other tiles, short tiles)
        todo = [i for k in (0, 1, 2) for i in range(plan.chunk_first_tile(side, k, chunk_range[0]),
                                                 plan.chunk_first_tile(side, k, chunk_range[1]))]
    for i in todo:
        t = plan.tile(side, i)
        src, dst = src_bufs[t.src_buf], dst_bufs[t.dst_buf]
        left, col, row = int(t.count), int(t.first_col), 0
        assert col < t.row_len
        while left:
            n = min(int(t.row_len) - col, left)
            exec_copy(src, dst, t.src_byte_off + row * t.src_byte_stride + col * t.elem_bytes_src, 0,
                      t.dst_byte_off + row * t.dst_byte_stride + col * t.elem_bytes_dst, 0, 1, n,
                      t.elem_bytes_src, t.elem_bytes_dst, t.pad_bytes if n == left else 0)
            left -= n
            row += 1
            col = 0


def tile_checksums(plan, side, wire_chunks, n_src_tensors):
    """Per-tensor (A, B) computed the way the device does: per tile, terms with positions counted
    from the tile's wire-side byte offset, then shifted by the tile's run_unit_base and added up."""
    mask = (1 << 64) - 1
    sums = [[0, 0] for _ in range(n_src_tensors)]
    for i in range(plan.num_tiles(side)):
        t = plan.tile(side, i)
        if side == 0:
            chunk, off, stride, es = t.dst_buf, t.dst_byte_off, t.dst_byte_stride, t.elem_bytes_dst
        else:
            chunk, off, stride, es = t.src_buf, t.src_byte_off, t.src_byte_stride, t.elem_bytes_src
        buf = wire_chunks[chunk]
        a = b = 0
        left, col, row = int(t.count), int(t.first_col), 0
        while left:
            n = min(int(t.row_len) - col, left)
            rel = row * stride + col * es              # bytes from the tile's wire-side offset
            h = buf[off + rel: off + rel + n * es].view("<u2").astype(object)
            k0 = rel // 2
            a += int(sum(h))
            b += int(sum((k0 + j + 1) * int(v) for j, v in enumerate(h)))
            left -= n
            row += 1
            col = 0
        sums[t.src_tensor][0] = (sums[t.src_tensor][0] + a) & mask
        sums[t.src_tensor][1] = (sums[t.src_tensor][1] + b + int(t.run_unit_base) * a) & mask
    return np.array(sums, dtype=np.uint64)


@contextlib.contextmanager
def tile_sizes(tile_bytes):
    """Plans created inside the block use `tile_bytes` for every tile kind (None: library defaults)."""
    import paper_2604_09107_amd as th
    keys = (th.TH_CFG_TILE_BYTES, th.TH_CFG_TILE_BYTES_ANY, th.TH_CFG_TILE_BYTES_CHECKSUM, th.TH_CFG_TILE_BYTES_NARROW,
            th.TH_CFG_TILE_BYTES_PROGRESS)
    old = [th.th_config_get(k) for k in keys]
    try:
        if tile_bytes:
            for k in keys:
                th.th_config_set(k, tile_bytes)
        yield
    finally:
        for k, v in zip(keys, old):
            th.th_config_set(k, v)


def flat_u8(arrs):
    return [np.ascontiguousarray(a).reshape(-1).view(np.uint8) for a in arrs]


LARGE_DST_LEN = (1 << 31) + (1 << 28)  # bf16 elements: 4.8 GB


def large_offset_segments(src_dt):
    """Four bf16-destination segments whose last rows start beyond byte 2^32 of a 4.8 GB source tensor
    and of a 4.8 GB destination tensor (oracle-style dict of int64 arrays, and the source length):
    0 strided rows at element alignment, 1 strided rows with every offset a multiple of 16 bytes (48 rows
    each, spread over the whole tensor),
    2 one aligned row, 3 one row at odd element offsets."""
    es_s = 4 if src_dt == "f32" else 2
    src_len = (1 << 32) // es_s + (1 << 29) // es_s
    pitch = ((1 << 32) // es_s // 47 // 8 + 1) * 8  # the last of 48 rows starts past byte 2^32
    o = {k: np.zeros(4, dtype=np.int64) for k in
         ("src_tensor", "dst_tensor", "src_off", "src_stride", "dst_off", "dst_stride", "nrows", "row_len")}
    o["src_off"][0], o["src_stride"][0], o["dst_off"][0], o["dst_stride"][0] = 7, pitch + 3, 11, 46_000_001
    o["nrows"][0], o["row_len"][0] = 48, 1000
    o["src_off"][1], o["src_stride"][1], o["dst_off"][1], o["dst_stride"][1] = 4096, pitch, 500_000, 46_000_000
    o["nrows"][1], o["row_len"][1] = 48, 1024
    o["src_off"][2], o["dst_off"][2] = src_len - (1 << 22), 2_320_000_000
    o["nrows"][2], o["row_len"][2] = 1, 1 << 20
    o["src_off"][3], o["dst_off"][3] = src_len - (1 << 21) + 3, 2_330_000_005
    o["nrows"][3], o["row_len"][3] = 1, 300_001
    for k in (2, 3):
        o["src_stride"][k] = o["dst_stride"][k] = o["row_len"][k]
    last_src = o["src_off"] + (o["nrows"] - 1) * o["src_stride"] + o["row_len"]
    last_dst = o["dst_off"] + (o["nrows"] - 1) * o["dst_stride"] + o["row_len"]
    assert last_src.max() <= src_len and last_dst.max() <= LARGE_DST_LEN
    assert np.all((last_src - o["row_len"]) * es_s > 1 << 32) and np.all((last_dst - o["row_len"]) * 2 > 1 << 32)
    return o, src_len


def library_segments(th, o, src_dt, dst_dt):
    """The library's segment records for an oracle-style segment dict (one dtype pair for all)."""
    segs = np.zeros(len(o["nrows"]), dtype=th.binding.SEGMENT_NP)
    segs["src_tensor"], segs["dst_tensor"] = o["src_tensor"], o["dst_tensor"]
    segs["src_elem_off"], segs["src_row_stride"] = o["src_off"], o["src_stride"]
    segs["dst_elem_off"], segs["dst_row_stride"] = o["dst_off"], o["dst_stride"]
    segs["nrows"], segs["row_len"] = o["nrows"], o["row_len"]
    segs["src_dtype"] = th.TH_F32 if src_dt == "f32" else th.TH_BF16
    segs["dst_dtype"] = th.TH_F32 if dst_dt == "f32" else th.TH_BF16
    return segs
