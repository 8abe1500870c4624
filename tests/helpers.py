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
