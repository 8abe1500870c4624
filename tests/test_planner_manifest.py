"""Host-side tests of the C-ABI library (no GPU): the planner's manifest, run on
the CPU by a test-only numpy executor, must reproduce the oracle's wire stream
and destination tensors bit for bit; error paths; exported symbols."""
import ctypes
import os
import re

import numpy as np
import pytest

import synth
import paper_2604_09107_amd as th
from oracle import checksum, layouts, reshard, segments
from helpers import (LARGE_DST_LEN, exec_runs_pack, exec_runs_unpack, exec_tiles, flat_u8, holder_tensors_cpu,
                     large_offset_segments, library_segments, tile_checksums, tile_sizes)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST = th.TH_FLAG_HOST_ONLY
MODEL_WORKLOADS = ["cfg1_tiny_tp2_to_tp1", "small_dense_tp1_to_tp4", "small_dense_tp4_to_tp2", "small_moe_ep4_to_tp2",
                   "small_dense_trainer_to_rollout", "small_dense_rollout_to_trainer",
                   "small_moe_stacked_to_per_expert", "small_dense_kvrep_tp8_to_tp2", "small_dense_kvrep_tp2_to_tp16"]


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "th.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(th_[a-z0-9_]+)\s*\(", text))
    assert {"th_plan_create", "th_plan_create_from_segments", "th_pack", "th_unpack", "th_plan_destroy"} <= names
    lib = ctypes.CDLL(th.library_path())
    for n in sorted(names):
        assert hasattr(lib, n), n
    assert th.th_version()


@pytest.mark.parametrize("name", MODEL_WORKLOADS)
def test_tensor_lists_match_oracle(name):
    w = synth.workload(name)
    plan = th.th_plan_create(w["model"], w["holders"][0], w["reader"], w["chunk_bytes"], HOST)
    for side, lay in ((0, w["holders"][0]), (1, w["reader"])):
        want = layouts.registered_tensors(w["model"], lay)
        got = plan.tensors(side)
        assert [(t["name"], t["rows"], t["cols"], t["dtype"]) for t in got] == \
               [(t["name"], t["rows"], t["cols"], t["dtype"]) for t in want]
    plan.destroy()


@pytest.mark.parametrize("tile_bytes", [4096, 65536])
@pytest.mark.parametrize("name", MODEL_WORKLOADS)
def test_manifest_reproduces_oracle(name, tile_bytes):
    w = synth.workload(name)
    model, dst = w["model"], w["reader"]
    old = th.th_config_get(th.TH_CFG_TILE_BYTES)
    old_any = th.th_config_get(th.TH_CFG_TILE_BYTES_ANY)
    th.th_config_set(th.TH_CFG_TILE_BYTES, tile_bytes)
    th.th_config_set(th.TH_CFG_TILE_BYTES_ANY, tile_bytes)
    try:
        want_dst = reshard.empty_tensors(model, dst, fill=0x5A5A)
        got_runs = reshard.empty_tensors(model, dst, fill=0x5A5A)
        got_tiles = reshard.empty_tensors(model, dst, fill=0x5A5A)
        for src in w["holders"]:
            tensors = holder_tensors_cpu(model, src, w["seed"], pattern=True)
            wire = reshard.pack(model, src, dst, tensors)
            reshard.unpack(model, src, dst, wire, want_dst)
            want_chunks = reshard.chunks(wire, w["chunk_bytes"])

            plan = th.th_plan_create(model, src, dst, w["chunk_bytes"], HOST)
            assert plan.wire_bytes == len(wire)
            assert plan.num_chunks == len(want_chunks)
            assert [plan.chunk_bytes(c) for c in range(plan.num_chunks)] == [len(c) for c in want_chunks]
            assert plan.payload_bytes == sum(
                len(it["src_r"]) * len(it["src_c"]) * reshard.ESIZE[it["dst_dtype"]]
                for it in reshard.plan_items(model, src, dst))
            # runs (chunk manifest)
            chunks = exec_runs_pack(plan, flat_u8(tensors))
            for c, (g, x) in enumerate(zip(chunks, want_chunks)):
                assert np.array_equal(g, x), "runs: chunk %d" % c
            exec_runs_unpack(plan, chunks, flat_u8(got_runs))
            # tiles (device work list), both directions
            tchunks = [np.full(len(c), 0xEE, dtype=np.uint8) for c in want_chunks]
            exec_tiles(plan, 0, flat_u8(tensors), tchunks)
            for c, (g, x) in enumerate(zip(tchunks, want_chunks)):
                assert np.array_equal(g, x), "tiles: chunk %d" % c
            exec_tiles(plan, 1, tchunks, flat_u8(got_tiles))
            # tiles: vector-path tiles first, then the others, then the short ones, each sub-list grouped by chunk
            short_slots = th.th_config_get(th.TH_CFG_SHORT_TILE_SLOTS)
            for side in (0, 1):
                n = plan.num_chunks
                firsts = [[plan.chunk_first_tile(side, k, c) for c in range(n + 1)] for k in range(3)]
                assert firsts[0][0] == 0 and firsts[0][-1] == firsts[1][0] and firsts[1][-1] == firsts[2][0]
                assert firsts[2][-1] == plan.num_tiles(side)
                for k in range(3):
                    assert firsts[k] == sorted(firsts[k])
                    for c in range(n):
                        for i in range(firsts[k][c], firsts[k][c + 1]):
                            t = plan.tile(side, i)
                            assert (t.dst_buf if side == 0 else t.src_buf) == c
                            if k < 2:
                                assert (t.kind == 0) == (k == 0)
                            else:  # a tile of a short run fits the slots that make a run short
                                slot = 8 if (t.elem_bytes_src, t.elem_bytes_dst) == (4, 2) else 16
                                if t.kind == 1:
                                    rows = t.count // t.row_len
                                    slots = rows * ((t.row_len * t.elem_bytes_dst + slot - 1) // slot + 1)
                                else:
                                    slots = (t.count * t.elem_bytes_dst + slot - 1) // slot
                                assert slots <= short_slots + 1
            plan.destroy()
        for a, b, x in zip(got_runs, got_tiles, want_dst):
            assert np.array_equal(a, x) and np.array_equal(b, x)
    finally:
        th.th_config_set(th.TH_CFG_TILE_BYTES, old)
        th.th_config_set(th.TH_CFG_TILE_BYTES_ANY, old_any)


@pytest.mark.parametrize("name", MODEL_WORKLOADS)
def test_direct_list_equals_the_wire_free_definition(name):
    """th_reshard's work list, run on the CPU, gives the oracle's wire-free result definition."""
    w = synth.workload(name)
    model, dst = w["model"], w["reader"]
    tensors = [holder_tensors_cpu(model, src, w["seed"], pattern=True) for src in w["holders"]]
    want, written = reshard.reshard_by_definition(model, w["holders"], tensors, dst)
    got = reshard.empty_tensors(model, dst, fill=0)
    for src, ts in zip(w["holders"], tensors):
        plan = th.th_plan_create(model, src, dst, w["chunk_bytes"], HOST)
        assert plan.num_tiles(2) > 0
        exec_tiles(plan, 2, flat_u8(ts), flat_u8(got))
        plan.destroy()
    for g, x in zip(got, want):
        assert np.array_equal(g, x)


@pytest.mark.parametrize("tile_bytes", [4096, None])
def test_tile_checksum_bases_reproduce_the_oracle_checksums(tile_bytes):
    """The per-tile position bases of the work list, used the way the device uses them, give the
    oracle's per-tensor checksums - on both directions, for model and explicit-segment plans."""
    w = synth.workload("small_moe_ep4_to_tp2")
    model, src, dst = w["model"], w["holders"][0], w["reader"]
    tensors = holder_tensors_cpu(model, src, 5)
    wire = reshard.pack(model, src, dst, tensors)
    want = checksum.model_checksums(model, src, dst, wire, len(tensors))
    with tile_sizes(tile_bytes):
        plan = th.th_plan_create(model, src, dst, 64 * 1024, HOST)
    chunks = reshard.chunks(wire, 64 * 1024)
    for side in (0, 1):
        assert np.array_equal(tile_checksums(plan, side, chunks, len(tensors)), want), side
    plan.destroy()

    d = synth.scatter_description(80, 23, min_bytes=256, max_bytes=16384)
    pool = synth.to_bits(synth.scatter_values(d["pool_elems"], 23))
    srcs = [pool[o:o + m] for o, m in zip(d["pool_off"], d["n_elems"])]
    osegs = dict(src_tensor=d["seg_src_tensor"], dst_tensor=np.zeros(80, dtype=np.int64),
                 src_off=d["seg_src_off"], src_stride=d["seg_src_stride"], dst_off=d["seg_dst_off"],
                 dst_stride=d["seg_dst_stride"], nrows=d["seg_nrows"], row_len=d["seg_row_len"])
    wire = segments.pack(osegs, srcs, "f32", "bf16")
    offs, _ = segments.wire_offsets(osegs, "bf16")
    want = checksum.segment_checksums(osegs, offs, "bf16", wire, 80)
    with tile_sizes(tile_bytes):
        plan = th.th_plan_create_from_segments(scatter_segments(d), d["n_elems"], [d["arena_elems"]], 8192, HOST)
    chunks = reshard.chunks(wire, 8192)
    for side in (0, 1):
        assert np.array_equal(tile_checksums(plan, side, chunks, 80), want), side
    plan.destroy()


@pytest.mark.parametrize("name", ["small_dense_tp1_to_tp4", "small_dense_trainer_to_rollout", "small_moe_ep4_to_tp2"])
def test_narrowing_at_unpack_manifest(name):
    """TH_FLAG_NARROW_AT_UNPACK: the wire carries the holder's dtype; runs, tiles and checksum bases
    reproduce the oracle's wider stream and the same reader tensors."""
    w = synth.workload(name)
    model, dst = w["model"], w["reader"]
    flags = HOST | th.TH_FLAG_NARROW_AT_UNPACK
    want = reshard.empty_tensors(model, dst, fill=0x5A5A)
    got = reshard.empty_tensors(model, dst, fill=0x5A5A)
    direct = reshard.empty_tensors(model, dst, fill=0x5A5A)
    for src in w["holders"]:
        tensors = holder_tensors_cpu(model, src, w["seed"], pattern=True)
        wire = reshard.pack(model, src, dst, tensors, narrow_at="unpack")
        reshard.unpack(model, src, dst, wire, want, narrow_at="unpack")
        with tile_sizes(4096):
            plan = th.th_plan_create(model, src, dst, 32 * 1024, flags)
        assert plan.wire_bytes == len(wire) and plan.payload_bytes <= plan.src_read_bytes
        want_chunks = reshard.chunks(wire, 32 * 1024)
        chunks = exec_runs_pack(plan, flat_u8(tensors))
        tchunks = [np.full(len(c), 0xEE, dtype=np.uint8) for c in want_chunks]
        exec_tiles(plan, 0, flat_u8(tensors), tchunks)
        for a, b, x in zip(chunks, tchunks, want_chunks):
            assert np.array_equal(a, x) and np.array_equal(b, x)
        exec_tiles(plan, 1, tchunks, flat_u8(got))
        exec_tiles(plan, 2, flat_u8(tensors), flat_u8(direct))
        cs = checksum.model_checksums(model, src, dst, wire, len(tensors), narrow_at="unpack")
        for side in (0, 1):
            assert np.array_equal(tile_checksums(plan, side, want_chunks, len(tensors)), cs)
        plan.destroy()
    for g, d, x in zip(got, direct, want):
        assert np.array_equal(g, x) and np.array_equal(d, x)


def test_tensors_complete_matches_the_oracle_prefix():
    """Chunks done -> leading source tensors whose run has fully arrived (the paper's progress unit)."""
    for name in ("small_dense_tp1_to_tp4", "small_moe_ep4_to_tp2", "small_dense_tp4_to_tp2"):
        w = synth.workload(name)
        model, dst = w["model"], w["reader"]
        for src in w["holders"]:
            cb = 64 * 1024
            plan = th.th_plan_create(model, src, dst, cb, HOST)
            n_src = plan.num_tensors(0)
            end = np.zeros(n_src, dtype=np.int64)
            for it in reshard.plan_items(model, src, dst):
                n = len(it["src_r"]) * len(it["src_c"]) * reshard.ESIZE[it["wire_dtype"]]
                end[it["src_id"]] = max(end[it["src_id"]], it["wire_off"] + n)
            prev = 0
            for c in range(plan.num_chunks + 1):
                done = min(c * cb, plan.wire_bytes)
                want = 0
                while want < n_src and end[want] <= done:
                    want += 1
                got = plan.tensors_complete(c)
                assert got == want and got >= prev
                prev = got
            assert plan.tensors_complete(plan.num_chunks) == n_src
            plan.destroy()


def test_chunks_are_self_contained():
    """Unpacking any subset of chunks, in any order, touches only that subset's elements."""
    w = synth.workload("small_dense_tp1_to_tp4")
    model, src, dst = w["model"], w["holders"][0], w["reader"]
    tensors = holder_tensors_cpu(model, src, 1, pattern=True)
    want = reshard.empty_tensors(model, dst, fill=0)
    wire = reshard.pack(model, src, dst, tensors)
    reshard.unpack(model, src, dst, wire, want)
    plan = th.th_plan_create(model, src, dst, 64 * 1024, HOST)
    n = plan.num_chunks
    assert n > 8
    chunks = [np.full(plan.chunk_bytes(c), 0xEE, dtype=np.uint8) for c in range(n)]
    got = reshard.empty_tensors(model, dst, fill=0)
    for c in list(range(n - 1, -1, -2)) + list(range(n - 2, -1, -2)):  # odd/even, backwards
        exec_tiles(plan, 0, flat_u8(tensors), chunks, (c, c + 1))
        assert np.array_equal(chunks[c], reshard.chunks(wire, 64 * 1024)[c])
        exec_tiles(plan, 1, chunks, flat_u8(got), (c, c + 1))
    for g, x in zip(got, want):
        assert np.array_equal(g, x)
    plan.destroy()


def scatter_segments(d, dst_dtype=th.TH_BF16):
    n = len(d["perm"])
    segs = np.zeros(n, dtype=th.binding.SEGMENT_NP)
    segs["src_tensor"] = d["seg_src_tensor"]
    segs["dst_tensor"] = 0
    segs["src_elem_off"] = d["seg_src_off"]
    segs["dst_elem_off"] = d["seg_dst_off"]
    segs["src_row_stride"] = d["seg_src_stride"]
    segs["dst_row_stride"] = d["seg_dst_stride"]
    segs["nrows"] = d["seg_nrows"]
    segs["row_len"] = d["seg_row_len"]
    segs["src_dtype"] = th.TH_F32
    segs["dst_dtype"] = dst_dtype
    return segs


@pytest.mark.parametrize("chunk_bytes,tile_bytes", [(4096, 4096), (65536, 8192), (1 << 20, 65536)])
def test_explicit_segments_manifest_reproduces_oracle(chunk_bytes, tile_bytes):
    d = synth.scatter_description(150, 21, min_bytes=256, max_bytes=65536)
    pool = synth.to_bits(synth.scatter_values(d["pool_elems"], 21, special_rate=0.05))
    srcs = [pool[o:o + m] for o, m in zip(d["pool_off"], d["n_elems"])]
    osegs = dict(src_tensor=d["seg_src_tensor"], dst_tensor=np.zeros(150, dtype=np.int64),
                 src_off=d["seg_src_off"], src_stride=d["seg_src_stride"], dst_off=d["seg_dst_off"],
                 dst_stride=d["seg_dst_stride"], nrows=d["seg_nrows"], row_len=d["seg_row_len"])
    wire = segments.pack(osegs, srcs, "f32", "bf16")
    arena = np.full(d["arena_elems"] + 16, 0x7777, dtype=np.uint16)
    segments.unpack(osegs, wire, [arena], "bf16")

    old = th.th_config_get(th.TH_CFG_TILE_BYTES)
    old_any = th.th_config_get(th.TH_CFG_TILE_BYTES_ANY)
    th.th_config_set(th.TH_CFG_TILE_BYTES, tile_bytes)
    th.th_config_set(th.TH_CFG_TILE_BYTES_ANY, tile_bytes)
    try:
        plan = th.th_plan_create_from_segments(scatter_segments(d), d["n_elems"], [len(arena)], chunk_bytes, HOST)
    finally:
        th.th_config_set(th.TH_CFG_TILE_BYTES, old)
        th.th_config_set(th.TH_CFG_TILE_BYTES_ANY, old_any)
    assert plan.wire_bytes == len(wire)
    assert plan.src_read_bytes == 2 * plan.payload_bytes == 4 * d["arena_elems"]
    want_chunks = reshard.chunks(wire, chunk_bytes)
    for use_tiles in (False, True):
        if use_tiles:
            chunks = [np.full(len(c), 0xEE, dtype=np.uint8) for c in want_chunks]
            exec_tiles(plan, 0, flat_u8(srcs), chunks)
        else:
            chunks = exec_runs_pack(plan, flat_u8(srcs))
        for c, (g, x) in enumerate(zip(chunks, want_chunks)):
            assert np.array_equal(g, x), (use_tiles, c)
        got = np.full(len(arena), 0x7777, dtype=np.uint16)
        if use_tiles:
            exec_tiles(plan, 1, chunks, [got.view(np.uint8)])
        else:
            exec_runs_unpack(plan, chunks, [got.view(np.uint8)])
        assert np.array_equal(got, arena)
    plan.destroy()


@pytest.mark.parametrize("src_dt", ["bf16", "f32"])
def test_offsets_beyond_four_gib_inside_one_tensor(src_dt):
    """Rows that start past byte 2^32 of a 4.8 GB source and of a 4.8 GB destination tensor: the runs
    and all three tile lists, run on the CPU, give the oracle's wire and destination.  (Both tensors
    are untouched zero pages except where the segments read and write.)"""
    o, src_len = large_offset_segments(src_dt)
    npd = np.uint32 if src_dt == "f32" else np.uint16
    src = np.zeros(src_len, dtype=npd)
    rng = np.random.default_rng(9)
    for k in range(4):
        for r in range(int(o["nrows"][k])):
            a = int(o["src_off"][k] + r * o["src_stride"][k])
            src[a:a + int(o["row_len"][k])] = rng.integers(1, 1 << (8 * src.itemsize), size=int(o["row_len"][k])).astype(npd)
    wire = segments.pack(o, [src], src_dt, "bf16")
    want = np.zeros(LARGE_DST_LEN, dtype=np.uint16)
    segments.unpack(o, wire, [want], "bf16")
    plan = th.th_plan_create_from_segments(library_segments(th, o, src_dt, "bf16"), [src_len], [LARGE_DST_LEN],
                                           1 << 20, HOST | th.TH_FLAG_PTRS_ALIGNED16)
    assert {plan.tile(s_, i).kind for s_ in (0, 1) for i in range(plan.num_tiles(s_))} == {0, 1, 2}
    src_u8 = src.view(np.uint8)
    chunks = exec_runs_pack(plan, [src_u8], fill=0)
    assert np.array_equal(np.concatenate(chunks)[:plan.wire_bytes], wire)
    for what in ("runs", "tiles", "direct"):
        dst = np.zeros(LARGE_DST_LEN, dtype=np.uint16)
        if what == "runs":
            exec_runs_unpack(plan, chunks, [dst.view(np.uint8)])
        elif what == "tiles":
            tchunks = [np.zeros(plan.chunk_bytes(c), dtype=np.uint8) for c in range(plan.num_chunks)]
            exec_tiles(plan, 0, [src_u8], tchunks)
            assert np.array_equal(np.concatenate(tchunks)[:plan.wire_bytes], wire)
            exec_tiles(plan, 1, tchunks, [dst.view(np.uint8)])
        else:
            exec_tiles(plan, 2, [src_u8], [dst.view(np.uint8)])
        # compared around every destination row (a whole-array comparison would fault in 10 GB of zero pages)
        for k in range(4):
            for r in range(int(o["nrows"][k])):
                a = int(o["dst_off"][k] + r * o["dst_stride"][k])
                lo, hi = max(0, a - 64), min(LARGE_DST_LEN, a + int(o["row_len"][k]) + 64)
                assert np.array_equal(dst[lo:hi], want[lo:hi]), (what, k, r)
        del dst
    plan.destroy()


def test_error_paths():
    w = synth.workload("cfg1_tiny_tp2_to_tp1")
    model, src, dst = w["model"], w["holders"][0], w["reader"]
    with pytest.raises(th.ThError) as e:
        th.th_plan_create(dict(model, vocab=1001), src, dst, 1 << 20, HOST)
    assert e.value.code == -2 and "vocab" in str(e.value) or "embed" in str(e.value)
    with pytest.raises(th.ThError) as e:  # 3 ranks over 6 query / 2 KV heads: neither divisor nor multiple
        th.th_plan_create(dict(model, n_q_heads=6, hidden=384, vocab=999), synth.layout(3, 0), dst, 1 << 20, HOST)
    assert e.value.code == -3
    with pytest.raises(th.ThError) as e:
        th.th_plan_create(model, src, dst, 1000, HOST)  # not a multiple of 16
    assert e.value.code == -1
    with pytest.raises(th.ThError) as e:
        th.th_plan_create(model, synth.layout(2, 2), dst, 1 << 20, HOST)  # rank out of range
    assert e.value.code == -1
    with pytest.raises(th.ThError) as e:  # reader keeps fp32 norms but holder stores bf16: widening
        th.th_plan_create(model, synth.layout(2, 0, f32_store="bf16"), synth.layout(1, 0, f32_store="f32"), 1 << 20, HOST)
    assert e.value.code == -3
    with pytest.raises(th.ThError) as e:  # padding smaller than the vocabulary
        th.th_plan_create(model, synth.layout(2, 0, padded_vocab=512), dst, 1 << 20, HOST)
    assert e.value.code == -1
    with pytest.raises(th.ThError) as e:  # padded size not divisible by the ranks
        th.th_plan_create(model, synth.layout(2, 0, padded_vocab=1001), dst, 1 << 20, HOST)
    assert e.value.code == -2
    plan = th.th_plan_create(model, src, dst, 1 << 20, HOST)
    with pytest.raises(th.ThError) as e:
        th.th_pack(plan, [0] * plan.num_tensors(0), [0], 0, 1)
    assert e.value.code == -1 and "HOST_ONLY" in str(e.value)
    with pytest.raises(th.ThError):
        plan.tensor_info(0, 10 ** 6)
    plan.destroy()
    plan.destroy()  # idempotent in the binding
    with pytest.raises(th.ThError):
        th.th_config_set(th.TH_CFG_TILE_BYTES, 1000)
    with pytest.raises(th.ThError):
        th.th_config_set(99, 0)

    # explicit segments: out-of-range, overlapping destination rows, dtype clash
    S = th.binding.SEGMENT_NP
    seg = np.zeros(1, dtype=S)
    seg["nrows"], seg["row_len"], seg["src_row_stride"], seg["dst_row_stride"] = 4, 8, 8, 8
    seg["src_dtype"], seg["dst_dtype"] = th.TH_F32, th.TH_BF16
    th.th_plan_create_from_segments(seg, [32], [32], 4096, HOST).destroy()
    with pytest.raises(th.ThError) as e:
        th.th_plan_create_from_segments(seg, [31], [32], 4096, HOST)
    assert e.value.code == -4
    with pytest.raises(th.ThError) as e:
        th.th_plan_create_from_segments(seg, [32], [31], 4096, HOST)
    assert e.value.code == -4
    bad = seg.copy()
    bad["dst_row_stride"] = 7
    with pytest.raises(th.ThError) as e:
        th.th_plan_create_from_segments(bad, [32], [32], 4096, HOST)
    assert e.value.code == -1
    bad = seg.copy()
    bad["src_dtype"], bad["dst_dtype"] = th.TH_BF16, th.TH_F32
    with pytest.raises(th.ThError) as e:
        th.th_plan_create_from_segments(bad, [32], [32], 4096, HOST)
    assert e.value.code == -3
    bad = seg.copy()
    bad["src_tensor"] = 1
    with pytest.raises(th.ThError) as e:
        th.th_plan_create_from_segments(bad, [32], [32], 4096, HOST)
    assert e.value.code == -4
    # a tile record holds a rectangle's row length in 32 bits: rows of 2^31 elements are refused unless
    # the segment is a single row, which is cut with 64-bit offsets
    huge = seg.copy()
    huge["nrows"], huge["row_len"], huge["src_row_stride"], huge["dst_row_stride"] = 2, 1 << 31, (1 << 31) + 8, 1 << 31
    huge["src_dtype"] = th.TH_BF16
    with pytest.raises(th.ThError) as e:
        th.th_plan_create_from_segments(huge, [1 << 34], [1 << 34], 1 << 30, HOST)
    assert e.value.code == -3 and "single-row" in str(e.value)
    huge["nrows"], huge["row_len"], huge["src_elem_off"], huge["dst_elem_off"] = 1, 1 << 32, 3, 5
    plan = th.th_plan_create_from_segments(huge, [1 << 34], [1 << 34], 1 << 30, HOST)
    assert plan.wire_bytes == 2 << 32 and plan.num_chunks == 8
    for side in (0, 1, 2):
        last = plan.tile(side, plan.num_tiles(side) - 1)
        tensor_side_end = (last.dst_byte_off if side else last.src_byte_off) + 2 * last.count
        assert tensor_side_end == 2 * ((1 << 32) + (5 if side else 3))
    plan.destroy()


def test_empty_plan_and_empty_segments():
    p = th.th_plan_create_from_segments(np.zeros(0, dtype=th.binding.SEGMENT_NP), [], [], 4096, HOST)
    assert p.num_chunks == 0 and p.wire_bytes == 0 and p.num_runs == 0
    p.destroy()
    seg = np.zeros(2, dtype=th.binding.SEGMENT_NP)
    seg["src_dtype"], seg["dst_dtype"] = th.TH_BF16, th.TH_BF16
    seg["nrows"][1], seg["row_len"][1], seg["src_row_stride"][1], seg["dst_row_stride"][1] = 1, 3, 3, 3
    p = th.th_plan_create_from_segments(seg, [8], [8], 4096, HOST)  # first segment is empty
    assert p.num_runs == 1 and p.wire_bytes == 6
    p.destroy()


def test_full_size_plans_cover_every_destination_element_once():
    """Full-size configurations, manifest only: payload equals the reader's bytes and no
    two runs overlap on the wire or in the destination (interval check, no data)."""
    for name in ("cfg2_8b_tp1_to_tp4", "cfg4_moe_ep8_to_tp2"):
        w = synth.workload(name)
        model, dst = w["model"], w["reader"]
        plan = th.th_plan_create(model, w["holders"][0], dst, w["chunk_bytes"], HOST)
        assert plan.wire_bytes == reshard.wire_bytes(model, w["holders"][0], dst)
        dst_regs = layouts.registered_tensors(model, dst)
        per_tensor = {}
        wire_iv = []
        for i in range(plan.num_runs):
            r = plan.run(i)
            es = 4 if r.dst_dtype == 2 else 2
            if r.dst_byte_stride == r.row_len * es or r.nrows == 1:
                per_tensor.setdefault(r.dst_tensor, []).append((r.dst_byte_off, r.dst_byte_off + r.nrows * r.row_len * es))
            else:
                for k in range(r.nrows):
                    a = r.dst_byte_off + k * r.dst_byte_stride
                    per_tensor.setdefault(r.dst_tensor, []).append((a, a + r.row_len * es))
            assert r.wire_byte_stride == r.row_len * es or r.nrows == 1  # these configs are dense on the wire
            a = r.chunk * w["chunk_bytes"] + r.chunk_byte_off
            wire_iv.append((a, a + r.nrows * r.row_len * es))
        wire_iv.sort()
        assert wire_iv[0][0] == 0 and wire_iv[-1][1] == plan.wire_bytes
        assert all(a[1] == b[0] for a, b in zip(wire_iv, wire_iv[1:]))  # 16-byte multiples: no gaps here
        covered = 0
        for t, iv in per_tensor.items():
            iv.sort()
            assert all(a[1] <= b[0] for a, b in zip(iv, iv[1:])), dst_regs[t]["name"]
            covered += sum(b - a for a, b in iv)
        assert covered == plan.payload_bytes
        if name.startswith("cfg2"):
            assert covered == sum(t["rows"] * t["cols"] * reshard.ESIZE[t["dtype"]] for t in dst_regs)
        plan.destroy()


@pytest.mark.parametrize("flags", [0, th.TH_FLAG_PTRS_ALIGNED16])
def test_tiles_of_a_contiguous_destination_start_on_cache_lines(flags):
    """Within a run whose destination is contiguous, every tile after the first starts on a 128-byte
    line of the destination buffer (dense path always; vector path when rows are whole lines)."""
    rng = np.random.default_rng(77)
    n = 40
    q = 8 if flags else 1                           # elements per 16 bytes in the aligned regime
    segs = np.zeros(n, dtype=th.binding.SEGMENT_NP)
    src_len, fill = [], 0
    for k in range(n):
        ln = int(rng.integers(3000, 40000)) // q * q
        segs[k]["src_tensor"], segs[k]["dst_tensor"] = k, 0
        segs[k]["src_elem_off"], segs[k]["src_row_stride"] = int(rng.integers(0, 9)) * q, ln
        segs[k]["dst_elem_off"], segs[k]["dst_row_stride"] = fill, ln
        segs[k]["nrows"], segs[k]["row_len"] = 1, ln
        segs[k]["src_dtype"] = segs[k]["dst_dtype"] = th.TH_BF16
        src_len.append(ln + 64)
        fill += ln + int(rng.integers(0, 7)) * q    # runs start at any element (or any 16 bytes)
    plan = th.th_plan_create_from_segments(segs, src_len, [fill + 8], 1 << 20, flags | HOST)
    for side in (0, 1):
        starts = {}                                  # run (and chunk) -> destination offsets of its tiles
        for i in range(plan.num_tiles(side)):
            t = plan.tile(side, i)
            assert t.kind == (0 if flags else 2)
            starts.setdefault((t.src_tensor, t.src_buf, t.dst_buf), []).append(t.dst_byte_off)
        later = 0
        for offs in starts.values():
            for off in sorted(offs)[1:]:             # every tile of the run but its first
                assert off % 128 == 0, (side, off)
                later += 1
        assert later > 50
    plan.destroy()


@pytest.fixture
def no_short_runs():
    """Plans that publish progress have no short class; compare them with plain plans built the same way."""
    old = th.th_config_get(th.TH_CFG_SHORT_TILE_SLOTS)
    th.th_config_set(th.TH_CFG_SHORT_TILE_SLOTS, 0)
    yield
    th.th_config_set(th.TH_CFG_SHORT_TILE_SLOTS, old)


@pytest.mark.parametrize("name,chunk_bytes,tile_bytes", [("small_dense_tp1_to_tp4", 128 * 1024, 4096),
                                                        ("small_moe_ep4_to_tp2", 64 * 1024, 4096),
                                                        ("small_dense_tp4_to_tp2", 256 * 1024, 16384)])
def test_plans_that_publish_progress_keep_the_plain_lists(name, chunk_bytes, tile_bytes, no_short_runs):
    """Prefix order is a property of the launch (which record a workgroup takes), not of the lists:
    a plan with the flag holds the same tiles in the same places as one without (and without a
    short-run class), so everything the list tests establish carries over."""
    w = synth.workload(name)
    model, src, dst = w["model"], w["holders"][0], w["reader"]
    with tile_sizes(tile_bytes):
        plain = th.th_plan_create(model, src, dst, chunk_bytes, HOST)
        ordered = th.th_plan_create(model, src, dst, chunk_bytes, HOST | th.TH_FLAG_PROGRESS)
    for side in (0, 1, 2):
        assert [bytes(ordered.tile(side, i)) for i in range(ordered.num_tiles(side))] == \
               [bytes(plain.tile(side, i)) for i in range(plain.num_tiles(side))]
    for side in (0, 1):
        assert plain.chunk_first_tile(side, 1, 0) == plain.num_tiles(side)      # vector-path tiles only
        for k in range(3):
            assert [ordered.chunk_first_tile(side, k, c) for c in range(plain.num_chunks + 1)] == \
                   [plain.chunk_first_tile(side, k, c) for c in range(plain.num_chunks + 1)]
    plain.destroy()
    ordered.destroy()


def test_plan_that_publishes_progress_with_mixed_paths_keeps_one_list(no_short_runs):
    """Launches run class after class, which cannot finish chunk after chunk: a plan that publishes
    progress and has tiles of more than one path class keeps them all in one list in chunk order."""
    n = 60
    segs = np.zeros(n, dtype=th.binding.SEGMENT_NP)
    segs["src_tensor"] = np.arange(n) // 3
    segs["nrows"], segs["row_len"] = 8, 2048
    segs["src_row_stride"], segs["dst_row_stride"] = 2560, 2048
    segs["src_elem_off"] = (np.arange(n) % 3) * 30000 + (np.arange(n) % 2)    # every other run is off by one element
    segs["dst_elem_off"] = np.arange(n) * 8 * 2048
    segs["src_dtype"] = segs["dst_dtype"] = th.TH_BF16
    args = (segs, np.full(n // 3, 90000), [n * 8 * 2048], 96 * 1024)
    with tile_sizes(4096):
        plain = th.th_plan_create_from_segments(*args, HOST | th.TH_FLAG_PTRS_ALIGNED16)
        ordered = th.th_plan_create_from_segments(*args, HOST | th.TH_FLAG_PTRS_ALIGNED16 | th.TH_FLAG_PROGRESS)
    mixed = 0
    for side in (0, 1):
        total = plain.num_tiles(side)
        n_vec = plain.chunk_first_tile(side, 1, 0)
        assert ordered.num_tiles(side) == total
        if 0 < n_vec < total:     # pack: every other run starts off a 16-byte boundary of its tensor
            mixed += 1
            assert ordered.chunk_first_tile(side, 1, 0) == 0 and ordered.chunk_first_tile(side, 2, 0) == total
            merged = 1
        else:                     # unpack: wire and reader tensor are aligned, vector path throughout
            assert n_vec == total and ordered.chunk_first_tile(side, 1, 0) == total
            merged = 0
        for c in range(plain.num_chunks):
            a = [bytes(plain.tile(side, i)) for k in range(3)
                 for i in range(plain.chunk_first_tile(side, k, c), plain.chunk_first_tile(side, k, c + 1))]
            t0, t1 = ordered.chunk_first_tile(side, merged, c), ordered.chunk_first_tile(side, merged, c + 1)
            assert [bytes(ordered.tile(side, i)) for i in range(t0, t1)] == a
    assert mixed == 1
    plain.destroy()
    ordered.destroy()
