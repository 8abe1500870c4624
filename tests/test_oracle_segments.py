"""Pins for the explicit-segment oracle: element-by-element Python loops on tiny
inputs, exactly-once coverage of the arena, byte counts, zero gaps."""
import numpy as np

import synth
from oracle import rne, segments


def small_case(n=60, seed=9):
    d = synth.scatter_description(n, seed, min_bytes=256, max_bytes=4096)
    segs = dict(src_tensor=d["seg_src_tensor"], dst_tensor=np.zeros(n, dtype=np.int64),
                src_off=d["seg_src_off"], src_stride=d["seg_src_stride"],
                dst_off=d["seg_dst_off"], dst_stride=d["seg_dst_stride"],
                nrows=d["seg_nrows"], row_len=d["seg_row_len"])
    pool = synth.to_bits(synth.scatter_values(d["pool_elems"], seed, special_rate=0.2))
    srcs = [pool[o:o + m] for o, m in zip(d["pool_off"], d["n_elems"])]
    return d, segs, srcs


def test_description_is_well_formed():
    d = synth.scatter_description(2000, 5)
    S, R = d["row_stride"], d["n_elems"] // d["row_stride"]
    assert np.all(d["n_elems"] * 4 >= 4096) and np.all(d["n_elems"] * 4 <= 64 << 20)
    assert np.all(S >= 16) and np.all(S <= np.minimum(d["n_elems"], 16384))
    assert np.all(d["r0"] + d["nr"] <= R) and np.all(d["c0"] + d["nc"] <= S)
    assert np.all(d["nr"] >= (R + 1) // 2) and np.all(d["nc"] >= (S + 1) // 2)
    assert sorted(d["perm"]) == list(range(2000))
    # last element touched lies inside the tensor
    last = (d["r0"] + d["nr"] - 1) * S + d["c0"] + d["nc"] - 1
    assert np.all(last < d["n_elems"])
    # arena slices tile [0, arena_elems) without gaps
    assert d["arena_off"][0] == 0
    assert np.array_equal(d["arena_off"][1:], np.cumsum(d["nr"] * d["nc"])[:-1])


def test_pack_matches_python_loops():
    d, segs, srcs = small_case()
    wire = segments.pack(segs, srcs, "f32", "bf16")
    expect = bytearray()
    prev = None
    for k in range(len(segs["nrows"])):
        t = int(segs["src_tensor"][k])
        if t != prev:
            expect += b"\0" * (-len(expect) % 16)
            prev = t
        for r in range(int(segs["nrows"][k])):
            for c in range(int(segs["row_len"][k])):
                u = srcs[t][int(segs["src_off"][k]) + r * int(segs["src_stride"][k]) + c]
                expect += int(rne.narrow(np.array([u], dtype=np.uint32))[0]).to_bytes(2, "little")
    assert wire.tobytes() == bytes(expect)
    offs, total = segments.wire_offsets(segs, "bf16")
    assert total == len(wire) and np.all(offs % 2 == 0)


def test_unpack_fills_arena_exactly_once_in_index_order():
    d, segs, srcs = small_case()
    wire = segments.pack(segs, srcs, "f32", "bf16")
    arena = np.full(d["arena_elems"] + 8, 0xABCD, dtype=np.uint16)
    counts = [np.zeros(len(arena), dtype=np.int32)]
    segments.unpack(segs, wire, [arena], "bf16", counts)
    assert np.all(counts[0][:d["arena_elems"]] == 1) and np.all(counts[0][d["arena_elems"]:] == 0)
    assert np.all(arena[d["arena_elems"]:] == 0xABCD)
    # arena = slices in tensor-index order, each row-major and narrowed
    expect = []
    for i in range(len(d["n_elems"])):
        S = int(d["row_stride"][i])
        m = srcs[i][:(len(srcs[i]) // S) * S].reshape(-1, S)
        sl = m[d["r0"][i]:d["r0"][i] + d["nr"][i], d["c0"][i]:d["c0"][i] + d["nc"][i]]
        expect.append(rne.narrow(sl).reshape(-1))
    assert np.array_equal(arena[:d["arena_elems"]], np.concatenate(expect))


def test_mixed_dtypes_and_same_tensor_runs_share_alignment():
    # two segments of the same source tensor follow each other without a gap; a new tensor re-aligns
    segs = dict(src_tensor=np.array([0, 0, 1]), dst_tensor=np.array([0, 0, 1]),
                src_off=np.array([1, 20, 0]), src_stride=np.array([5, 7, 3]),
                dst_off=np.array([0, 9, 2]), dst_stride=np.array([3, 3, 4]),
                nrows=np.array([3, 1, 2]), row_len=np.array([3, 3, 3]))
    srcs = [np.arange(40, dtype=np.uint16) + 100, np.arange(10, dtype=np.uint32) + 0x3F800000]
    dts_s, dts_d = ["bf16", "bf16", "f32"], ["bf16", "bf16", "f32"]
    offs, total = segments.wire_offsets(segs, dts_d)
    assert list(offs) == [0, 18, 32] and total == 32 + 24
    wire = segments.pack(segs, srcs, dts_s, dts_d)
    assert list(wire[:18].view(np.uint16)) == [101, 102, 103, 106, 107, 108, 111, 112, 113]
    assert list(wire[18:24].view(np.uint16)) == [120, 121, 122]
    assert not wire[24:32].any()
    assert list(wire[32:].view(np.uint32) - 0x3F800000) == [0, 1, 2, 3, 4, 5]
    dsts = [np.zeros(12, dtype=np.uint16), np.zeros(12, dtype=np.uint32)]
    segments.unpack(segs, wire, dsts, dts_d)
    assert list(dsts[0]) == [101, 102, 103, 106, 107, 108, 111, 112, 113, 120, 121, 122]
    assert list(dsts[1][2:5] - 0x3F800000) == [0, 1, 2] and list(dsts[1][6:9] - 0x3F800000) == [3, 4, 5]
