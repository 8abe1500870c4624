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


# ---- narrowing at unpack: the wire carries the holder's dtype ------------------------------------

def mixed_case():
    """Five segments over three source tensors, two dtypes, strided on both sides."""
    segs = dict(src_tensor=np.array([0, 0, 1, 2, 2]), dst_tensor=np.array([0, 0, 1, 0, 0]),
                src_off=np.array([2, 31, 1, 0, 40]), src_stride=np.array([7, 5, 6, 9, 11]),
                dst_off=np.array([0, 12, 3, 30, 60]), dst_stride=np.array([4, 5, 4, 7, 3]),
                nrows=np.array([3, 2, 2, 4, 1]), row_len=np.array([3, 5, 3, 5, 3]))
    rng = np.random.default_rng(11)
    f32 = lambda n: rng.integers(0, 1 << 32, n, dtype=np.uint64).astype(np.uint32)
    srcs = [f32(60), np.arange(20, dtype=np.uint16) + 0x4000, f32(64)]
    # the rounding cases that matter, planted where segments read them
    srcs[0][2:5] = [0x3F808000, 0x3F818000, 0x7F800001]       # tie to even (down / up), signalling NaN
    srcs[2][0:3] = [0x7F7F8000, 0x00008001, 0xFFC12345]       # overflow to Inf, subnormal, negative NaN
    dts_s = ["f32", "f32", "bf16", "f32", "f32"]
    dts_d = ["bf16", "bf16", "bf16", "bf16", "bf16"]
    return segs, srcs, dts_s, dts_d


def test_wire_offsets_follow_the_wire_dtype():
    """Segment sizes on the wire are counted in the dtype the wire carries: with narrowing at unpack
    that is the source's, so fp32 segments take 4 bytes per element; a new source tensor re-aligns."""
    segs, srcs, dts_s, dts_d = mixed_case()
    offs_p, total_p = segments.wire_offsets(segs, dts_d)
    offs_u, total_u = segments.wire_offsets(segs, dts_s)
    # by hand: element counts 9, 10 | 6 | 20, 3
    assert list(offs_p) == [0, 18, 48, 64, 104] and total_p == 110
    assert list(offs_u) == [0, 36, 80, 96, 176] and total_u == 188
    # the stream is 2 bytes longer per narrowed element, up to the alignment gaps
    narrowed = 9 + 10 + 20 + 3
    gaps_p = (48 - 38) + (64 - 60)
    gaps_u = (80 - 76) + (96 - 92)
    assert (total_u - gaps_u) - (total_p - gaps_p) == 2 * narrowed


def test_pack_narrowing_at_unpack_matches_python_loops():
    segs, srcs, dts_s, dts_d = mixed_case()
    wire = segments.pack(segs, srcs, dts_s, dts_d, narrow_at="unpack")
    expect = bytearray()
    prev = None
    for k in range(len(segs["nrows"])):
        t = int(segs["src_tensor"][k])
        if t != prev:
            expect += b"\0" * (-len(expect) % 16)
            prev = t
        es = 4 if dts_s[k] == "f32" else 2
        for r in range(int(segs["nrows"][k])):
            for c in range(int(segs["row_len"][k])):
                u = int(srcs[t][int(segs["src_off"][k]) + r * int(segs["src_stride"][k]) + c])
                expect += u.to_bytes(es, "little")      # source bits, unconverted
    assert wire.tobytes() == bytes(expect)
    assert len(wire) == segments.wire_offsets(segs, dts_s)[1]


def test_unpack_of_a_source_dtype_wire_gives_the_same_reader_bits():
    """Narrowing at unpack lands the same bits in the same places as narrowing at pack, element by
    element: destination[d_off + r * d_stride + c] = narrow(source[s_off + r * s_stride + c])."""
    segs, srcs, dts_s, dts_d = mixed_case()
    sentinel = 0xABCD
    by_pack = [np.full(80, sentinel, dtype=np.uint16), np.full(16, sentinel, dtype=np.uint16)]
    by_unpack = [a.copy() for a in by_pack]
    counts = [np.zeros(80, dtype=np.int32), np.zeros(16, dtype=np.int32)]
    segments.unpack(segs, segments.pack(segs, srcs, dts_s, dts_d), by_pack, dts_d)
    segments.unpack(segs, segments.pack(segs, srcs, dts_s, dts_d, narrow_at="unpack"), by_unpack, dts_d,
                    counts=counts, wire_dtype=dts_s)
    loops = [np.full(80, sentinel, dtype=np.uint16), np.full(16, sentinel, dtype=np.uint16)]
    for k in range(len(segs["nrows"])):
        for r in range(int(segs["nrows"][k])):
            for c in range(int(segs["row_len"][k])):
                u = srcs[int(segs["src_tensor"][k])][int(segs["src_off"][k]) + r * int(segs["src_stride"][k]) + c]
                v = rne.narrow(np.array([u], dtype=np.uint32))[0] if dts_s[k] == "f32" else u
                loops[int(segs["dst_tensor"][k])][int(segs["dst_off"][k]) + r * int(segs["dst_stride"][k]) + c] = v
    for a, b, c in zip(by_pack, by_unpack, loops):
        assert np.array_equal(a, c) and np.array_equal(b, c)
    assert all(cnt.max() == 1 for cnt in counts)            # every covered element written once
    assert (loops[0] == sentinel).sum() == 80 - (9 + 10 + 20 + 3)
    # the planted rounding cases arrived as the narrowing rule says
    assert list(loops[0][0:3]) == [0x3F80, 0x3F82, 0x7FC0]
    assert list(loops[0][30:33]) == [0x7F80, 0x0001, 0xFFC1]


def test_scattered_case_narrowing_at_unpack_round_trip():
    d, segs, srcs = small_case()
    wire = segments.pack(segs, srcs, "f32", "bf16", narrow_at="unpack")
    offs, total = segments.wire_offsets(segs, "f32")
    assert total == len(wire) and np.all(offs % 16 == 0)    # one segment per tensor: every one re-aligns
    n_el = int((d["seg_nrows"] * d["seg_row_len"]).sum())
    assert total - 4 * n_el == sum(-4 * int(a) * int(b) % 16 for a, b in zip(d["seg_nrows"][:-1], d["seg_row_len"][:-1]))
    arena = np.full(d["arena_elems"] + 8, 0xABCD, dtype=np.uint16)
    segments.unpack(segs, wire, [arena], "bf16", wire_dtype="f32")
    ref = np.full(d["arena_elems"] + 8, 0xABCD, dtype=np.uint16)
    segments.unpack(segs, segments.pack(segs, srcs, "f32", "bf16"), [ref], "bf16")
    assert np.array_equal(arena, ref)
