"""Pins for the checksum oracle: Python big-integer loops, closed forms, sensitivity."""
import numpy as np

import synth
from oracle import checksum, reshard, segments
from helpers import holder_tensors_cpu

M = (1 << 64) - 1


def slow(run):
    h = np.asarray(run).view("<u2")
    a = b = 0
    for k, v in enumerate(h):
        a += int(v)
        b += (k + 1) * int(v)
    return a & M, b & M


def test_matches_big_integer_loop():
    rng = np.random.default_rng(0)
    for n in (0, 2, 14, 1000, 4098):
        run = rng.integers(0, 256, size=n, dtype=np.uint8)
        assert checksum.run_checksum(run) == slow(run)


def test_closed_form_constant_and_wraparound():
    n = 1 << 17
    run = np.full(2 * n, 0xFF, dtype=np.uint8)  # every unit = 0xFFFF
    a, b = checksum.run_checksum(run)
    assert a == (0xFFFF * n) & M and b == (0xFFFF * n * (n + 1) // 2) & M
    # a run long enough for B to exceed 2^64 must wrap, not saturate
    n = 1 << 26
    run = np.full(2 * n, 0xFF, dtype=np.uint8)
    a, b = checksum.run_checksum(run)
    assert 0xFFFF * n * (n + 1) // 2 > M and b == (0xFFFF * n * (n + 1) // 2) & M


def test_sensitive_to_value_position_and_order():
    rng = np.random.default_rng(1)
    run = rng.integers(0, 256, size=4096, dtype=np.uint8)
    base = checksum.run_checksum(run)
    flipped = run.copy()
    flipped[1001] ^= 0x10
    assert checksum.run_checksum(flipped)[0] != base[0]
    swapped = run.copy().view("<u2")
    assert swapped[10] != swapped[500]
    swapped[10], swapped[500] = swapped[500], swapped[10]
    got = checksum.run_checksum(swapped.view(np.uint8))
    assert got[0] == base[0] and got[1] != base[1]
    shifted = np.concatenate([np.zeros(2, dtype=np.uint8), run[:-2]])
    assert checksum.run_checksum(shifted) != base


def test_additive_over_a_split_with_position_offset():
    """B of a run = B of its head + B of its tail + (units in head) * A of its tail: the identity a
    tiled implementation relies on."""
    rng = np.random.default_rng(2)
    run = rng.integers(0, 256, size=6000, dtype=np.uint8)
    cut = 2 * 1234
    a, b = checksum.run_checksum(run)
    a1, b1 = checksum.run_checksum(run[:cut])
    a2, b2 = checksum.run_checksum(run[cut:])
    assert a == (a1 + a2) & M and b == (b1 + b2 + (cut // 2) * a2) & M


def test_model_checksums_cover_each_tensor_run_once():
    w = synth.workload("small_dense_tp1_to_tp4")
    model, src, dst = w["model"], w["holders"][0], w["reader"]
    tensors = holder_tensors_cpu(model, src, 3)
    wire = reshard.pack(model, src, dst, tensors)
    cs = checksum.model_checksums(model, src, dst, wire, len(tensors))
    # total A = sum of all 16-bit units of the stream (gaps are zero)
    assert int(cs[:, 0].sum(dtype=np.uint64)) == int(wire.view("<u2").astype(np.uint64).sum())
    items = list(reshard.plan_items(model, src, dst))
    it = items[3]
    n = len(it["src_r"]) * len(it["src_c"]) * 2
    assert tuple(int(x) for x in cs[it["src_id"]]) == slow(wire[it["wire_off"]:it["wire_off"] + n])


def test_segment_checksums_group_consecutive_segments_of_a_tensor():
    segs = dict(src_tensor=np.array([0, 0, 1, 0]), dst_tensor=np.zeros(4, dtype=np.int64),
                src_off=np.array([0, 8, 0, 4]), src_stride=np.array([4, 4, 4, 4]),
                dst_off=np.array([0, 8, 16, 24]), dst_stride=np.array([4, 4, 4, 4]),
                nrows=np.array([2, 1, 2, 1]), row_len=np.array([3, 3, 2, 1]))
    srcs = [np.arange(100, 120, dtype=np.uint16), np.arange(200, 220, dtype=np.uint16)]
    wire = segments.pack(segs, srcs, "bf16", "bf16")
    offs, total = segments.wire_offsets(segs, "bf16")
    cs = checksum.segment_checksums(segs, offs, "bf16", wire, 2)
    r0 = slow(wire[0:18])            # segments 0 and 1 are one run of tensor 0
    r2 = slow(wire[offs[3]:offs[3] + 2])  # its later segment is a run of its own
    assert int(cs[0, 0]) == (r0[0] + r2[0]) & M and int(cs[0, 1]) == (r0[1] + r2[1]) & M
    assert tuple(int(x) for x in cs[1]) == slow(wire[offs[2]:offs[2] + 8])
