"""th_pack_noalloc (the th_pack variant for callers that cannot allocate) against th_pack, byte for
byte, through the C ABI.  The entry point keeps its device pointer tables in a fixed array inside
the library that every call on the GPU shares, so the checks run on calls in a row: a larger input
first, then a smaller one that reuses the front of the tables, then the larger one again."""
import numpy as np
import pytest
import torch

import synth
import paper_2604_09107_amd as th
from paper_2604_09107_amd import device as dev
from helpers import holder_tensors_cpu
from test_planner_manifest import scatter_segments

pytestmark = pytest.mark.gpu

SENT8 = 0xEE


def to_dev(bits2d):
    return synth.from_bits(np.ascontiguousarray(bits2d).reshape(-1), "cuda")


def model_case(name, chunk_bytes):
    w = synth.workload(name)
    model, src, dst = w["model"], w["holders"][0], w["reader"]
    plan = th.th_plan_create(model, src, dst, chunk_bytes)
    src_dev = [to_dev(t) for t in holder_tensors_cpu(model, src, w["seed"], pattern=True)]
    return plan, src_dev, dev.ptrs(src_dev)


def scatter_case(n, seed, chunk_bytes):
    d = synth.scatter_description(n, seed, min_bytes=256, max_bytes=1 << 16)
    pool = torch.empty(d["pool_elems"] + 4, dtype=torch.float32, device="cuda")[1:]   # 4-byte aligned only
    pool[:d["pool_elems"]] = synth.scatter_values(d["pool_elems"], seed, "cuda", 0.05)
    plan = th.th_plan_create_from_segments(scatter_segments(d), d["n_elems"], [d["arena_elems"] + 8], chunk_bytes)
    return plan, pool, pool.data_ptr() + d["pool_off"].astype(np.uint64) * np.uint64(4)


def pack_both_ways(plan, src_ptrs, first, count, stream):
    """Wire bytes of chunks [first, first + count) from th_pack and from th_pack_noalloc."""
    out = []
    for call in (th.th_pack, th.th_pack_noalloc):
        wire, wptrs = dev.alloc_wire(plan, fill_byte=SENT8)
        call(plan, src_ptrs, wptrs[first:first + count], first, count, stream)
        torch.cuda.synchronize()
        out.append(wire.cpu().numpy())
    return out


def assert_equal_wire(plan, src_ptrs, first, count, stream, what):
    ref, got = pack_both_ways(plan, src_ptrs, first, count, stream)
    lo = first * plan.chunk_bytes(0)
    hi = lo + sum(plan.chunk_bytes(c) for c in range(first, first + count))
    assert not np.all(ref[lo:hi] == SENT8), what
    bad = np.nonzero(ref != got)[0]
    assert bad.size == 0, "%s: differs first at byte %d (%d bytes differ)" % (what, bad[0], bad.size)
    # chunks outside the range were not touched by either call
    assert np.all(got[:lo] == SENT8) and np.all(got[hi:plan.wire_bytes] == SENT8), what


def test_two_calls_in_a_row_the_second_smaller():
    stream = dev.current_stream()
    big, big_keep, big_ptrs = model_case("small_dense_tp1_to_tp4", 64 * 1024)     # many chunks: wire table in the array
    small, small_keep, small_ptrs = model_case("cfg1_tiny_tp2_to_tp1", 1 << 20)   # 3 chunks: wire pointers inline
    assert big.num_chunks > 8 >= small.num_chunks and big.num_tensors(0) > small.num_tensors(0)
    assert_equal_wire(big, big_ptrs, 0, big.num_chunks, stream, "larger plan")
    assert_equal_wire(small, small_ptrs, 0, small.num_chunks, stream, "smaller plan after the larger one")
    assert_equal_wire(big, big_ptrs, 3, big.num_chunks - 5, stream, "chunk sub-range of the larger plan")
    assert_equal_wire(small, small_ptrs, 1, 1, stream, "one chunk of the smaller plan")
    big.destroy()
    small.destroy()


def test_more_tensors_than_one_argument_batch_and_narrowing():
    """600 fp32 tensors (three batches of table entries) narrowed to bf16, then 100 of another pool."""
    stream = dev.current_stream()
    a, a_keep, a_ptrs = scatter_case(600, 41, 32 * 1024)
    b, b_keep, b_ptrs = scatter_case(100, 42, 4 * 1024)
    assert a.num_chunks > 8 and b.num_chunks > 8
    assert_equal_wire(a, a_ptrs, 0, a.num_chunks, stream, "600 tensors")
    assert_equal_wire(b, b_ptrs, 0, b.num_chunks, stream, "100 tensors after 600")
    a.destroy()
    b.destroy()


def test_calls_back_to_back_without_a_wait_between_them():
    """Stream order alone keeps the second call's table writes behind the first call's kernel."""
    stream = dev.current_stream()
    big, big_keep, big_ptrs = model_case("small_dense_tp1_to_tp4", 64 * 1024)
    small, small_keep, small_ptrs = model_case("cfg1_tiny_tp2_to_tp1", 64 * 1024)
    assert small.num_chunks > 8
    want = []
    for plan, ptrs in ((big, big_ptrs), (small, small_ptrs)):
        wire, wptrs = dev.alloc_wire(plan, fill_byte=SENT8)
        th.th_pack(plan, ptrs, wptrs, 0, plan.num_chunks, stream)
        want.append(wire)
    got = []
    for _ in range(3):
        for plan, ptrs in ((big, big_ptrs), (small, small_ptrs)):
            wire, wptrs = dev.alloc_wire(plan, fill_byte=SENT8)
            th.th_pack_noalloc(plan, ptrs, wptrs, 0, plan.num_chunks, stream)
            got.append(wire)
    torch.cuda.synchronize()
    for i, g in enumerate(got):
        assert torch.equal(g, want[i % 2]), "call %d" % i
    big.destroy()
    small.destroy()


def test_limits_and_argument_errors():
    stream = dev.current_stream()
    plan, keep, ptrs = model_case("cfg1_tiny_tp2_to_tp1", 1 << 20)
    wire, wptrs = dev.alloc_wire(plan, fill_byte=SENT8)
    with pytest.raises(th.ThError) as e:
        th.th_pack_noalloc(plan, ptrs[:-1], wptrs, 0, plan.num_chunks, stream)
    assert e.value.code == -1
    with pytest.raises(th.ThError) as e:
        th.th_pack_noalloc(plan, ptrs, wptrs[:1], plan.num_chunks, 1, stream)
    assert e.value.code == -4
    bad = ptrs.copy()
    bad[1] += 2
    with pytest.raises(th.ThError) as e:
        th.th_pack_noalloc(plan, bad, wptrs, 0, plan.num_chunks, stream)
    assert e.value.code == -1 and "misaligned" in str(e.value)
    torch.cuda.synchronize()
    assert bool((wire == SENT8).all())          # nothing ran
    plan.destroy()
    # more source tensors than the fixed table holds: refused with a clear message
    n = 5000
    segs = np.zeros(n, dtype=th.binding.SEGMENT_NP)
    segs["src_tensor"] = np.arange(n)
    segs["nrows"], segs["row_len"] = 1, 8
    segs["src_row_stride"] = segs["dst_row_stride"] = 8
    segs["dst_elem_off"] = np.arange(n) * 8
    segs["src_dtype"] = segs["dst_dtype"] = th.TH_BF16
    many = th.th_plan_create_from_segments(segs, np.full(n, 8), [8 * n], 1 << 20)
    src = torch.zeros(8 * n, dtype=torch.bfloat16, device="cuda")
    sp = src.data_ptr() + np.arange(n, dtype=np.uint64) * np.uint64(16)
    wire, wptrs = dev.alloc_wire(many, fill_byte=SENT8)
    with pytest.raises(th.ThError) as e:
        th.th_pack_noalloc(many, sp, wptrs, 0, many.num_chunks, stream)
    assert e.value.code == -4 and "4096" in str(e.value)
    th.th_pack(many, sp, wptrs, 0, many.num_chunks, stream)     # the allocating entry point takes it
    torch.cuda.synchronize()
    assert not bool(wire[:many.wire_bytes].any())
    many.destroy()
