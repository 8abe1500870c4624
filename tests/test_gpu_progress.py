"""The progress counter that one launch advances while it runs (th_pack_progress /
th_unpack_progress): results bit for bit against the oracle, and the counter's contract observed
from the host - it starts at 0, only grows, ends at the number of chunks, and a chunk below the
counter is complete at the moment the host sees the counter pass it."""
import time

import numpy as np
import pytest
import torch

import synth
import paper_2604_09107_amd as th
from paper_2604_09107_amd import device as dev
from oracle import layouts, reshard
from helpers import holder_tensors_cpu

pytestmark = pytest.mark.gpu

SENT8, SENT16 = 0xEE, 0xA5C3


def to_dev(bits2d):
    return synth.from_bits(np.ascontiguousarray(bits2d).reshape(-1), "cuda")


def host_counter():
    t = torch.full((1,), -1, dtype=torch.int64, pin_memory=True)
    return t, t.numpy()


@pytest.mark.parametrize("name,chunk_bytes", [("cfg1_tiny_tp2_to_tp1", 64 * 1024), ("small_dense_tp1_to_tp4", 32 * 1024),
                                              ("small_dense_tp4_to_tp2", 16 * 1024), ("small_moe_ep4_to_tp2", 16 * 1024),
                                              ("small_dense_trainer_to_rollout", 48 * 1024)])
@pytest.mark.parametrize("where", ["pinned_host", "device"])
def test_progress_calls_move_what_the_oracle_says(name, chunk_bytes, where):
    """Every holder of the workload through th_pack_progress / th_unpack_progress (all chunks, then
    two sub-ranges), wire and reader tensors against the oracle; the counter ends at the range's
    length.  Plain th_pack / th_unpack on the same plan (prefix-ordered lists) give the same bytes."""
    w = synth.workload(name)
    model, dst = w["model"], w["reader"]
    stream = dev.current_stream()
    want = reshard.empty_tensors(model, dst, fill=SENT16)
    for t, x in zip(layouts.registered_tensors(model, dst), want):
        if t["dtype"] == "f32":
            x[...] = SENT16 * 0x10001
    dst_dev = dst_plain = None
    keep, view = host_counter()
    dev_flag = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    flag_ptr = keep.data_ptr() if where == "pinned_host" else dev_flag.data_ptr()

    def flag_value():
        return int(view[0]) if where == "pinned_host" else int(dev_flag[0].item())

    for src in w["holders"]:
        plan = th.th_plan_create(model, src, dst, chunk_bytes, th.TH_FLAG_PROGRESS)
        tensors = holder_tensors_cpu(model, src, w["seed"], pattern=True)
        src_dev = [to_dev(t) for t in tensors]
        if dst_dev is None:
            dst_dev = dev.alloc_tensors(plan, 1, fill_bits=SENT16)
            dst_plain = dev.alloc_tensors(plan, 1, fill_bits=SENT16)
        n = plan.num_chunks
        assert n >= 12
        wire = reshard.pack(model, src, dst, tensors)
        reshard.unpack(model, src, dst, wire, want)
        # all chunks in one call
        wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=SENT8)
        th.th_pack_progress(plan, dev.ptrs(src_dev), wptrs, 0, n, flag_ptr, stream)
        torch.cuda.synchronize()
        assert flag_value() == n
        assert np.array_equal(wire_dev.cpu().numpy()[:plan.wire_bytes], wire)
        # two sub-ranges, the second first
        wire2, wptrs2 = dev.alloc_wire(plan, fill_byte=SENT8)
        cut = n // 3
        th.th_pack_progress(plan, dev.ptrs(src_dev), wptrs2[cut:], cut, n - cut, flag_ptr, stream)
        torch.cuda.synchronize()
        assert flag_value() == n - cut
        assert bool((wire2[:cut * chunk_bytes] == SENT8).all())
        th.th_pack_progress(plan, dev.ptrs(src_dev), wptrs2[:cut], 0, cut, flag_ptr, stream)
        torch.cuda.synchronize()
        assert flag_value() == cut
        assert torch.equal(wire2, wire_dev)
        # unpack with progress: a range, then the rest
        th.th_unpack_progress(plan, wptrs[cut:], cut, n - cut, dev.ptrs(dst_dev), flag_ptr, stream)
        torch.cuda.synchronize()
        assert flag_value() == n - cut
        th.th_unpack_progress(plan, wptrs[:cut], 0, cut, dev.ptrs(dst_dev), flag_ptr, stream)
        torch.cuda.synchronize()
        assert flag_value() == cut
        # the plain calls on the prefix-ordered plan
        wire3, wptrs3 = dev.alloc_wire(plan, fill_byte=SENT8)
        th.th_pack(plan, dev.ptrs(src_dev), wptrs3, 0, n, stream)
        th.th_unpack(plan, wptrs3, 0, n, dev.ptrs(dst_plain), stream)
        torch.cuda.synchronize()
        assert torch.equal(wire3, wire_dev)
        # an empty range completes at once
        th.th_pack_progress(plan, dev.ptrs(src_dev), wptrs[:0], n, 0, flag_ptr, stream)
        torch.cuda.synchronize()
        assert flag_value() == 0
        plan.destroy()
    for g, p, x in zip(dst_dev, dst_plain, want):
        assert np.array_equal(synth.to_bits(g), x.reshape(-1))
        assert np.array_equal(synth.to_bits(p), x.reshape(-1))


def test_counter_seen_from_the_host_during_one_launch():
    """The MoE-shaped reshard (693 chunks of 4 MiB, about 350,000 tiles) packed by one call while the
    host polls the counter in pinned memory.  Whenever the counter has moved, the newest chunk below
    it is copied to the host at once, on another stream, while the launch is still running: the copy
    must already hold the chunk's final bytes."""
    w = synth.workload("cfg4_moe_ep8_to_tp2")
    model, src, dst = w["model"], w["holders"][0], w["reader"]
    stream = dev.current_stream()
    plan = th.th_plan_create(model, src, dst, w["chunk_bytes"], th.TH_FLAG_PROGRESS)
    plain = th.th_plan_create(model, src, dst, w["chunk_bytes"])
    n, cb = plan.num_chunks, plan.chunk_bytes(0)
    src_dev = [synth.weight_values(t["rows"] * t["cols"], t["dtype"], w["seed"] * 16, i, "cuda",
                                   is_norm="norm" in t["name"]) for i, t in enumerate(plan.tensors(0))]
    wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=SENT8)
    ref_dev, rptrs = dev.alloc_wire(plain, fill_byte=SENT8)
    th.th_pack(plain, dev.ptrs(src_dev), rptrs, 0, n, stream)       # the reference wire (itself checked against the
    torch.cuda.synchronize()                                        # oracle by the full-size parity tests)
    keep, view = host_counter()
    side = torch.cuda.Stream()
    grabbed = torch.empty((64, cb), dtype=torch.uint8, pin_memory=True)
    seen, taken = [], []
    for attempt in range(3):                                        # the first call also uploads the pointer tables
        wire_dev.fill_(SENT8)
        torch.cuda.synchronize()
        seen, taken = [], []
        view[0] = -1
        th.th_pack_progress(plan, dev.ptrs(src_dev), wptrs, 0, n, keep.data_ptr(), stream)
        deadline = time.perf_counter() + 20.0
        last = -1
        while last < n and time.perf_counter() < deadline:
            v = int(view[0])
            if v != last:
                seen.append(v)
                if v > 0 and len(taken) < grabbed.shape[0]:
                    c = v - 1                                       # complete, says the counter
                    with torch.cuda.stream(side):
                        grabbed[len(taken), :plan.chunk_bytes(c)].copy_(
                            wire_dev[c * cb:c * cb + plan.chunk_bytes(c)], non_blocking=True)
                    taken.append(c)
                last = v
        torch.cuda.synchronize()
        assert last == n, "the counter stopped at %d of %d" % (last, n)
        if len(seen) > 8:
            break
    print("[progress] counter values seen by the host: %d distinct, first %s, chunks copied early: %d" % (
        len(seen), seen[:6], len(taken)), flush=True)
    assert seen[0] in (-1, 0) and seen[-1] == n
    assert all(b > a for a, b in zip(seen, seen[1:])), "the counter went backwards"
    assert len(seen) > 8, "the host never saw the launch in flight: %s" % seen
    assert torch.equal(wire_dev, ref_dev)
    ref = ref_dev.cpu().numpy()
    for k, c in enumerate(taken):
        nb = plan.chunk_bytes(c)
        assert np.array_equal(grabbed[k, :nb].numpy(), ref[c * cb:c * cb + nb]), \
            "chunk %d was reported complete before its bytes were there" % c
    # whole tensors, the paper's unit
    assert plan.tensors_complete(n) == plan.num_tensors(0)
    assert 0 < plan.tensors_complete(n // 2) < plan.num_tensors(0)
    # the unpack side: counter contract and reader tensors equal to the plain calls'
    dst_dev = dev.alloc_tensors(plan, 1, fill_bits=SENT16)
    dst_ref = dev.alloc_tensors(plain, 1, fill_bits=SENT16)
    th.th_unpack(plain, rptrs, 0, n, dev.ptrs(dst_ref), stream)
    torch.cuda.synchronize()
    view[0] = -1
    th.th_unpack_progress(plan, wptrs, 0, n, dev.ptrs(dst_dev), keep.data_ptr(), stream)
    seen_u, last = [], -1
    deadline = time.perf_counter() + 20.0
    while last < n and time.perf_counter() < deadline:
        v = int(view[0])
        if v != last:
            seen_u.append(v)
            last = v
    torch.cuda.synchronize()
    assert last == n and all(b > a for a, b in zip(seen_u, seen_u[1:]))
    for a, b in zip(dst_dev, dst_ref):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    plan.destroy()
    plain.destroy()


def test_scattered_narrowing_sweep_with_progress():
    """Explicit segments (fp32 sources at 4-byte alignment narrowed into a 2-byte aligned arena: the
    any-alignment paths, every store written through) and a plan that mixes aligned and unaligned
    runs (one list in chunk order, all-paths kernel): wire and arena against the segment oracle."""
    from oracle import segments
    from test_planner_manifest import scatter_segments
    stream = dev.current_stream()
    keep, view = host_counter()
    n, seed = 400, 23
    d = synth.scatter_description(n, seed, min_bytes=256, max_bytes=1 << 17)
    pool_dev = torch.empty(d["pool_elems"] + 4, dtype=torch.float32, device="cuda")[1:]
    pool_dev[:d["pool_elems"]] = synth.scatter_values(d["pool_elems"], seed, "cuda", 0.05)
    pool = synth.to_bits(pool_dev[:d["pool_elems"]])
    srcs = [pool[o:o + m] for o, m in zip(d["pool_off"], d["n_elems"])]
    osegs = dict(src_tensor=d["seg_src_tensor"], dst_tensor=np.zeros(n, dtype=np.int64),
                 src_off=d["seg_src_off"], src_stride=d["seg_src_stride"], dst_off=d["seg_dst_off"],
                 dst_stride=d["seg_dst_stride"], nrows=d["seg_nrows"], row_len=d["seg_row_len"])
    wire = segments.pack(osegs, srcs, "f32", "bf16")
    arena = np.full(d["arena_elems"] + 8, 0x7777, dtype=np.uint16)
    segments.unpack(osegs, wire, [arena], "bf16")
    plan = th.th_plan_create_from_segments(scatter_segments(d), d["n_elems"], [len(arena)], 16 * 1024,
                                           th.TH_FLAG_PROGRESS)
    nck = plan.num_chunks
    assert nck > 20
    src_ptrs = pool_dev.data_ptr() + d["pool_off"].astype(np.uint64) * np.uint64(4)
    arena_dev = torch.empty(len(arena) + 1, dtype=torch.bfloat16, device="cuda")
    arena_dev.view(torch.int16).fill_(0x7777)
    wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=SENT8)
    th.th_pack_progress(plan, src_ptrs, wptrs, 0, nck, keep.data_ptr(), stream)
    torch.cuda.synchronize()
    assert int(view[0]) == nck
    assert np.array_equal(wire_dev.cpu().numpy()[:plan.wire_bytes], wire)
    th.th_unpack_progress(plan, wptrs, 0, nck, [arena_dev[1:].data_ptr()], keep.data_ptr(), stream)
    torch.cuda.synchronize()
    assert int(view[0]) == nck
    assert np.array_equal(synth.to_bits(arena_dev[1:]), arena)
    plan.destroy()
    # aligned and unaligned bf16 runs in one plan
    m = 90
    segs = np.zeros(m, dtype=th.binding.SEGMENT_NP)
    segs["src_tensor"] = np.arange(m) // 3
    segs["nrows"], segs["row_len"] = 8, 2048
    segs["src_row_stride"], segs["dst_row_stride"] = 2560, 2048
    segs["src_elem_off"] = (np.arange(m) % 3) * 30000 + (np.arange(m) % 2)
    segs["dst_elem_off"] = np.arange(m) * 8 * 2048
    segs["src_dtype"] = segs["dst_dtype"] = th.TH_BF16
    plan = th.th_plan_create_from_segments(segs, np.full(m // 3, 90000), [m * 8 * 2048], 96 * 1024,
                                           th.TH_FLAG_PTRS_ALIGNED16 | th.TH_FLAG_PROGRESS)
    assert {plan.tile(0, i).kind for i in range(plan.num_tiles(0))} == {0, 2}
    assert plan.chunk_first_tile(0, 1, 0) == 0 and plan.chunk_first_tile(0, 2, 0) == plan.num_tiles(0)
    rng = np.random.default_rng(5)
    src_bits = [rng.integers(0, 1 << 16, 90000, dtype=np.uint16) for _ in range(m // 3)]
    osegs = dict(src_tensor=segs["src_tensor"].astype(np.int64), dst_tensor=np.zeros(m, dtype=np.int64),
                 src_off=segs["src_elem_off"].astype(np.int64), src_stride=segs["src_row_stride"].astype(np.int64),
                 dst_off=segs["dst_elem_off"].astype(np.int64), dst_stride=segs["dst_row_stride"].astype(np.int64),
                 nrows=segs["nrows"].astype(np.int64), row_len=segs["row_len"].astype(np.int64))
    wire = segments.pack(osegs, src_bits, "bf16", "bf16")
    src_dev = [synth.from_bits(b, "cuda") for b in src_bits]
    wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=SENT8)
    th.th_pack_progress(plan, dev.ptrs(src_dev), wptrs, 0, plan.num_chunks, keep.data_ptr(), stream)
    torch.cuda.synchronize()
    assert int(view[0]) == plan.num_chunks
    assert np.array_equal(wire_dev.cpu().numpy()[:plan.wire_bytes], wire)
    plan.destroy()


def test_argument_errors():
    w = synth.workload("cfg1_tiny_tp2_to_tp1")
    model, src, dst = w["model"], w["holders"][0], w["reader"]
    stream = dev.current_stream()
    plain = th.th_plan_create(model, src, dst, 1 << 16)
    plan = th.th_plan_create(model, src, dst, 1 << 16, th.TH_FLAG_PROGRESS)
    src_dev = [to_dev(t) for t in holder_tensors_cpu(model, src, w["seed"], pattern=True)]
    wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=SENT8)
    flag = torch.zeros(2, dtype=torch.int64, device="cuda")
    with pytest.raises(th.ThError) as e:
        th.th_pack_progress(plain, dev.ptrs(src_dev), wptrs, 0, plan.num_chunks, flag.data_ptr(), stream)
    assert e.value.code == -1 and "TH_FLAG_PROGRESS" in str(e.value)
    with pytest.raises(th.ThError) as e:
        th.th_pack_progress(plan, dev.ptrs(src_dev), wptrs, 0, plan.num_chunks, flag.data_ptr() + 4, stream)
    assert e.value.code == -1
    with pytest.raises(th.ThError) as e:
        th.th_unpack_progress(plan, wptrs, 0, plan.num_chunks, dev.ptrs(src_dev)[:1], 0, stream)
    assert e.value.code == -1
    with pytest.raises(th.ThError) as e:
        th.th_pack_progress(plan, dev.ptrs(src_dev), wptrs[:1], plan.num_chunks, 1, flag.data_ptr(), stream)
    assert e.value.code == -4
    torch.cuda.synchronize()
    assert bool((wire_dev == SENT8).all())
    plan.destroy()
    plain.destroy()


def test_progress_and_noalloc_calls_recorded_into_a_graph():
    """th_pack_progress + th_unpack_progress (kernels only: the counters are cleared by a kernel, not
    a memset) and th_pack_noalloc (which needs no earlier call outside capture) recorded into HIP
    graphs and replayed for new weight versions in the same registered tensors; every replay, with
    eager work and synchronisation between the replays, against the oracle."""
    w = synth.workload("small_dense_tp1_to_tp4")
    model, src, dst = w["model"], w["holders"][0], w["reader"]
    plan = th.th_plan_create(model, src, dst, 64 * 1024, th.TH_FLAG_PROGRESS)
    n = plan.num_chunks
    tensors = holder_tensors_cpu(model, src, 500)
    src_dev = [to_dev(t) for t in tensors]
    dst_dev = dev.alloc_tensors(plan, 1, fill_bits=SENT16)
    wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=SENT8)
    wire_na, wptrs_na = dev.alloc_wire(plan, fill_byte=SENT8)
    sp, dp = dev.ptrs(src_dev), dev.ptrs(dst_dev)
    keep, view = host_counter()
    flag2 = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    s = torch.cuda.Stream()
    # the progress calls need their pointer tables on the device before capture: one eager call each
    th.th_pack_progress(plan, sp, wptrs, 0, n, keep.data_ptr(), s.cuda_stream)
    th.th_unpack_progress(plan, wptrs, 0, n, dp, flag2.data_ptr(), s.cuda_stream)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        th.th_pack_progress(plan, sp, wptrs, 0, n, keep.data_ptr(), s.cuda_stream)
        th.th_unpack_progress(plan, wptrs, 0, n, dp, flag2.data_ptr(), s.cuda_stream)
    g_na = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_na, stream=s):
        th.th_pack_noalloc(plan, sp, wptrs_na, 0, n, s.cuda_stream)       # never called outside capture
    for rep in range(4):
        tensors = holder_tensors_cpu(model, src, 600 + rep)
        for d_, t in zip(src_dev, tensors):
            d_.copy_(to_dev(t))
        for t in dst_dev:
            t.view(torch.int16).fill_(0x25C3)
        wire_dev.fill_(SENT8)
        wire_na.fill_(SENT8)
        view[0] = -1
        flag2.fill_(-1)
        # eager work of the program's own between the replays, on the shared arrays too
        th.th_pack_noalloc(plan, sp, wptrs_na[n // 2:], n // 2, n - n // 2, dev.current_stream())
        torch.cuda.synchronize()
        wire_na.fill_(SENT8)
        torch.cuda.synchronize()
        g.replay()
        g_na.replay()
        torch.cuda.synchronize()
        wire = reshard.pack(model, src, dst, tensors)
        want = reshard.empty_tensors(model, dst, fill=0x25C3)
        for t, x in zip(layouts.registered_tensors(model, dst), want):
            if t["dtype"] == "f32":
                x[...] = 0x25C3 * 0x10001
        reshard.unpack(model, src, dst, wire, want)
        assert int(view[0]) == n and int(flag2.item()) == n, "replay %d" % rep
        assert np.array_equal(wire_dev.cpu().numpy()[:plan.wire_bytes], wire), "replay %d" % rep
        assert np.array_equal(wire_na.cpu().numpy()[:plan.wire_bytes], wire), "replay %d (noalloc)" % rep
        for g_, x in zip(dst_dev, want):
            assert np.array_equal(synth.to_bits(g_), x.reshape(-1)), "replay %d" % rep
    del g, g_na
    plan.destroy()
