"""GPU parity at the full benchmark sizes, in the launch configuration bench.py
times (default tile size, all chunks in one call).  The oracle cannot hold these
workloads whole, so it is run tensor by tensor on a sample of holder tensors
(wire bytes and landing place compared bit for bit), and properties that hold
at any size cover the rest."""
import time

import numpy as np
import pytest
import torch

import synth
import paper_2604_09107_amd as th
from paper_2604_09107_amd import device as dev
from oracle import checksum, layouts, reshard, segments
from test_planner_manifest import scatter_segments

pytestmark = pytest.mark.gpu


def log(msg):
    print("[fullsize %s] %s" % (time.strftime("%H:%M:%S"), msg), flush=True)


def int16_sum(t):
    """Sum of all 16-bit halves of a device buffer, as a Python int (exact)."""
    v = t.view(torch.int16)
    total = 0
    step = 1 << 28
    for lo in range(0, v.numel(), step):
        total += int(v[lo:lo + step].sum(dtype=torch.int64).item())
    return total


def run_model_fullsize(name, sample_fn, part=0, holders=None, sends_everything=True):
    w = synth.workload(name)
    model, dst = w["model"], w["parts"][part]["reader"]
    w["holders"] = [h for i, h in enumerate(w["parts"][part]["holders"]) if holders is None or i in holders]
    lts = layouts.logical_tensors(model)
    stream = dev.current_stream()
    dst_dev = None
    dst_regs = layouts.registered_tensors(model, dst)
    wire_sum = 0
    for h, src in enumerate(w["holders"]):
        plan = th.th_plan_create(model, src, dst, w["chunk_bytes"])
        regs = layouts.registered_tensors(model, src)
        log("%s holder %d: %d tensors, wire %.2f GB, %d chunks, %d tiles" % (
            name, h, len(regs), plan.wire_bytes / 1e9, plan.num_chunks, plan.num_tiles(0)))
        src_dev = [synth.weight_values(t["rows"] * t["cols"], t["dtype"], w["seed"] * 16 + h, i, "cuda",
                                       is_norm=lts[t["parts"][0][0]]["role"] == "norm")
                   for i, t in enumerate(regs)]
        if dst_dev is None:
            dst_dev = dev.alloc_tensors(plan, 1, fill_bits=0x7FA5)
        wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=0xEE)
        th.th_pack(plan, dev.ptrs(src_dev), wptrs, 0, plan.num_chunks, stream)
        th.th_unpack(plan, wptrs, 0, plan.num_chunks, dev.ptrs(dst_dev), stream)
        torch.cuda.synchronize()
        log("packed + unpacked")
        assert plan.wire_bytes == reshard.wire_bytes(model, src, dst)
        wire_sum += int16_sum(wire_dev[:plan.wire_bytes])
        sample = set(sample_fn(regs))
        checked = 0
        dst_cache = {}
        for it in reshard.plan_items(model, src, dst):
            if it["src_id"] not in sample:
                continue
            reg = regs[it["src_id"]]
            src_bits = synth.to_bits(src_dev[it["src_id"]]).reshape(reg["rows"], reg["cols"])
            want = reshard.item_wire(it, src_bits)
            got = wire_dev[it["wire_off"]:it["wire_off"] + want.nbytes].cpu().numpy().view(want.dtype)
            assert np.array_equal(got, want), "wire of %s differs" % reg["name"]
            if it["dst_id"] not in dst_cache:
                dst_cache = {it["dst_id"]: synth.to_bits(dst_dev[it["dst_id"]]).reshape(
                    dst_regs[it["dst_id"]]["rows"], dst_regs[it["dst_id"]]["cols"])}
            landed = dst_cache[it["dst_id"]][np.ix_(it["dst_r"], it["dst_c"])]
            assert np.array_equal(landed.reshape(-1), want), "%s landed wrong in %s" % (
                reg["name"], dst_regs[it["dst_id"]]["name"])
            checked += 1
        log("oracle agreed on %d sampled plan items" % checked)
        assert checked > 0
        if sends_everything:
            assert checked >= len(sample) - 2 * len([t for t in regs if "norm" in t["name"]])
        plan.destroy()
        del src_dev, wire_dev
    return w, dst_dev, dst_regs, wire_sum


def layer_sample(regs, layers):
    keep = []
    for i, t in enumerate(regs):
        n = t["name"]
        if not n.startswith("layers.") or int(n.split(".")[1]) in layers:
            keep.append(i)
    return keep


def test_8b_tp1_to_tp4_full_size():
    w, dst_dev, dst_regs, wire_sum = run_model_fullsize(
        "cfg2_8b_tp1_to_tp4", lambda regs: layer_sample(regs, {0, 17, 31}))
    # the reader's shard is covered completely: same multiset of 16-bit halves as the wire
    assert sum(int16_sum(t) for t in dst_dev) == wire_sum


def test_70b_tp8_to_tp4_full_size():
    w, dst_dev, dst_regs, wire_sum = run_model_fullsize(
        "cfg3_70b_tp8_to_tp4", lambda regs: layer_sample(regs, {0, 41, 79}))
    assert sum(int16_sum(t) for t in dst_dev) == wire_sum


def test_moe_ep8_to_tp2_full_size():
    w, dst_dev, dst_regs, wire_sum = run_model_fullsize(
        "cfg4_moe_ep8_to_tp2", lambda regs: layer_sample(regs, {0, 11, 23}))
    # experts 8..63 of the stacked tensors belong to other holders: their slabs keep the sentinel
    for t, reg in zip(dst_dev, dst_regs):
        if ".experts.w" in reg["name"]:
            slabs = t.view(torch.int16).view(64, -1)
            assert bool((slabs[8:] == 0x7FA5).all()), reg["name"]
            assert not bool((slabs[:8] == 0x7FA5).all())


@pytest.mark.parametrize("arena_shift", [0, 1])
def test_scattered_sweep_full_size(arena_shift):
    """100,000 fp32 tensors (about 40 GB) narrowed into a dense bf16 arena through 16 MiB chunks.
    arena_shift 0: the arena starts on a cache line, as in the benchmark (tiles that start on a line
    take the write-through stores); 1: it starts one element later, so nothing is aligned."""
    n, seed, chunk = 100_000, 5, 16 << 20
    d = synth.scatter_description(n, seed)
    log("pool %.1f GB, arena %.1f GB" % (d["pool_elems"] * 4 / 1e9, d["arena_elems"] * 2 / 1e9))
    pool_dev = synth.scatter_values(d["pool_elems"] + 3, seed, "cuda")[1:]   # 4-byte aligned only
    arena_dev = torch.empty(d["arena_elems"] + 9, dtype=torch.bfloat16, device="cuda")
    arena_dev.view(torch.int16).fill_(0x7FA5)
    arena = arena_dev[arena_shift:]
    log("inputs generated")
    plan = th.th_plan_create_from_segments(scatter_segments(d), d["n_elems"], [d["arena_elems"] + 8], chunk)
    wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=0xEE)
    src_ptrs = pool_dev.data_ptr() + d["pool_off"].astype(np.uint64) * np.uint64(4)
    stream = dev.current_stream()
    th.th_pack(plan, src_ptrs, wptrs, 0, plan.num_chunks, stream)
    th.th_unpack(plan, wptrs, 0, plan.num_chunks, [arena.data_ptr()], stream)
    torch.cuda.synchronize()
    log("packed + unpacked: wire %.2f GB in %d chunks, %d / %d tiles" % (
        plan.wire_bytes / 1e9, plan.num_chunks, plan.num_tiles(0), plan.num_tiles(1)))
    osegs = dict(src_tensor=d["seg_src_tensor"], dst_tensor=np.zeros(n, dtype=np.int64),
                 src_off=d["seg_src_off"], src_stride=d["seg_src_stride"], dst_off=d["seg_dst_off"],
                 dst_stride=d["seg_dst_stride"], nrows=d["seg_nrows"], row_len=d["seg_row_len"])
    offs, total = segments.wire_offsets(osegs, "bf16")
    assert total == plan.wire_bytes
    assert plan.payload_bytes == 2 * d["arena_elems"] and plan.src_read_bytes == 4 * d["arena_elems"]
    # sample: random segments, the smallest and the largest ones, and the first / last on the wire
    rng = np.random.default_rng(seed)
    size = d["seg_nrows"] * d["seg_row_len"]
    order = np.argsort(size)
    ks = set(rng.choice(n, 1500, replace=False).tolist()) | set(order[:200].tolist()) | set(order[-12:].tolist())
    ks |= {0, 1, n - 2, n - 1}

    class Lazy:  # source tensors fetched from the device on demand
        def __getitem__(self, t):
            o, m = int(d["pool_off"][t]), int(d["n_elems"][t])
            return synth.to_bits(pool_dev[o:o + m])

    for k in sorted(ks):
        want = segments.segment_wire(osegs, k, Lazy(), "f32", "bf16")
        got = wire_dev[int(offs[k]):int(offs[k]) + want.nbytes].cpu().numpy().view(np.uint16)
        assert np.array_equal(got, want), "wire of segment %d differs" % k
        a = int(d["seg_dst_off"][k])
        landed = synth.to_bits(arena[a:a + len(want)])
        assert np.array_equal(landed, want), "segment %d landed wrong" % k
        # the gap up to the next segment's start is zero
        end = int(offs[k]) + want.nbytes
        nxt = int(offs[k + 1]) if k + 1 < n else end
        assert nxt - end <= 14 and not wire_dev[end:nxt].any().item()
    log("oracle agreed on %d sampled segments" % len(ks))
    # any-size properties: arena = every wire element exactly once (sums of 16-bit halves agree, gaps are
    # zero and add nothing), guard elements around the arena untouched
    assert int16_sum(arena[:d["arena_elems"]]) == int16_sum(wire_dev[:plan.wire_bytes])
    g = synth.to_bits(arena_dev)
    assert np.all(g[:arena_shift] == 0x7FA5) and np.all(g[d["arena_elems"] + arena_shift:] == 0x7FA5)
    plan.destroy()


def test_8b_last_reader_rank_full_size():
    w, dst_dev, dst_regs, wire_sum = run_model_fullsize(
        "cfg2_8b_tp1_to_tp4_all_readers", lambda regs: layer_sample(regs, {1, 30}), part=3)
    assert sum(int16_sum(t) for t in dst_dev) == wire_sum


def test_70b_second_reader_full_size():
    w, dst_dev, dst_regs, wire_sum = run_model_fullsize(
        "cfg3_70b_tp8_to_tp4_two_readers", lambda regs: layer_sample(regs, {2, 78}), part=1)
    assert sum(int16_sum(t) for t in dst_dev) == wire_sum


def test_moe_other_holder_full_size():
    """A holder that is not the reader's primary source sends its eight experts and nothing else."""
    w, dst_dev, dst_regs, wire_sum = run_model_fullsize(
        "cfg4_moe_ep8_to_tp2_all_holders", lambda regs: layer_sample(regs, {0, 12, 23}), holders={5}, sends_everything=False)
    for t, reg in zip(dst_dev, dst_regs):
        v = t.view(torch.int16)
        if ".experts.w" in reg["name"]:
            slabs = v.view(64, -1)
            assert bool((slabs[:40] == 0x7FA5).all()) and bool((slabs[48:] == 0x7FA5).all()), reg["name"]
            assert not bool((slabs[40:48] == 0x7FA5).all(dim=1).any())
        else:
            assert bool((v == 0x7FA5).all()), reg["name"]


def sums_host(t):
    return t.cpu().numpy().view(np.uint64).reshape(-1, 2)


@pytest.mark.parametrize("name,layers", [("cfg2_8b_tp1_to_tp4", {0, 17, 31}), ("cfg4_moe_ep8_to_tp2", {0, 23})])
def test_model_checksums_full_size(name, layers):
    """Fused checksums in the configuration the benchmark's checksum sweep times: both sides agree
    for every holder tensor, the oracle (from the source bits alone) on a sample of them, and the
    reader tensors equal those of the plain calls."""
    w = synth.workload(name)
    model, src, dst = w["model"], w["holders"][0], w["reader"]
    lts = layouts.logical_tensors(model)
    regs = layouts.registered_tensors(model, src)
    stream = dev.current_stream()
    plan = th.th_plan_create(model, src, dst, w["chunk_bytes"], th.TH_FLAG_CHECKSUM)
    plain = th.th_plan_create(model, src, dst, w["chunk_bytes"])
    src_dev = [synth.weight_values(t["rows"] * t["cols"], t["dtype"], w["seed"] * 16, i, "cuda",
                                   is_norm=lts[t["parts"][0][0]]["role"] == "norm")
               for i, t in enumerate(regs)]
    dst_dev = dev.alloc_tensors(plan, 1, fill_bits=0x7FA5)
    ref_dev = dev.alloc_tensors(plain, 1, fill_bits=0x7FA5)
    wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=0xEE)
    ps = torch.zeros(2 * len(regs), dtype=torch.int64, device="cuda")
    us = torch.zeros_like(ps)
    log("%s: %d tensors, wire %.2f GB, %d tiles" % (name, len(regs), plan.wire_bytes / 1e9, plan.num_tiles(0)))
    th.th_pack_checksum(plan, dev.ptrs(src_dev), wptrs, 0, plan.num_chunks, ps.data_ptr(), stream)
    th.th_unpack_checksum(plan, wptrs, 0, plan.num_chunks, dev.ptrs(dst_dev), us.data_ptr(), stream)
    torch.cuda.synchronize()
    log("packed + unpacked with checksums")
    got_p, got_u = sums_host(ps), sums_host(us)
    assert np.array_equal(got_p, got_u)
    sample = set(layer_sample(regs, layers))
    runs = {}
    for it in reshard.plan_items(model, src, dst):
        if it["src_id"] in sample:
            reg = regs[it["src_id"]]
            bits = synth.to_bits(src_dev[it["src_id"]]).reshape(reg["rows"], reg["cols"])
            runs.setdefault(it["src_id"], []).append((it["wire_off"], reshard.item_wire(it, bits).view(np.uint8)))
    for t, parts in runs.items():
        lo = min(o for o, _ in parts)
        run = np.zeros(max(o + len(b) for o, b in parts) - lo, dtype=np.uint8)
        for o, b in parts:
            run[o - lo:o - lo + len(b)] = b
        assert tuple(int(v) for v in got_p[t]) == checksum.run_checksum(run), regs[t]["name"]
    sends = {it["src_id"] for it in reshard.plan_items(model, src, dst)}
    for t in range(len(regs)):
        if t not in sends:
            assert not got_p[t].any(), regs[t]["name"]
    log("oracle agreed on the checksums of %d sampled tensors" % len(runs))
    assert len(runs) >= 10
    # the checksum variant moves the same data as the plain calls
    th.th_pack(plain, dev.ptrs(src_dev), wptrs, 0, plain.num_chunks, stream)
    th.th_unpack(plain, wptrs, 0, plain.num_chunks, dev.ptrs(ref_dev), stream)
    torch.cuda.synchronize()
    for a, b in zip(dst_dev, ref_dev):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    plan.destroy()
    plain.destroy()


def test_scattered_checksums_full_size():
    """Checksums of the 100,000-tensor narrowing sweep: equal on both sides for every tensor, equal
    to the oracle's for a sample (each tensor is one segment, so its run is that segment's wire)."""
    n, seed, chunk = 100_000, 5, 16 << 20
    d = synth.scatter_description(n, seed)
    pool_dev = synth.scatter_values(d["pool_elems"] + 3, seed, "cuda")[1:]
    arena_dev = torch.empty(d["arena_elems"] + 9, dtype=torch.bfloat16, device="cuda")
    arena = arena_dev[1:]
    plan = th.th_plan_create_from_segments(scatter_segments(d), d["n_elems"], [d["arena_elems"] + 8], chunk,
                                           th.TH_FLAG_CHECKSUM)
    wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=0xEE)
    src_ptrs = pool_dev.data_ptr() + d["pool_off"].astype(np.uint64) * np.uint64(4)
    ps = torch.zeros(2 * n, dtype=torch.int64, device="cuda")
    us = torch.zeros_like(ps)
    stream = dev.current_stream()
    th.th_pack_checksum(plan, src_ptrs, wptrs, 0, plan.num_chunks, ps.data_ptr(), stream)
    th.th_unpack_checksum(plan, wptrs, 0, plan.num_chunks, [arena.data_ptr()], us.data_ptr(), stream)
    torch.cuda.synchronize()
    log("scattered sweep packed + unpacked with checksums")
    got_p, got_u = sums_host(ps), sums_host(us)
    assert np.array_equal(got_p, got_u)
    assert np.array_equal(np.sort(d["seg_src_tensor"]), np.arange(n))   # one segment per tensor, wire order shuffled
    osegs = dict(src_tensor=d["seg_src_tensor"], dst_tensor=np.zeros(n, dtype=np.int64),
                 src_off=d["seg_src_off"], src_stride=d["seg_src_stride"], dst_off=d["seg_dst_off"],
                 dst_stride=d["seg_dst_stride"], nrows=d["seg_nrows"], row_len=d["seg_row_len"])
    rng = np.random.default_rng(seed + 1)
    size = d["seg_nrows"] * d["seg_row_len"]
    order = np.argsort(size)
    ks = set(rng.choice(n, 800, replace=False).tolist()) | set(order[:100].tolist()) | set(order[-8:].tolist())
    ks |= {0, n - 1}

    class Lazy:
        def __getitem__(self, t):
            o, m = int(d["pool_off"][t]), int(d["n_elems"][t])
            return synth.to_bits(pool_dev[o:o + m])

    for k in sorted(ks):
        want = segments.segment_wire(osegs, k, Lazy(), "f32", "bf16")
        t = int(d["seg_src_tensor"][k])
        assert tuple(int(v) for v in got_p[t]) == checksum.run_checksum(want.view(np.uint8)), "tensor %d" % t
    log("oracle agreed on the checksums of %d sampled tensors" % len(ks))
    plan.destroy()
