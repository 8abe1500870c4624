"""GPU parity at the full benchmark sizes, in the launch configuration bench.py
times (default tile size, all chunks in one call).  The oracle cannot hold these
workloads whole, so it is streamed: holder tensor by holder tensor (segment by
segment for the scattered sweep) the source bits come back from the device, the
oracle computes what that tensor puts on the wire, and the GPU's wire bytes and
the place where they landed in the reader's tensors are compared bit for bit.
Every holder tensor and every segment goes through it; properties that hold at
any size (sentinels in what the plan does not own, zero gaps, sums of 16-bit
halves) are checked on top."""
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import synth
import paper_2604_09107_amd as th
from paper_2604_09107_amd import device as dev
from oracle import checksum, layouts, reshard, segments
from test_planner_manifest import scatter_segments

pytestmark = pytest.mark.gpu

ORACLE_THREADS = 16   # numpy indexing and the C narrowing routine release the interpreter lock


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


class Backlog:
    """Oracle comparisons queued on a thread pool, bounded by the bytes they hold."""

    def __init__(self, limit_bytes=8 << 30):
        self.pool = ThreadPoolExecutor(ORACLE_THREADS)
        self.limit = limit_bytes
        self.pending = []   # (future, bytes)
        self.held = 0

    def submit(self, nbytes, fn, *args):
        while self.pending and self.held + nbytes > self.limit:
            f, b = self.pending.pop(0)
            f.result()
            self.held -= b
        self.pending.append((self.pool.submit(fn, *args), nbytes))
        self.held += nbytes

    def drain(self):
        for f, _ in self.pending:
            f.result()
        self.pending, self.held = [], 0
        self.pool.shutdown()


def compare_item(it, src_bits, got_wire, dst_bits, src_name, dst_name):
    want = reshard.item_wire(it, src_bits)
    assert np.array_equal(got_wire.view(want.dtype), want), "wire of %s differs" % src_name
    landed = dst_bits[np.ix_(it["dst_r"], it["dst_c"])]
    assert np.array_equal(landed.reshape(-1), want), "%s landed wrong in %s" % (src_name, dst_name)


def run_model_fullsize(name, part=0, holders=None):
    """Packs and unpacks every chosen holder of the workload's part, then streams every plan item
    through the oracle.  Returns what the any-size checks need."""
    w = synth.workload(name)
    model, dst = w["model"], w["parts"][part]["reader"]
    w["holders"] = [h for i, h in enumerate(w["parts"][part]["holders"]) if holders is None or i in holders]
    lts = layouts.logical_tensors(model)
    stream = dev.current_stream()
    dst_dev = None
    dst_regs = layouts.registered_tensors(model, dst)
    wire_sum = 0
    covered = 0
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
        backlog = Backlog()
        src_cache, dst_cache = (None, None), (None, None)
        checked, prev_end, senders = 0, 0, set()
        for it in reshard.plan_items(model, src, dst):
            sid, did = it["src_id"], it["dst_id"]
            if src_cache[0] != sid:
                src_cache = (sid, synth.to_bits(src_dev[sid]).reshape(regs[sid]["rows"], regs[sid]["cols"]))
            if dst_cache[0] != did:
                dst_cache = (did, synth.to_bits(dst_dev[did]).reshape(dst_regs[did]["rows"], dst_regs[did]["cols"]))
            n = len(it["src_r"]) * len(it["src_c"])
            nb = n * reshard.ESIZE[it["wire_dtype"]]
            off = it["wire_off"]
            # the alignment gap in front of the item is zero
            assert off - prev_end <= 14 and (off == prev_end or not wire_dev[prev_end:off].any().item())
            prev_end = off + nb
            got = wire_dev[off:off + nb].cpu().numpy()
            backlog.submit(src_cache[1].nbytes + dst_cache[1].nbytes + nb, compare_item, it, src_cache[1], got,
                           dst_cache[1], regs[sid]["name"], dst_regs[did]["name"])
            checked += 1
            covered += n
            senders.add(sid)
        backlog.drain()
        assert prev_end == plan.wire_bytes
        log("oracle agreed on all %d plan items (%d of %d holder tensors send)" % (checked, len(senders), len(regs)))
        assert checked > 0
        plan.destroy()
        del src_dev, wire_dev
    return w, dst_dev, dst_regs, wire_sum, covered


def reader_elements(dst_regs):
    return sum(t["rows"] * t["cols"] for t in dst_regs)


def test_8b_tp1_to_tp4_full_size():
    w, dst_dev, dst_regs, wire_sum, covered = run_model_fullsize("cfg2_8b_tp1_to_tp4")
    # every element of the reader's shard was covered by a plan item (each verified in place above)
    assert covered == reader_elements(dst_regs)
    assert sum(int16_sum(t) for t in dst_dev) == wire_sum


def test_70b_tp8_to_tp4_full_size():
    w, dst_dev, dst_regs, wire_sum, covered = run_model_fullsize("cfg3_70b_tp8_to_tp4")
    assert covered == reader_elements(dst_regs)
    assert sum(int16_sum(t) for t in dst_dev) == wire_sum


def test_moe_ep8_to_tp2_full_size():
    w, dst_dev, dst_regs, wire_sum, covered = run_model_fullsize("cfg4_moe_ep8_to_tp2")
    # experts 8..63 of the stacked tensors belong to other holders: their slabs keep the sentinel
    for t, reg in zip(dst_dev, dst_regs):
        if ".experts.w" in reg["name"]:
            slabs = t.view(torch.int16).view(64, -1)
            assert bool((slabs[8:] == 0x7FA5).all()), reg["name"]
            assert not bool((slabs[:8] == 0x7FA5).all())


def scatter_oracle_segments(d, n):
    return dict(src_tensor=d["seg_src_tensor"], dst_tensor=np.zeros(n, dtype=np.int64),
                src_off=d["seg_src_off"], src_stride=d["seg_src_stride"], dst_off=d["seg_dst_off"],
                dst_stride=d["seg_dst_stride"], nrows=d["seg_nrows"], row_len=d["seg_row_len"])


def for_every_scatter_segment(d, pool_dev, fn, batch_elems=1 << 29):
    """Calls fn(k, sources) for every segment k of the scattered sweep on the oracle's thread pool.
    The fp32 pool comes back from the device in batches of consecutive tensors (2 GiB each);
    `sources` maps a tensor id of the batch to its bits."""
    n = len(d["n_elems"])
    where = np.empty(n, dtype=np.int64)          # tensor id -> position of its segment in the wire order
    where[d["seg_src_tensor"]] = np.arange(n)
    backlog = Backlog(limit_bytes=12 << 30)
    t = 0
    while t < n:
        t_end = t
        while t_end < n and (t_end == t or d["pool_off"][t_end] + d["n_elems"][t_end] - d["pool_off"][t] <= batch_elems):
            t_end += 1
        base = int(d["pool_off"][t])
        stop = int(d["pool_off"][t_end - 1] + d["n_elems"][t_end - 1])
        block = synth.to_bits(pool_dev[base:stop])
        srcs = {i: block[int(d["pool_off"][i]) - base:int(d["pool_off"][i]) - base + int(d["n_elems"][i])]
                for i in range(t, t_end)}

        def batch(ids, srcs=srcs):
            for i in ids:
                fn(int(where[i]), srcs)

        ids = np.arange(t, t_end)
        for part in np.array_split(ids, min(len(ids), 4 * ORACLE_THREADS)):
            backlog.submit(block.nbytes // (4 * ORACLE_THREADS), batch, part)
        t = t_end
    backlog.drain()


@pytest.mark.parametrize("name,arena_shift", [("cfg5_scatter_fp32_to_bf16", 0), ("cfg5_scatter_fp32_to_bf16", 1),
                                              ("tiny_tensors_fp32_to_bf16", 0)])
def test_scattered_sweep_full_size(name, arena_shift):
    """100,000 fp32 tensors (about 40 GB) narrowed into a dense bf16 arena through 16 MiB chunks; and
    400,000 tensors of 256 B to 4 KiB the same way (every run short: one wavefront each).
    arena_shift 0: the arena starts on a cache line, as in the benchmark (tiles that start on a line
    take the write-through stores); 1: it starts one element later, so nothing is aligned."""
    w = synth.workload(name)
    n, seed, chunk = w["n_tensors"], w["seed"], w["chunk_bytes"]
    d = synth.scatter_description(n, seed, **w["sizes"])
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
    osegs = scatter_oracle_segments(d, n)
    offs, total = segments.wire_offsets(osegs, "bf16")
    assert total == plan.wire_bytes
    assert plan.payload_bytes == 2 * d["arena_elems"] and plan.src_read_bytes == 4 * d["arena_elems"]
    wire_host = wire_dev.cpu().numpy()
    arena_host = synth.to_bits(arena[:d["arena_elems"]])
    log("wire and arena on the host")

    def compare(k, srcs):
        want = segments.segment_wire(osegs, k, srcs, "f32", "bf16")
        lo = int(offs[k])
        assert np.array_equal(wire_host[lo:lo + want.nbytes].view(np.uint16), want), "wire of segment %d differs" % k
        a = int(d["seg_dst_off"][k])
        assert np.array_equal(arena_host[a:a + len(want)], want), "segment %d landed wrong" % k
        # the gap up to the next segment's start is zero
        end = lo + want.nbytes
        nxt = int(offs[k + 1]) if k + 1 < n else end
        assert nxt - end <= 14 and not wire_host[end:nxt].any()

    for_every_scatter_segment(d, pool_dev, compare)
    log("oracle agreed on all %d segments" % n)
    # any-size properties: arena = every wire element exactly once (sums of 16-bit halves agree, gaps are
    # zero and add nothing), guard elements around the arena untouched
    assert int16_sum(arena[:d["arena_elems"]]) == int16_sum(wire_dev[:plan.wire_bytes])
    g = synth.to_bits(arena_dev)
    assert np.all(g[:arena_shift] == 0x7FA5) and np.all(g[d["arena_elems"] + arena_shift:] == 0x7FA5)
    plan.destroy()


def test_8b_last_reader_rank_full_size():
    w, dst_dev, dst_regs, wire_sum, covered = run_model_fullsize("cfg2_8b_tp1_to_tp4_all_readers", part=3)
    assert covered == reader_elements(dst_regs)
    assert sum(int16_sum(t) for t in dst_dev) == wire_sum


def test_70b_second_reader_full_size():
    w, dst_dev, dst_regs, wire_sum, covered = run_model_fullsize("cfg3_70b_tp8_to_tp4_two_readers", part=1)
    assert covered == reader_elements(dst_regs)
    assert sum(int16_sum(t) for t in dst_dev) == wire_sum


def test_moe_other_holder_full_size():
    """A holder that is not the reader's primary source sends its eight experts and nothing else."""
    w, dst_dev, dst_regs, wire_sum, covered = run_model_fullsize("cfg4_moe_ep8_to_tp2_all_holders", holders={5})
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


@pytest.mark.parametrize("name", ["cfg2_8b_tp1_to_tp4", "cfg4_moe_ep8_to_tp2"])
def test_model_checksums_full_size(name):
    """Fused checksums in the configuration the benchmark's checksum sweep times: both sides agree
    for every holder tensor, the oracle (from the source bits alone) agrees on every one of them, and
    the reader tensors equal those of the plain calls."""
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
    backlog = Backlog()
    cache = (None, None)
    open_run = {}

    def check_run(t, parts):
        lo = min(o for o, _ in parts)
        run = np.zeros(max(o + len(b) for o, b in parts) - lo, dtype=np.uint8)
        for o, b in parts:
            run[o - lo:o - lo + len(b)] = b
        assert tuple(int(v) for v in got_p[t]) == checksum.run_checksum(run), regs[t]["name"]

    def run_of(t, items, bits):
        check_run(t, [(it["wire_off"], reshard.item_wire(it, bits).view(np.uint8)) for it in items])

    n_runs = 0
    for it in list(reshard.plan_items(model, src, dst)) + [None]:
        if open_run and (it is None or it["src_id"] != open_run["t"]):   # a tensor's items are consecutive
            backlog.submit(open_run["bits"].nbytes, run_of, open_run["t"], open_run["items"], open_run["bits"])
            n_runs += 1
            open_run = {}
        if it is None:
            break
        if not open_run:
            reg = regs[it["src_id"]]
            open_run = dict(t=it["src_id"], items=[],
                            bits=synth.to_bits(src_dev[it["src_id"]]).reshape(reg["rows"], reg["cols"]))
        open_run["items"].append(it)
    backlog.drain()
    sends = {it["src_id"] for it in reshard.plan_items(model, src, dst)}
    for t in range(len(regs)):
        if t not in sends:
            assert not got_p[t].any(), regs[t]["name"]
    log("oracle agreed on the checksums of all %d sending tensors" % n_runs)
    assert n_runs == len(sends)
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
    osegs = scatter_oracle_segments(d, n)

    def compare(k, srcs):
        want = segments.segment_wire(osegs, k, srcs, "f32", "bf16")
        t = int(d["seg_src_tensor"][k])
        assert tuple(int(v) for v in got_p[t]) == checksum.run_checksum(want.view(np.uint8)), "tensor %d" % t

    for_every_scatter_segment(d, pool_dev, compare)
    log("oracle agreed on the checksums of all %d tensors" % n)
    plan.destroy()
