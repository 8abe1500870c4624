"""Benchmark of the reshard hot path on one MI355X.

One step = th_pack of every chunk + th_unpack of every chunk of the workload's
plan(s), inputs resident in HBM.  Prints one JSON line.  Byte accounting: a
bf16 element costs 2 bytes read + 2 written per direction (8 per sweep), a
narrowed fp32 element 4 + 2 at pack and 2 + 2 at unpack (10 per sweep).  The
plan (host planner + one table upload) is created once per (holder, reader,
model) and reused for every weight version, so it is timed separately and
reported as plan_ms.

Without --workload the line is the 70B-shaped reshard (the largest single-GPU
configuration, two plans, about 106 GB resident) and carries the 8B-shaped
reshard as a second, complete block under "secondary": the two workloads the
bandwidth target is stated for.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published peak
PRIMARY, SECONDARY = "cfg3_70b_tp8_to_tp4", "cfg2_8b_tp1_to_tp4"

# HBM bytes per launch (FETCH_SIZE + WRITE_SIZE from two rocprofv3 --pmc runs, each scaled by what
# the counter reads for th_reference_copy of known size; summaries under profiles/).  Valid only for
# the kernel sources they were taken with: bench.py reports null once those files have changed.
TRAFFIC_SOURCES = ("th_kernels.hip", "th_planner.cpp", "th_internal.hpp")
TRAFFIC_SHA256 = "070358030b56162ce929f6e75ccc9f7c200d40d1f79d6cb8095b91f4b1bed5b1"
TRAFFIC_BYTES = {
    "cfg2_8b_tp1_to_tp4": {"th_pack": 8047590041, "th_unpack": 8046980732},
    "cfg3_70b_tp8_to_tp4": {"th_pack": 35349565265, "th_unpack": 35348346210},
    "cfg4_moe_ep8_to_tp2": {"th_pack": 5821519863, "th_unpack": 5821209113},
    "cfg5_scatter_fp32_to_bf16": {"th_pack": 36887235165, "th_unpack": 22477880886},
}


def measured_traffic(workload, kernel):
    import hashlib
    h = hashlib.sha256()
    for f in TRAFFIC_SOURCES:
        h.update(open(os.path.join(ROOT, "paper_2604_09107_amd", "csrc", f), "rb").read())
    if h.hexdigest() != TRAFFIC_SHA256:
        return None
    return TRAFFIC_BYTES.get(workload, {}).get(kernel)


def build_inputs(th, dev, synth, w, torch):
    """Plans, resident source tensors, wire buffers and destination tensors of a model workload.
    Tensor shapes and dtypes come from the plan; a tensor whose name says it is a normalisation
    weight holds ones, every other one seeded N(0, 0.02) values."""
    model = w["model"]
    jobs = []
    resident = {}          # holder layout -> its tensors in HBM (a holder feeding several readers is resident once)
    plan_ms = 0.0
    for part in w["parts"]:
        dst = part["reader"]
        dst_dev = None
        for src in part["holders"]:
            t0 = time.perf_counter()
            plan = th.th_plan_create(model, src, dst, w["chunk_bytes"])
            plan_ms += (time.perf_counter() - t0) * 1e3
            regs = plan.tensors(0)
            key = tuple(sorted(src.items()))
            if key not in resident:
                h = len(resident)
                resident[key] = [synth.weight_values(t["rows"] * t["cols"], t["dtype"], w["seed"] * 16 + h, i, "cuda",
                                                     is_norm="norm" in t["name"])
                                 for i, t in enumerate(regs)]
            src_dev = resident[key]
            if dst_dev is None:
                dst_dev = dev.alloc_tensors(plan, 1, fill_bits=0)
            wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=0)
            jobs.append(dict(plan=plan, make_plan=lambda flags, src=src, dst=dst: th.th_plan_create(
                                 model, src, dst, w["chunk_bytes"], flags), src=src_dev, src_ptrs=dev.ptrs(src_dev), wire=wire_dev,
                             wptrs=wptrs, layout=src, reader=dst, regs=regs, dst=dst_dev, dst_ptrs=dev.ptrs(dst_dev)))
    return jobs, plan_ms


def host_threads():
    """Threads the all-cores leg uses: the cores this process may run on."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        n = min(n, int(env))
    return max(1, n)


def run_timed(work, n_threads):
    """Seconds to run the callables in `work`, one after the other or on a pool of threads (numpy's
    indexing and the C narrowing routine release the interpreter lock)."""
    if n_threads == 1:
        t0 = time.perf_counter()
        for f in work:
            f()
        return time.perf_counter() - t0
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(n_threads) as pool:
        t0 = time.perf_counter()
        list(pool.map(lambda f: f(), work))
        return time.perf_counter() - t0


def baseline_record(sweep_bytes, t1, tn, threads, what):
    return dict(value=round(sweep_bytes / t1 / 1e9, 3), unit="GB/s", cores=1, kind="oracle",
                all_cores=dict(value=round(sweep_bytes / tn / 1e9, 3), unit="GB/s", cores=threads,
                               host_cores=os.cpu_count()),
                sample="%s (%.2f GB moved; %.1f s on one thread, %.1f s on %d threads)"
                       % (what, sweep_bytes / 1e9, t1, tn, threads))


def cpu_baseline(synth, w, jobs, budget_bytes=20e9):
    """The oracle as it stands, on the host cores, over a bounded prefix of the same workload: plan
    items (holder tensors in wire order) until about budget_bytes of sweep bytes (about 10 s on one
    thread), first on one thread, then the same items on all cores (one item per task)."""
    import numpy as np
    from oracle import layouts, reshard
    model = w["model"]
    job = jobs[0]
    dst = job["reader"]
    dst_regs = layouts.registered_tensors(model, dst)
    items, srcs, sweep_bytes = [], {}, 0
    for it in reshard.plan_items(model, job["layout"], dst):
        reg = job["regs"][it["src_id"]]
        if it["src_id"] not in srcs:                                           # D2H, not timed
            srcs[it["src_id"]] = synth.to_bits(job["src"][it["src_id"]]).reshape(reg["rows"], reg["cols"])
        n = len(it["src_r"]) * len(it["src_c"])
        sweep_bytes += n * (reshard.ESIZE[it["src_dtype"]] + 3 * reshard.ESIZE[it["dst_dtype"]])
        items.append(it)
        if sweep_bytes >= budget_bytes:
            break
    dst_cpu = {}
    for it in items:
        if it["dst_id"] not in dst_cpu:
            t = dst_regs[it["dst_id"]]
            dst_cpu[it["dst_id"]] = np.zeros((t["rows"], t["cols"]), dtype=reshard.NPBITS[t["dtype"]])

    def one(it):
        def f():
            wire = reshard.item_wire(it, srcs[it["src_id"]])                                  # pack: gather + convert
            nr, nc = len(it["src_r"]), len(it["src_c"])
            dst_cpu[it["dst_id"]][np.ix_(it["dst_r"], it["dst_c"])] = wire.reshape(nr, nc)   # unpack: scatter
        return f

    work = [one(it) for it in items]
    threads = host_threads()
    t1 = run_timed(work, 1)
    tn = run_timed(work, threads)
    return baseline_record(sweep_bytes, t1, tn, threads,
                           "first %d plan items of the workload in wire order" % len(items))


def build_scatter_inputs(th, dev, synth, w, torch):
    """The scattered sweep: fp32 pool (4-byte aligned tensors), explicit segments, dense bf16 arena."""
    import numpy as np
    d = synth.scatter_description(w["n_tensors"], w["seed"], **w["sizes"])
    pool = synth.scatter_values(d["pool_elems"] + 3, w["seed"], "cuda")[1:]
    # the arena itself starts where the allocator puts it (line-aligned); the slices inside it are only
    # 2-byte aligned
    arena_store = torch.zeros(d["arena_elems"] + 8, dtype=torch.bfloat16, device="cuda")
    arena = arena_store
    n = w["n_tensors"]
    segs = np.zeros(n, dtype=th.binding.SEGMENT_NP)
    segs["src_tensor"], segs["dst_tensor"] = d["seg_src_tensor"], 0
    segs["src_elem_off"], segs["dst_elem_off"] = d["seg_src_off"], d["seg_dst_off"]
    segs["src_row_stride"], segs["dst_row_stride"] = d["seg_src_stride"], d["seg_dst_stride"]
    segs["nrows"], segs["row_len"] = d["seg_nrows"], d["seg_row_len"]
    segs["src_dtype"], segs["dst_dtype"] = th.TH_F32, th.TH_BF16
    t0 = time.perf_counter()
    plan = th.th_plan_create_from_segments(segs, d["n_elems"], [d["arena_elems"] + 8], w["chunk_bytes"])
    plan_ms = (time.perf_counter() - t0) * 1e3
    wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=0)
    src_ptrs = pool.data_ptr() + d["pool_off"].astype(np.uint64) * np.uint64(4)
    job = dict(plan=plan, make_plan=lambda flags: th.th_plan_create_from_segments(
                   segs, d["n_elems"], [d["arena_elems"] + 8], w["chunk_bytes"], flags), src=pool, src_ptrs=src_ptrs, wire=wire_dev, wptrs=wptrs, desc=d,
               keep=arena_store, dst=[arena], dst_ptrs=np.array([arena.data_ptr()], dtype=np.uint64))
    return [job], plan_ms


def cpu_baseline_scatter(synth, w, jobs, budget_bytes=6e9):
    """The segment oracle on the host over a bounded prefix of the wire order, one thread and all cores."""
    import numpy as np
    from oracle import segments
    d, pool = jobs[0]["desc"], jobs[0]["src"]
    n = w["n_tensors"]
    osegs = dict(src_tensor=d["seg_src_tensor"], dst_tensor=np.zeros(n, dtype=np.int64),
                 src_off=d["seg_src_off"], src_stride=d["seg_src_stride"], dst_off=d["seg_dst_off"],
                 dst_stride=d["seg_dst_stride"], nrows=d["seg_nrows"], row_len=d["seg_row_len"])
    srcs, outs, sweep_bytes, k = {}, [], 0, 0
    while k < n and sweep_bytes < budget_bytes:
        t = int(d["seg_src_tensor"][k])
        o, m = int(d["pool_off"][t]), int(d["n_elems"][t])
        srcs[t] = synth.to_bits(pool[o:o + m])                           # D2H, not timed
        nel = int(d["seg_nrows"][k]) * int(d["seg_row_len"][k])
        outs.append(np.zeros(nel, dtype=np.uint16))
        sweep_bytes += nel * 10
        k += 1

    def one(i):
        def f():
            wire = segments.segment_wire(osegs, i, srcs, "f32", "bf16")  # pack: gather + narrow
            outs[i][:] = wire                                            # unpack: dense destination slice
        return f

    work = [one(i) for i in range(k)]
    threads = host_threads()
    t1 = run_timed(work, 1)
    tn = run_timed(work, threads)
    return baseline_record(sweep_bytes, t1, tn, threads, "first %d segments of the wire order" % k)


def resident_bytes(jobs):
    """Bytes of HBM the workload's inputs, wire buffers and outputs occupy (shared buffers once)."""
    seen, total = set(), 0
    for j in jobs:
        for t in (j["src"] if isinstance(j["src"], list) else [j["src"]]) + [j["wire"]] + list(j["dst"]):
            if t.data_ptr() not in seen:
                seen.add(t.data_ptr())
                total += t.numel() * t.element_size()
    return total


def time_with_events(torch, fn, reps):
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(reps):
        fn()
    c1.record()
    torch.cuda.synchronize()
    return c0.elapsed_time(c1) / reps


def measure(args, name, extras, want_cpu_baseline, mods):
    """Times one workload; returns (headline fields, everything else) as two dicts."""
    np, torch, synth, th, dev = mods
    w = synth.workload(name)
    if w["kind"] == "scatter":
        jobs, plan_ms = build_scatter_inputs(th, dev, synth, w, torch)
    else:
        jobs, plan_ms = build_inputs(th, dev, synth, w, torch)
    stream = dev.current_stream()

    pack_bytes = sum(j["plan"].src_read_bytes + j["plan"].payload_bytes for j in jobs)     # read src + write wire
    unpack_bytes = sum(2 * j["plan"].payload_bytes for j in jobs)                           # read wire + write dst
    sweep_bytes = pack_bytes + unpack_bytes

    def step(events=None):
        for call, side in ((th.th_pack, 0), (th.th_unpack, 1)):
            for j in jobs:
                n = j["plan"].num_chunks
                if events is not None:
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                if side == 0:
                    th.th_pack(j["plan"], j["src_ptrs"], j["wptrs"], 0, n, stream)
                else:
                    th.th_unpack(j["plan"], j["wptrs"], 0, n, j["dst_ptrs"], stream)
                if events is not None:
                    e1.record()
                    events[side].append((e0, e1))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = ([], [])
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # Per-launch durations from events recorded around every launch, on the launch stream, inside
    # the timed region (one kernel launch per th_pack / th_unpack call).
    n_launch = len(events[0])
    pack_all = sorted(a.elapsed_time(b) for a, b in events[0])
    unpack_all = sorted(a.elapsed_time(b) for a, b in events[1])
    pack_ms = sum(pack_all) / n_launch
    unpack_ms = sum(unpack_all) / n_launch
    k_pack = pack_bytes / len(jobs) / (pack_ms * 1e-3) / 1e9      # algorithmic bytes of an average launch
    k_unpack = unpack_bytes / len(jobs) / (unpack_ms * 1e-3) / 1e9
    dom = ("th_pack", k_pack, pack_ms) if pack_ms >= unpack_ms else ("th_unpack", k_unpack, unpack_ms)

    value = sweep_bytes / (ms_per_step * 1e-3) / 1e9
    head = {
        "value": round(value, 1), "unit": "GB/s", "ms_per_step": round(ms_per_step, 4),
        "dtype": "f32->bf16 (integer RNE)" if w["kind"] == "scatter" else "bf16",
        "config": {"workload": name, "shapes": w["model_name"], "chunk_bytes": w["chunk_bytes"],
                   "plans": len(jobs), "payload_bytes": sum(j["plan"].payload_bytes for j in jobs),
                   "sweep_bytes": sweep_bytes, "chunks": sum(j["plan"].num_chunks for j in jobs),
                   "resident_bytes": resident_bytes(jobs),
                   "tile_bytes": th.th_config_get(th.TH_CFG_TILE_BYTES),
                   "tile_bytes_any": th.th_config_get(th.TH_CFG_TILE_BYTES_ANY),
                   "tile_bytes_narrow": th.th_config_get(th.TH_CFG_TILE_BYTES_NARROW),
                   "short_tile_slots": th.th_config_get(th.TH_CFG_SHORT_TILE_SLOTS)},
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "plan_ms": round(plan_ms, 3),
        "kernels": {"th_pack": {"ms": round(pack_ms, 4), "GB/s": round(k_pack, 1),
                                "median_ms": round(pack_all[n_launch // 2], 4), "min_ms": round(pack_all[0], 4)},
                    "th_unpack": {"ms": round(unpack_ms, 4), "GB/s": round(k_unpack, 1),
                                  "median_ms": round(unpack_all[n_launch // 2], 4),
                                  "min_ms": round(unpack_all[0], 4)}},
        "roofline": {"bound": "hbm", "kernel": dom[0], "achieved": round(dom[1], 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(dom[1] / HBM_PEAK_GBPS, 4),
                     "traffic": measured_traffic(name, dom[0])},
    }
    out = {"d2d_copy_GB/s": yardsticks(jobs, stream, mods)}
    if extras:
        out.update(extra_sweeps(args, jobs, sweep_bytes, stream, mods))
    if want_cpu_baseline:
        out["cpu_baseline"] = (cpu_baseline_scatter if w["kind"] == "scatter" else cpu_baseline)(synth, w, jobs)
    for j in jobs:
        for k in ("plan", "ck_plan", "pr_plan"):
            if k in j:
                j[k].destroy()
    return head, out


def yardsticks(jobs, stream, mods):
    """What a plain device-to-device copy of the plan's payload reaches: torch's copy_ and the library's
    own copy kernel (same launch shape as the aligned path; also the known-size kernel that the HBM
    byte counters of a profile are scaled by)."""
    np, torch, synth, th, dev = mods
    nbytes = jobs[0]["plan"].payload_bytes
    a = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    b = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    for _ in range(3):
        b.copy_(a)
    torch.cuda.synchronize()
    ms = time_with_events(torch, lambda: b.copy_(a), 10)
    copy_gbps = 2 * nbytes / (ms * 1e-3) / 1e9
    n16 = nbytes // 16 * 16
    for _ in range(3):
        th.th_reference_copy(b.data_ptr(), a.data_ptr(), n16, stream)
    ms = time_with_events(torch, lambda: th.th_reference_copy(b.data_ptr(), a.data_ptr(), n16, stream), 10)
    ref_gbps = 2 * n16 / (ms * 1e-3) / 1e9
    return {"torch_copy_": round(copy_gbps, 1), "th_reference_copy": round(ref_gbps, 1), "bytes": n16}


def extra_sweeps(args, jobs, sweep_bytes, stream, mods):
    """Secondary figures of a workload: the wire-free reshard, the sweep with
    checksums, the sweep in one call per chunk (eager, as a graph, through a ring of two buffers),
    the sweep in launches that publish their own progress (alone, and with a reader consuming the
    prefix meanwhile), and the offload replica in pinned host memory."""
    np, torch, synth, th, dev = mods
    out = {}
    # plans with checksums and with a progress counter are made here, after the headline sweep was
    # timed, so that their device tables do not move the tensors of that sweep
    for j in jobs:
        j["ck_plan"] = j["make_plan"](th.TH_FLAG_CHECKSUM)
        j["pr_plan"] = j["make_plan"](th.TH_FLAG_PROGRESS)
    # co-located variant: th_reshard straight from holder tensors to reader tensors (no wire)
    direct_bytes = sum(j["plan"].src_read_bytes + j["plan"].payload_bytes for j in jobs)

    def direct():
        for j in jobs:
            th.th_reshard(j["plan"], j["src_ptrs"], j["dst_ptrs"], stream)

    for _ in range(3):
        direct()
    direct_ms = time_with_events(torch, direct, 10)
    out["th_reshard_direct"] = {"ms": round(direct_ms, 4), "GB/s": round(direct_bytes / (direct_ms * 1e-3) / 1e9, 1)}

    # sweep with the per-tensor wire checksums fused into both directions
    sums = [(torch.zeros(2 * j["plan"].num_tensors(0), dtype=torch.int64, device="cuda"),
             torch.zeros(2 * j["plan"].num_tensors(0), dtype=torch.int64, device="cuda")) for j in jobs]

    def checksum_step():
        for j, (ps, us) in zip(jobs, sums):
            ps.zero_()
            us.zero_()
            n = j["ck_plan"].num_chunks
            th.th_pack_checksum(j["ck_plan"], j["src_ptrs"], j["wptrs"], 0, n, ps.data_ptr(), stream)
        for j, (ps, us) in zip(jobs, sums):
            th.th_unpack_checksum(j["ck_plan"], j["wptrs"], 0, j["ck_plan"].num_chunks, j["dst_ptrs"], us.data_ptr(),
                                  stream)

    for _ in range(3):
        checksum_step()
    checksum_ms = time_with_events(torch, checksum_step, 10)
    checksums_agree = all(bool((ps == us).all()) for ps, us in sums)
    out["checksum_sweep"] = {"ms": round(checksum_ms, 4), "GB/s": round(sweep_bytes / (checksum_ms * 1e-3) / 1e9, 1),
                             "pack_and_unpack_sums_agree": checksums_agree}

    # streaming use: one call per chunk (a reader consuming the prefix that has arrived)
    def per_chunk_sweep():
        for j in jobs:
            for c in range(j["plan"].num_chunks):
                th.th_pack(j["plan"], j["src_ptrs"], j["wptrs"][c:c + 1], c, 1, stream)
        for j in jobs:
            for c in range(j["plan"].num_chunks):
                th.th_unpack(j["plan"], j["wptrs"][c:c + 1], c, 1, j["dst_ptrs"], stream)

    def wall_ms(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e3

    n_calls = 2 * sum(j["plan"].num_chunks for j in jobs)
    per_chunk_ms = wall_ms(per_chunk_sweep)
    out["per_chunk_calls_sweep"] = {"ms": round(per_chunk_ms, 4), "calls": n_calls,
                                    "GB/s": round(sweep_bytes / (per_chunk_ms * 1e-3) / 1e9, 1)}

    # the same prefix use in one launch per direction: the launch itself publishes how many leading
    # chunks are complete (counter in pinned host memory), nobody makes a call per chunk
    counter = torch.zeros(1, dtype=torch.int64, pin_memory=True)
    cview = counter.numpy()

    def prefix_sweep():
        for j in jobs:
            th.th_pack_progress(j["pr_plan"], j["src_ptrs"], j["wptrs"], 0, j["pr_plan"].num_chunks,
                                counter.data_ptr(), stream)
        for j in jobs:
            th.th_unpack_progress(j["pr_plan"], j["wptrs"], 0, j["pr_plan"].num_chunks, j["dst_ptrs"],
                                  counter.data_ptr(), stream)

    for _ in range(3):
        prefix_sweep()
    prefix_ms = time_with_events(torch, prefix_sweep, 10)
    out["prefix_launch_sweep"] = {"ms": round(prefix_ms, 4), "launches": 2 * len(jobs),
                                  "GB/s": round(sweep_bytes / (prefix_ms * 1e-3) / 1e9, 1)}

    # ... and a reader that consumes the prefix while the holder's launch is still running: th_pack
    # publishes its progress, the host polls the counter and hands every new batch of complete chunks
    # (a sixteenth of the plan at least) to th_unpack on a second stream
    unpack_stream = torch.cuda.Stream()

    def prefix_pipeline():
        calls = 0
        for j in jobs:
            n = j["pr_plan"].num_chunks
            batch = max(1, n // 16)
            cview[0] = 0
            unpack_stream.wait_stream(torch.cuda.current_stream())
            th.th_pack_progress(j["pr_plan"], j["src_ptrs"], j["wptrs"], 0, n, counter.data_ptr(), stream)
            taken = 0
            deadline = time.perf_counter() + 30.0
            while taken < n and time.perf_counter() < deadline:
                ready = int(cview[0])
                if ready - taken >= batch or (ready == n and ready > taken):
                    th.th_unpack(j["pr_plan"], j["wptrs"][taken:ready], taken, ready - taken, j["dst_ptrs"],
                                 unpack_stream.cuda_stream)
                    taken = ready
                    calls += 1
            torch.cuda.current_stream().wait_stream(unpack_stream)
        return calls

    prefix_pipeline()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        unpack_calls = prefix_pipeline()
    torch.cuda.synchronize()
    pipe_ms = (time.perf_counter() - t0) / 3 * 1e3
    out["prefix_pipeline_sweep"] = {"ms": round(pipe_ms, 4), "th_unpack_calls": unpack_calls,
                                    "GB/s": round(sweep_bytes / (pipe_ms * 1e-3) / 1e9, 1)}

    # per-chunk pipeline recorded once into a HIP graph and replayed (what a reader that serves
    # version after version out of the same registered tensors would do): pack(c) -> unpack(c)
    # chains dealt to four parallel branches, so that one chunk's tail overlaps the next one's start
    cap_stream = torch.cuda.Stream()
    branches = [torch.cuda.Stream() for _ in range(4)]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=cap_stream):
        for br in branches:
            br.wait_stream(cap_stream)
        for j in jobs:
            for c in range(j["plan"].num_chunks):
                br = branches[c % len(branches)].cuda_stream
                th.th_pack(j["plan"], j["src_ptrs"], j["wptrs"][c:c + 1], c, 1, br)
                th.th_unpack(j["plan"], j["wptrs"][c:c + 1], c, 1, j["dst_ptrs"], br)
        for br in branches:
            cap_stream.wait_stream(br)
    graph_ms = wall_ms(graph.replay)
    del graph
    out["per_chunk_graph_sweep"] = {"ms": round(graph_ms, 4), "kernel_nodes": n_calls, "branches": 4,
                                    "GB/s": round(sweep_bytes / (graph_ms * 1e-3) / 1e9, 1)}

    # chunk ring: two wire buffers reused round-robin, unpack(c) right after pack(c), so a chunk is
    # read back while it still sits in the memory-side cache (what a co-located pipeline would see)
    out["chunk_ring_sweep"] = None
    cb_max = max(j["plan"].chunk_bytes(0) for j in jobs if j["plan"].num_chunks)
    if 2 * cb_max <= (192 << 20):
        ring = torch.empty(2 * cb_max, dtype=torch.uint8, device="cuda")
        rp = [np.array([ring.data_ptr() + k * cb_max], dtype=np.uint64) for k in range(2)]

        def ring_sweep():
            for j in jobs:
                for c in range(j["plan"].num_chunks):
                    th.th_pack(j["plan"], j["src_ptrs"], rp[c & 1], c, 1, stream)
                    th.th_unpack(j["plan"], rp[c & 1], c, 1, j["dst_ptrs"], stream)

        ring_ms = wall_ms(ring_sweep)
        del ring
        out["chunk_ring_sweep"] = {"ms": round(ring_ms, 4), "ring_chunks": 2,
                                   "GB/s": round(sweep_bytes / (ring_ms * 1e-3) / 1e9, 1)}

    # offload replica: wire chunks in pinned host memory, written / read over the host link
    if args.offload_bytes > 0:
        j = jobs[0]
        plan = j["plan"]
        nck = max(1, min(plan.num_chunks, args.offload_bytes // plan.chunk_bytes(0)))
        nbytes = sum(plan.chunk_bytes(c) for c in range(nck))
        host = torch.empty(nbytes + 16, dtype=torch.uint8, pin_memory=True)
        hptrs = dev.chunk_ptrs(plan, host)[:nck]
        res = {}
        for what, call in (("th_pack", lambda: th.th_pack(plan, j["src_ptrs"], hptrs, 0, nck, stream)),
                           ("th_unpack", lambda: th.th_unpack(plan, hptrs, 0, nck, j["dst_ptrs"], stream))):
            call()
            torch.cuda.synchronize()
            ms = time_with_events(torch, call, 3)
            res[what] = {"ms": round(ms, 3), "host_link_GB/s": round(nbytes / (ms * 1e-3) / 1e9, 2)}
        out["offload_pinned_host"] = {"chunks": nck, "bytes": nbytes, **res}
        del host
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=None,
                    help="time this workload alone (default: %s, with %s as the secondary block)" % (PRIMARY, SECONDARY))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="time only the pack + unpack sweep")
    ap.add_argument("--offload-bytes", type=int, default=1 << 30,
                    help="bytes of wire chunks the offload leg places in pinned host memory (0: skip the leg)")
    ap.add_argument("--tile-bytes", type=int, default=0, help="override the vector-path tile size")
    ap.add_argument("--no-specialize", action="store_true", help="always launch the all-paths kernel")
    ap.add_argument("--tile-bytes-any", type=int, default=0, help="override the any-alignment tile size")
    ap.add_argument("--tile-bytes-narrow", type=int, default=0, help="override the tile size of narrowing copies")
    ap.add_argument("--short-slots", type=int, default=-1,
                    help="override the largest tile (in destination slots) that runs on one wavefront")
    ap.add_argument("--tile-bytes-checksum", type=int, default=0,
                    help="override the vector-path tile size of checksum plans")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the reshard path has no cross-GPU step (every holder/reader pair is an "
              "independent plan); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    # The second workload of the default line is timed by a child process of its own, before this
    # process touches the GPU: device memory that one workload has used and freed comes back in
    # other places, and either workload then runs 2-5 % slower than it does alone.
    secondary = None
    if args.workload is None:
        import subprocess
        cmd = [sys.executable, os.path.abspath(__file__), "--workload", SECONDARY, "--steps", str(args.steps),
               "--warmup", str(args.warmup), "--no-extras", "--no-cpu-baseline"]
        child = subprocess.run(cmd, capture_output=True, text=True)
        lines = [l for l in child.stdout.splitlines() if l.startswith("{")]
        if child.returncode == 0 and lines:
            full = json.loads(lines[-1])
            secondary = {k: full[k] for k in ("value", "unit", "ms_per_step", "dtype", "config", "pct_of_hbm_peak",
                                              "plan_ms", "kernels", "roofline")}
        else:
            secondary = {"error": "exit status %d: %s" % (child.returncode, child.stderr[-400:])}

    import numpy as np
    import torch
    import synth
    import paper_2604_09107_amd as th
    from paper_2604_09107_amd import device as dev

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.tile_bytes:
        th.th_config_set(th.TH_CFG_TILE_BYTES, args.tile_bytes)
    if args.no_specialize:
        th.th_config_set(th.TH_CFG_SPECIALIZE, 0)
    if args.tile_bytes_any:
        th.th_config_set(th.TH_CFG_TILE_BYTES_ANY, args.tile_bytes_any)
    if args.tile_bytes_narrow:
        th.th_config_set(th.TH_CFG_TILE_BYTES_NARROW, args.tile_bytes_narrow)
    if args.tile_bytes_checksum:
        th.th_config_set(th.TH_CFG_TILE_BYTES_CHECKSUM, args.tile_bytes_checksum)
    if args.short_slots >= 0:
        th.th_config_set(th.TH_CFG_SHORT_TILE_SLOTS, args.short_slots)
    # one throw-away plan first: the process's first HIP call loads the library's code object
    # (~0.1 s, once per process), which is not part of creating a plan
    w0 = synth.workload("cfg1_tiny_tp2_to_tp1")
    th.th_plan_create(w0["model"], w0["holders"][0], w0["reader"], w0["chunk_bytes"]).destroy()
    mods = (np, torch, synth, th, dev)

    name = args.workload or PRIMARY
    head, rest = measure(args, name, not args.no_extras, not args.no_cpu_baseline, mods)
    out = {"metric": "reshard pack+unpack effective HBM GB/s", "value": head.pop("value"), "unit": head.pop("unit"),
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head.pop("ms_per_step"),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head.pop("dtype"),
           "data": "synthetic"}
    out.update(head)
    out.update(rest)
    if secondary is not None:
        out["secondary"] = secondary
    print(json.dumps(out))


if __name__ == "__main__":
    main()
