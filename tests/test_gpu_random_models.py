"""Random model shapes and layout pairs on the GPU against the layout oracle: the same strategy as
the CPU property test of the planner (tiny dense / MoE shapes, any pair of TP / EP sizes that
divides, grouped QKV, padded vocabulary, stacked experts, narrowing at pack or at unpack), here run
through th_pack / th_unpack / th_reshard and the fused checksums instead of the CPU test executor."""
import numpy as np
import pytest
import torch
from hypothesis import HealthCheck, given, settings

import synth
import paper_2604_09107_amd as th
from paper_2604_09107_amd import device as dev
from oracle import checksum, layouts, reshard
from helpers import holder_tensors_cpu, tile_sizes
from test_planner_property import FIXED_EXAMPLES, N_EXAMPLES, cases

pytestmark = pytest.mark.gpu

SENT16 = 0x5A5A


@settings(max_examples=N_EXAMPLES, deadline=None, derandomize=FIXED_EXAMPLES,
          suppress_health_check=[HealthCheck.too_slow, HealthCheck.data_too_large])
@given(cases())
def test_random_model_plans_bit_exact(case):
    model, src, dst, chunk, tile, narrow_at = case
    tensors = holder_tensors_cpu(model, src, 3, pattern=False)
    wire = reshard.pack(model, src, dst, tensors, narrow_at=narrow_at)
    want = reshard.empty_tensors(model, dst, fill=SENT16)
    for t, wnt in zip(layouts.registered_tensors(model, dst), want):
        if wnt.dtype == np.uint32:
            wnt[...] = SENT16 * 0x10001
    reshard.unpack(model, src, dst, wire, want, narrow_at=narrow_at)
    flags = th.TH_FLAG_CHECKSUM | (th.TH_FLAG_NARROW_AT_UNPACK if narrow_at == "unpack" else 0)
    with tile_sizes(tile):
        plan = th.th_plan_create(model, src, dst, chunk, flags)
    try:
        assert plan.wire_bytes == len(wire)
        src_dev = [synth.from_bits(np.ascontiguousarray(t).reshape(-1), "cuda") for t in tensors]
        dst_dev = dev.alloc_tensors(plan, 1, fill_bits=SENT16)
        dir_dev = dev.alloc_tensors(plan, 1, fill_bits=SENT16)
        wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=0xEE)
        ps = torch.zeros(2 * len(tensors), dtype=torch.int64, device="cuda")
        us = torch.zeros_like(ps)
        stream = dev.current_stream()
        n = plan.num_chunks
        # ranges of 1..12 chunks: short ones carry their wire pointers in the kernel arguments
        c = 0
        k = 1
        while c < n:
            m = min(k, n - c)
            th.th_pack_checksum(plan, dev.ptrs(src_dev), wptrs[c:c + m], c, m, ps.data_ptr(), stream)
            th.th_unpack_checksum(plan, wptrs[c:c + m], c, m, dev.ptrs(dst_dev), us.data_ptr(), stream)
            c += m
            k = k % 12 + 1
        th.th_reshard(plan, dev.ptrs(src_dev), dev.ptrs(dir_dev), stream)
        torch.cuda.synchronize()
        assert np.array_equal(wire_dev.cpu().numpy()[:plan.wire_bytes], wire)
        for g, d, x in zip(dst_dev, dir_dev, want):
            assert np.array_equal(synth.to_bits(g), x.reshape(-1))
            assert np.array_equal(synth.to_bits(d), x.reshape(-1))
        if len(wire):
            cs = checksum.model_checksums(model, src, dst, wire, len(tensors), narrow_at=narrow_at)
            assert np.array_equal(ps.cpu().numpy().view(np.uint64).reshape(-1, 2), cs)
            assert np.array_equal(us.cpu().numpy().view(np.uint64).reshape(-1, 2), cs)
    finally:
        plan.destroy()
