"""Byte offsets beyond 4 GiB inside one tensor: explicit segments whose rows start past the 2^32-byte
mark of a source and of a destination tensor of 4.8 GB each, on the vector path (aligned single row,
aligned strided rows), the dense path (unaligned single row, strided rows gathered onto the wire) and
the strided-destination path, bf16 -> bf16 and fp32 -> bf16, through th_pack / th_unpack and through
th_reshard.  Wire bytes and every destination element (sentinels included) against the segment oracle.
"""
import numpy as np
import pytest
import torch

import synth
import paper_2604_09107_amd as th
from paper_2604_09107_amd import device as dev
from oracle import segments
from helpers import LARGE_DST_LEN as DST_LEN, large_offset_segments, library_segments

pytestmark = pytest.mark.gpu

SENT8 = 0xA5
SENT16 = 0x7777


def hashed_bits(n, torch_dtype, salt):
    """n elements of arbitrary bit patterns, made on the device block by block (a multiplicative hash
    of the element index: every pattern class shows up, NaNs and subnormals included)."""
    out = torch.empty(n, dtype=torch_dtype, device="cuda")
    bits = out.view(torch.int16 if torch_dtype == torch.bfloat16 else torch.int32)
    block = 1 << 26
    for lo in range(0, n, block):
        hi = min(n, lo + block)
        i = torch.arange(lo, hi, dtype=torch.int64, device="cuda")
        h = (i * 2654435761 + salt) ^ (i >> 13)
        if torch_dtype == torch.bfloat16:
            bits[lo:hi] = ((h >> 5) & 0xFFFF).to(torch.int32).to(torch.int16)
        else:
            bits[lo:hi] = (h & 0xFFFFFFFF).to(torch.int32)
    return out


@pytest.mark.parametrize("src_dt", ["bf16", "f32"])
def test_rows_beyond_four_gib_inside_one_tensor(src_dt):
    o, src_len = large_offset_segments(src_dt)
    src_dev = hashed_bits(src_len, torch.float32 if src_dt == "f32" else torch.bfloat16, 12345)
    print("[large] source on the host", flush=True)
    src = synth.to_bits(src_dev)
    wire = segments.pack(o, [src], src_dt, "bf16")
    del src
    want = np.full(DST_LEN, SENT16, dtype=np.uint16)
    segments.unpack(o, wire, [want], "bf16")

    segs = library_segments(th, o, src_dt, "bf16")
    plan = th.th_plan_create_from_segments(segs, [src_len], [DST_LEN], 1 << 20, th.TH_FLAG_PTRS_ALIGNED16)
    kinds = {plan.tile(side, i).kind for side in (0, 1) for i in range(plan.num_tiles(side))}
    assert kinds == {0, 1, 2}, "vector, strided and dense tiles are all in the plan: %s" % kinds
    stream = dev.current_stream()
    wire_dev, wptrs = dev.alloc_wire(plan, fill_byte=SENT8)
    dst_dev = torch.empty(DST_LEN, dtype=torch.bfloat16, device="cuda")
    for what in ("pack + unpack", "reshard"):
        print("[large] %s" % what, flush=True)
        dst_dev.view(torch.int16).fill_(SENT16)
        if what == "reshard":
            th.th_reshard(plan, [src_dev.data_ptr()], [dst_dev.data_ptr()], stream)
        else:
            th.th_pack(plan, [src_dev.data_ptr()], wptrs, 0, plan.num_chunks, stream)
            th.th_unpack(plan, wptrs, 0, plan.num_chunks, [dst_dev.data_ptr()], stream)
        torch.cuda.synchronize()
        if what != "reshard":
            assert np.array_equal(wire_dev.cpu().numpy()[:plan.wire_bytes], wire)
        got = synth.to_bits(dst_dev)
        bad = np.nonzero(got != want)[0]
        assert bad.size == 0, "%s: first difference at element %d (%d differ)" % (what, bad[0], bad.size)
        del got
    plan.destroy()
