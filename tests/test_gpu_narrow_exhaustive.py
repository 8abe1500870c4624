"""Every fp32 bit pattern through the kernels' fp32 -> bf16 narrowing, against the oracle's
definition of round-to-nearest-even (subnormals kept, overflow to infinity, NaN quieted with its
sign and top payload bits).  The kernels narrow with the hardware pair conversion on their main
paths and with an integer formula at run edges; this is the proof that both agree with the
definition on all 2^32 inputs, on each of the three copy paths:

  vector  th_pack, 16-byte aligned source and destination (one 16-byte load -> one 8-byte store);
  dense   th_pack, element-aligned source and destination (slots gathered with unaligned loads);
  any     th_unpack of an fp32 wire into a strided bf16 destination (narrowing at unpack).
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import synth
import paper_2604_09107_amd as th
from paper_2604_09107_amd import device as dev
from oracle import rne

pytestmark = pytest.mark.gpu

SLICE = 1 << 28
ROWS = 1 << 14          # the strided case sees a slice as ROWS x (SLICE / ROWS)
PAD = 24                # its destination rows lie PAD elements further apart than they are long


def one_segment(n, src_off, dst_off, nrows, row_len, src_stride, dst_stride):
    seg = np.zeros(1, dtype=th.binding.SEGMENT_NP)
    seg["src_elem_off"], seg["dst_elem_off"] = src_off, dst_off
    seg["nrows"], seg["row_len"] = nrows, row_len
    seg["src_row_stride"], seg["dst_row_stride"] = src_stride, dst_stride
    seg["src_dtype"], seg["dst_dtype"] = th.TH_F32, th.TH_BF16
    return seg


def oracle_narrow(u, pool):
    parts = np.array_split(u, 64)
    return np.concatenate(list(pool.map(rne.narrow, parts)))


def first_difference(got, want, u, what):
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, "%s: input %08x -> %04x, oracle %04x (%d of %d differ)" % (
        what, u[bad[0]], got[bad[0]], want[bad[0]], bad.size, len(u))


def test_all_fp32_bit_patterns_on_every_path():
    n, cols = SLICE, SLICE // ROWS
    stream = dev.current_stream()
    chunk = 64 << 20
    vec = th.th_plan_create_from_segments(one_segment(n, 0, 0, 1, n, n, n), [n + 4], [n + 8], chunk,
                                          th.TH_FLAG_PTRS_ALIGNED16)
    dense = th.th_plan_create_from_segments(one_segment(n, 1, 0, 1, n, n, n), [n + 4], [n + 8], chunk)
    strided = th.th_plan_create_from_segments(one_segment(n, 0, 3, ROWS, cols, cols, cols + PAD), [n + 4],
                                              [ROWS * (cols + PAD) + 8], chunk, th.TH_FLAG_NARROW_AT_UNPACK)
    assert [vec.tile(0, 0).kind, dense.tile(0, 0).kind, strided.tile(1, 0).kind] == [0, 2, 1]
    src = torch.empty(n + 4, dtype=torch.float32, device="cuda")
    wire_v, wp_v = dev.alloc_wire(vec)
    wire_d, wp_d = dev.alloc_wire(dense)
    wire_s, wp_s = dev.alloc_wire(strided)
    out_s = torch.empty(ROWS * (cols + PAD) + 8, dtype=torch.bfloat16, device="cuda")
    with ThreadPoolExecutor(16) as pool:
        for s in range((1 << 32) // n):
            print("[narrow] slice %d of %d" % (s, (1 << 32) // n), flush=True)
            u = np.arange(s * n, (s + 1) * n, dtype=np.uint64).astype(np.uint32)
            dev_bits = synth.from_bits(u, "cuda")
            src[:n] = dev_bits                      # aligned copy for the vector and strided cases
            th.th_pack(vec, [src.data_ptr()], wp_v, 0, vec.num_chunks, stream)
            th.th_pack(strided, [src.data_ptr()], wp_s, 0, strided.num_chunks, stream)
            out_s.view(torch.int16).fill_(0x7FA5)
            th.th_unpack(strided, wp_s, 0, strided.num_chunks, [out_s.data_ptr()], stream)
            torch.cuda.synchronize()
            src[1:n + 1] = dev_bits                 # the same bits one element further: 4-byte aligned only
            th.th_pack(dense, [src.data_ptr()], wp_d, 0, dense.num_chunks, stream)
            torch.cuda.synchronize()
            want = oracle_narrow(u, pool)
            first_difference(synth.to_bits(wire_v[:2 * n].view(torch.bfloat16)), want, u, "vector path")
            first_difference(synth.to_bits(wire_d[:2 * n].view(torch.bfloat16)), want, u, "dense path")
            got = synth.to_bits(out_s)[3:3 + ROWS * (cols + PAD)].reshape(ROWS, cols + PAD)
            first_difference(got[:, :cols].reshape(-1), want, u, "strided path")
            assert np.all(got[:, cols:] == 0x7FA5)               # between the rows nothing was written
    for p in (vec, dense, strided):
        p.destroy()
