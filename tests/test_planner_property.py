"""Property test of the host planner against the oracle over random model shapes, layout pairs,
chunk sizes and tile sizes (CPU only: the manifest is run by the numpy test executor)."""
import os

import numpy as np
from hypothesis import HealthCheck, given, settings, strategies as st

import synth
import paper_2604_09107_amd as th
from oracle import checksum, reshard
from helpers import exec_tiles, flat_u8, holder_tensors_cpu, tile_checksums, tile_sizes

HOST = th.TH_FLAG_HOST_ONLY
# The same 300 examples on every run, so that the suite is a fixed gate; TH_TEST_EXPLORE=<n> draws n new ones.
FIXED_EXAMPLES = not os.environ.get("TH_TEST_EXPLORE")
N_EXAMPLES = max(300, int(os.environ.get("TH_TEST_EXPLORE") or 0))


@st.composite
def cases(draw):
    nkv = draw(st.sampled_from([1, 2, 4]))
    per = draw(st.sampled_from([1, 2, 4]))
    hd = draw(st.sampled_from([2, 4, 8]))
    nq = nkv * per
    hidden = draw(st.sampled_from([8, 16, 24, 40]))
    ffn = draw(st.sampled_from([8, 16, 24]))
    vocab = draw(st.sampled_from([16, 24, 40]))
    moe = draw(st.booleans())
    model = dict(kind="moe" if moe else "dense", n_layers=draw(st.integers(1, 2)), hidden=hidden,
                 n_q_heads=nq, n_kv_heads=nkv, head_dim=hd, ffn=0 if moe else ffn, vocab=vocab,
                 tied_embeddings=draw(st.integers(0, 1)), n_experts=4 if moe else 0,
                 n_shared_experts=draw(st.integers(0, 1)) if moe else 0, expert_ffn=ffn if moe else 0,
                 weight_dtype=draw(st.sampled_from(["bf16", "f32"])), norm_dtype="f32")

    def tp_choices():
        out = []
        for t in (1, 2, 4, 8):
            ok_kv = nkv % t == 0 or (t % nkv == 0 and nq % t == 0)
            if ok_kv and nq % t == 0 and hidden % t == 0 and ffn % t == 0 and (nq * hd) % t == 0:
                out.append(t)
        return out

    tps = tp_choices()
    S, D = draw(st.sampled_from(tps)), draw(st.sampled_from(tps))

    def lay(T, side):
        pad = draw(st.sampled_from([0, 48, 64]))
        if pad and (pad < vocab or pad % T):
            pad = 0
        if not pad and vocab % T:
            pad = (vocab + T * 8 - 1) // (T * 8) * (T * 8)
        ep = draw(st.sampled_from([1, 2, 4])) if moe else 1
        return synth.layout(T, draw(st.integers(0, T - 1)), ep_size=ep, ep_rank=draw(st.integers(0, ep - 1)),
                            experts_stacked=draw(st.integers(0, 1)) if moe else 0,
                            f32_store=draw(st.sampled_from(["f32", "bf16"])) if side else "f32",
                            qkv_grouped=draw(st.integers(0, 1)), padded_vocab=pad)

    src, dst = lay(S, 0), lay(D, 1)
    if model["weight_dtype"] == "f32" and dst["f32_store"] == "bf16":
        pass  # whole model narrowed
    chunk = 16 * draw(st.integers(1, 64))
    tile = draw(st.sampled_from([4096, 8192]))
    narrow_at = draw(st.sampled_from(["pack", "unpack"]))
    return model, src, dst, chunk, tile, narrow_at


@settings(max_examples=N_EXAMPLES, deadline=None, derandomize=FIXED_EXAMPLES,
          suppress_health_check=[HealthCheck.too_slow, HealthCheck.data_too_large])
@given(cases())
def test_manifest_matches_oracle_on_random_shapes(case):
    model, src, dst, chunk, tile, narrow_at = case
    tensors = holder_tensors_cpu(model, src, 1, pattern=True)
    wire = reshard.pack(model, src, dst, tensors, narrow_at=narrow_at)
    want = reshard.empty_tensors(model, dst, fill=0x5A5A)
    reshard.unpack(model, src, dst, wire, want, narrow_at=narrow_at)
    with tile_sizes(tile):
        plan = th.th_plan_create(model, src, dst, chunk,
                                 HOST | (th.TH_FLAG_NARROW_AT_UNPACK if narrow_at == "unpack" else 0))
    try:
        assert plan.wire_bytes == len(wire)
        want_chunks = reshard.chunks(wire, chunk) if len(wire) else []
        assert plan.num_chunks == len(want_chunks)
        chunks = [np.full(len(c), 0xEE, dtype=np.uint8) for c in want_chunks]
        exec_tiles(plan, 0, flat_u8(tensors), chunks)
        for g, x in zip(chunks, want_chunks):
            assert np.array_equal(g, x)
        got = reshard.empty_tensors(model, dst, fill=0x5A5A)
        exec_tiles(plan, 1, chunks, flat_u8(got))
        direct = reshard.empty_tensors(model, dst, fill=0x5A5A)
        exec_tiles(plan, 2, flat_u8(tensors), flat_u8(direct))
        for g, d, x in zip(got, direct, want):
            assert np.array_equal(g, x) and np.array_equal(d, x)
        if len(wire):
            cs = checksum.model_checksums(model, src, dst, wire, len(tensors), narrow_at=narrow_at)
            for side in (0, 1):
                assert np.array_equal(tile_checksums(plan, side, want_chunks, len(tensors)), cs)
    finally:
        plan.destroy()
