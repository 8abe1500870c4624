"""Pins for the layout / reshard oracle.  The paper prints no worked example
for this path, so the pins are mathematical: agreement with numpy.split,
exactly-once coverage, round trips, byte conservation, brute force with a
closed form on tiny shapes, closed-form stream lengths."""
import itertools

import numpy as np
import pytest

import synth
from oracle import layouts, reshard

L = synth.layout


def tiny_model(**kw):
    m = dict(kind="dense", n_layers=1, hidden=8, n_q_heads=4, n_kv_heads=2, head_dim=2, ffn=12,
             vocab=8, tied_embeddings=0, n_experts=0, n_shared_experts=0, expert_ffn=0,
             weight_dtype="f32", norm_dtype="f32")
    m.update(kw)
    return m


def tiny_moe(**kw):
    m = tiny_model(kind="moe", ffn=0, n_experts=8, n_shared_experts=1, expert_ffn=4, n_kv_heads=4)
    m.update(kw)
    return m


def full_weights(model, seed=0):
    """One unique 32-bit id per element of every logical weight."""
    out = []
    for i, lt in enumerate(layouts.logical_tensors(model)):
        ids = (np.uint32(i) << np.uint32(20)) + np.arange(lt["rows"] * lt["cols"], dtype=np.uint32)
        out.append(ids.reshape(lt["rows"], lt["cols"]))
    return out


def shard_of(model, lay, full):
    """Registered tensors of a rank cut from the full weights with the oracle's index vectors
    (padding rows of a padded vocabulary are filled with a marker)."""
    lts = layouts.logical_tensors(model)
    out = []
    for t in layouts.registered_tensors(model, lay):
        parts = []
        for li, _ in t["parts"]:
            rows, cols = layouts.shard_index(model, lts[li], lay)
            parts.append(full[li][np.ix_(rows, cols)])
        a = np.concatenate(parts, axis=0)
        if a.shape[0] < t["rows"]:
            a = np.concatenate([a, np.full((t["rows"] - a.shape[0], a.shape[1]), 0xDEAD, dtype=a.dtype)], axis=0)
        out.append(a)
        assert out[-1].shape == (t["rows"], t["cols"])
    return out


# ---- (vi) numpy.split reference for dense models --------------------------------------

def split_reference(model, name, W, T, r):
    """Independent statement of the conventions with numpy.split / concatenate."""
    hd, nq, nkv = model["head_dim"], model["n_q_heads"], model["n_kv_heads"]
    leaf = name.split(".")[-1]
    if leaf in ("embed_tokens", "lm_head"):
        return np.split(W, T, axis=0)[r]
    if leaf in ("o_proj", "down_proj", "w2"):
        return np.split(W, T, axis=1)[r]
    if leaf == "qkv_proj":
        q, k, v = np.split(W, [nq * hd, (nq + nkv) * hd], axis=0)
        return np.concatenate([np.split(q, T, 0)[r], np.split(k, T, 0)[r], np.split(v, T, 0)[r]], 0)
    if leaf in ("gate_up_proj", "w13"):
        g, u = np.split(W, 2, axis=0)
        return np.concatenate([np.split(g, T, 0)[r], np.split(u, T, 0)[r]], 0)
    return W  # norms, router


@pytest.mark.parametrize("T", [1, 2])
def test_shards_match_numpy_split_tiny(T):
    model = tiny_model()
    full = full_weights(model)
    lts = layouts.logical_tensors(model)
    for r in range(T):
        regs = layouts.registered_tensors(model, L(T, r))
        got = shard_of(model, L(T, r), full)
        assert len(regs) == len(lts)
        for t, g, lt, W in zip(regs, got, lts, full):
            assert t["name"] == lt["name"]
            assert np.array_equal(g, split_reference(model, lt["name"], W, T, r)), lt["name"]


@pytest.mark.parametrize("T", [1, 2, 4])
def test_shards_match_numpy_split_small_dense(T):
    model = synth.MODELS["dense_small"]
    lts = layouts.logical_tensors(model)
    rng = np.random.default_rng(3)
    for li in [0, 2, 3, 5, 6, len(lts) - 1]:
        lt = lts[li]
        W = rng.integers(0, 1 << 16, size=(lt["rows"], lt["cols"]), dtype=np.uint16)
        for r in range(T):
            rows, cols = layouts.shard_index(model, lt, L(T, r))
            assert np.array_equal(W[np.ix_(rows, cols)], split_reference(model, lt["name"], W, T, r))


@pytest.mark.parametrize("T", [1, 2, 4])
def test_grouped_qkv_matches_numpy_reference(T):
    """Trainer-style fused QKV: per KV head of the rank, its query heads, then its K, then its V."""
    model = synth.MODELS["dense_small"]  # 8 query heads, 4 KV heads, head_dim 64
    hd, nq, nkv = model["head_dim"], model["n_q_heads"], model["n_kv_heads"]
    qkv = [t for t in layouts.logical_tensors(model) if t["part"] == "qkv"][0]
    W = np.random.default_rng(7).integers(0, 1 << 16, size=(qkv["rows"], qkv["cols"]), dtype=np.uint16)
    q, k, v = np.split(W, [nq * hd, (nq + nkv) * hd], axis=0)
    q_groups = np.split(q, nkv, axis=0)      # query heads of KV head g
    k_heads, v_heads = np.split(k, nkv, axis=0), np.split(v, nkv, axis=0)
    for r in range(T):
        mine = range(r * nkv // T, (r + 1) * nkv // T)
        want = np.concatenate([x for g in mine for x in (q_groups[g], k_heads[g], v_heads[g])], axis=0)
        rows, cols = layouts.shard_index(model, qkv, L(T, r, qkv_grouped=1))
        assert np.array_equal(W[np.ix_(rows, cols)], want)
        # same set of rows as the concatenated convention, different order
        rows_c, _ = layouts.shard_index(model, qkv, L(T, r))
        assert sorted(rows) == sorted(rows_c) and (T == nkv or not np.array_equal(rows, rows_c))


@pytest.mark.parametrize("T,padded", [(4, 4096), (2, 4096), (8, 4096), (1, 4000)])
def test_padded_vocabulary_matches_numpy_pad_then_split(T, padded):
    model = synth.MODELS["dense_small_v4000"]
    lts = layouts.logical_tensors(model)
    rng = np.random.default_rng(8)
    for li in (0, len(lts) - 1):  # embed_tokens, lm_head
        lt = lts[li]
        W = rng.integers(1, 1 << 16, size=(lt["rows"], lt["cols"]), dtype=np.uint16)
        Wp = np.pad(W, ((0, padded - lt["rows"]), (0, 0)))  # zero rows = padding
        for r in range(T):
            lay = L(T, r, padded_vocab=padded)
            want = np.split(Wp, T, axis=0)[r]
            rows, cols = layouts.shard_index(model, lt, lay)
            assert layouts.storage_rows(model, lt, lay) == want.shape[0] == padded // T
            n_real = len(rows)
            assert np.array_equal(W[np.ix_(rows, cols)], want[:n_real])
            assert not want[n_real:].any()  # what is left of the rank's tensor is padding
    with pytest.raises(ValueError):
        layouts.shard_index(model, lts[0], L(2, 0, padded_vocab=3000))
    with pytest.raises(ValueError):
        layouts.shard_index(model, lts[0], L(3, 0, padded_vocab=4096))


def test_trainer_to_rollout_and_back_is_the_identity():
    """Grouped QKV + padded vocabulary TP=4 -> plain TP=2 -> grouped + padded TP=4: every rank gets
    its tensors back, padding rows untouched."""
    model = synth.MODELS["dense_small_v4000"]
    full = full_weights(dict(model, weight_dtype="f32"))
    model = dict(model, weight_dtype="f32")
    trainer = [L(4, r, qkv_grouped=1, padded_vocab=4096) for r in range(4)]
    rollout = [L(2, r) for r in range(2)]
    t_shards = [shard_of(model, lay, full) for lay in trainer]
    r_shards = []
    for d in rollout:
        out = reshard.empty_tensors(model, d, fill=0)
        counts = [np.zeros(t.shape, dtype=np.int32) for t in out]
        for lay, ts in zip(trainer, t_shards):
            reshard.unpack(model, lay, d, reshard.pack(model, lay, d, ts), out, counts)
        assert all(np.all(c == 1) for c in counts)
        for o, wnt in zip(out, shard_of(model, d, full)):
            assert np.array_equal(o, wnt)
        r_shards.append(out)
    for lay, ts in zip(trainer, t_shards):
        back = reshard.empty_tensors(model, lay, fill=0xDEAD)
        for d, rs in zip(rollout, r_shards):
            reshard.unpack(model, d, lay, reshard.pack(model, d, lay, rs), back)
        for b, t in zip(back, ts):
            assert np.array_equal(b, t)


def test_gqa_grouping_kept_on_one_rank():
    model = synth.MODELS["dense8b"]
    hd, nq, nkv = model["head_dim"], model["n_q_heads"], model["n_kv_heads"]
    qkv = [t for t in layouts.logical_tensors(model) if t["part"] == "qkv"][0]
    for T in (2, 4, 8):
        for r in range(T):
            rows, _ = layouts.shard_index(model, qkv, L(T, r))
            q_heads = sorted(set(rows[rows < nq * hd] // hd))
            k_heads = sorted(set((rows[(rows >= nq * hd) & (rows < (nq + nkv) * hd)] - nq * hd) // hd))
            v_heads = sorted(set((rows[rows >= (nq + nkv) * hd] - (nq + nkv) * hd) // hd))
            assert k_heads == v_heads
            assert sorted(set(h // (nq // nkv) for h in q_heads)) == k_heads


def test_indivisible_split_is_an_error():
    model = tiny_model(vocab=9)
    emb = layouts.logical_tensors(model)[0]
    with pytest.raises(ValueError):
        layouts.shard_index(model, emb, L(2, 0))
    with pytest.raises(ValueError):  # 3 ranks over 2 KV heads / 4 query heads
        layouts.shard_index(tiny_model(), layouts.logical_tensors(tiny_model())[2], L(3, 0))


@pytest.mark.parametrize("T", [8, 16])
def test_replicated_kv_heads_match_numpy_reference(T):
    """More ranks than KV heads: every rank keeps its query heads and a copy of their KV head."""
    model = synth.MODELS["dense_small_kv"]  # 16 query heads, 4 KV heads
    hd, nq, nkv = model["head_dim"], model["n_q_heads"], model["n_kv_heads"]
    qkv = [t for t in layouts.logical_tensors(model) if t["part"] == "qkv"][0]
    W = np.random.default_rng(9).integers(0, 1 << 16, size=(qkv["rows"], qkv["cols"]), dtype=np.uint16)
    q, k, v = np.split(W, [nq * hd, (nq + nkv) * hd], axis=0)
    for r in range(T):
        g = r * nkv // T
        want = np.concatenate([np.split(q, T, 0)[r], np.split(k, nkv, 0)[g], np.split(v, nkv, 0)[g]], 0)
        rows, cols = layouts.shard_index(model, qkv, L(T, r))
        assert np.array_equal(W[np.ix_(rows, cols)], want)
        # the rank's query heads all use the KV head it keeps
        q_heads = set(rows[rows < nq * hd] // hd)
        assert {h // (nq // nkv) for h in q_heads} == {g}


@pytest.mark.parametrize("S,D", [(8, 2), (8, 4), (8, 16), (16, 8), (2, 8), (8, 8), (16, 1)])
def test_replicated_kv_every_reader_element_written_exactly_once(S, D):
    model = dict(synth.MODELS["dense_small_kv"], n_layers=1, weight_dtype="f32")
    full = full_weights(model)
    for d in range(D):
        dst, out, counts, payload = run_reader(model, S, D, d, full)
        want = shard_of(model, dst, full)
        for o, wnt, c in zip(out, want, counts):
            assert np.all(c == 1)
            assert np.array_equal(o, wnt)
        assert payload == sum(o.size * 4 for o in out)
    # the copies of a KV head are pulled evenly: with S = 16 holders, D = 8 readers the two readers
    # that share KV head 0 use different holder copies
    if (S, D) == (16, 8):
        qkv = [t for t in layouts.logical_tensors(model) if t["part"] == "qkv"][0]
        senders = {d: [s for s in range(S) if (layouts.row_supply_mask(model, qkv, L(S, s), L(D, d))
                                                & np.isin(layouts.shard_index(model, qkv, L(S, s))[0],
                                                          layouts.shard_index(model, qkv, L(D, d))[0])
                                                & (layouts.shard_index(model, qkv, L(S, s))[0] >= 16 * 32)).any()]
                   for d in (0, 1)}
        assert len(senders[0]) == 1 and len(senders[1]) == 1 and senders[0] != senders[1]


def test_registration_order_and_names():
    names = [t["name"] for t in layouts.registered_tensors(tiny_model(n_layers=2), L(1, 0))]
    assert names[:6] == ["embed_tokens", "layers.0.input_norm", "layers.0.qkv_proj", "layers.0.o_proj",
                         "layers.0.post_attn_norm", "layers.0.gate_up_proj"]
    assert names[-2:] == ["final_norm", "lm_head"]
    tied = [t["name"] for t in layouts.registered_tensors(tiny_model(tied_embeddings=1), L(1, 0))]
    assert tied[-1] == "final_norm"
    moe = [t["name"] for t in layouts.registered_tensors(tiny_moe(), L(1, 0, ep_size=4, ep_rank=1))]
    assert moe[5:11] == ["layers.0.router", "layers.0.experts.2.w13", "layers.0.experts.2.w2",
                         "layers.0.experts.3.w13", "layers.0.experts.3.w2", "layers.0.shared.0.w13"]
    st = layouts.registered_tensors(tiny_moe(), L(2, 0, experts_stacked=1))
    by = {t["name"]: t for t in st}
    assert by["layers.0.experts.w13"]["rows"] == 8 * 2 * 2 and by["layers.0.experts.w13"]["cols"] == 8
    assert by["layers.0.experts.w2"]["rows"] == 8 * 8 and by["layers.0.experts.w2"]["cols"] == 2
    assert [p[1] for p in by["layers.0.experts.w2"]["parts"]] == [8 * e for e in range(8)]


# ---- (iii) union over reader ranks = full tensor, write count 1 --------------------------

PAIRS = [(1, 1), (1, 2), (2, 1), (2, 2), (2, 4), (4, 2), (1, 4), (4, 1)]


def run_reader(model, S, D, d, full, src_extra=None, dst_extra=None):
    """Reader rank d of D pulls from every holder rank of S through pack/unpack."""
    dst = L(D, d, **(dst_extra or {}))
    out = reshard.empty_tensors(model, dst, fill=0xFFFF)
    counts = [np.zeros(t.shape, dtype=np.int32) for t in out]
    payload = 0
    for s in range(S):
        src = L(S, s, **(src_extra or {}))
        wire = reshard.pack(model, src, dst, shard_of(model, src, full))
        assert len(wire) == reshard.wire_bytes(model, src, dst)
        reshard.unpack(model, src, dst, wire, out, counts)
        payload += sum(len(it["src_r"]) * len(it["src_c"]) * 4 for it in reshard.plan_items(model, src, dst))
    return dst, out, counts, payload


@pytest.mark.parametrize("S,D", PAIRS)
def test_every_reader_element_written_exactly_once_and_correct(S, D):
    model = tiny_model(n_kv_heads=4, n_q_heads=4, vocab=8)
    full = full_weights(model)
    total = 0
    for d in range(D):
        dst, out, counts, payload = run_reader(model, S, D, d, full)
        want = shard_of(model, dst, full)
        for o, w, c in zip(out, want, counts):
            assert np.all(c == 1)
            assert np.array_equal(o, w)
        # byte conservation: what the holders send == what the reader stores
        assert payload == sum(o.size * 4 for o in out)
        total += sum(o.size for o, t in zip(out, layouts.registered_tensors(model, dst))
                     if layouts.logical_tensors(model)[t["parts"][0][0]]["part"] != "repl")
    lts = layouts.logical_tensors(model)
    assert total == sum(lt["rows"] * lt["cols"] for lt in lts if lt["part"] != "repl")


@pytest.mark.parametrize("k", [2, 4, 8])
def test_tp1_to_tpk_to_tp1_round_trip(k):
    model = tiny_model(n_q_heads=8, n_kv_heads=8, vocab=16, ffn=16, hidden=16)
    full = full_weights(model)
    mids = []
    for d in range(k):
        _, out, counts, _ = run_reader(model, 1, k, d, full)
        mids.append(out)
    # now the k shards are the holders and a TP=1 reader pulls from all of them
    dst = L(1, 0)
    back = reshard.empty_tensors(model, dst, fill=0)
    counts = [np.zeros(t.shape, dtype=np.int32) for t in back]
    for s in range(k):
        wire = reshard.pack(model, L(k, s), dst, mids[s])
        reshard.unpack(model, L(k, s), dst, wire, back, counts)
    for b, f, c in zip(back, full, counts):
        assert np.all(c == 1)
        assert np.array_equal(b, f)


@pytest.mark.parametrize("T", [1, 2, 4])
def test_same_layout_pack_unpack_is_identity_and_wire_is_the_shard(T):
    model = tiny_model(n_kv_heads=4)
    full = full_weights(model)
    for r in range(T):
        lay = L(T, r)
        mine = shard_of(model, lay, full)
        wire = reshard.pack(model, lay, lay, mine)
        # same layout: the stream is the registered tensors back to back, 16-byte aligned
        expect = bytearray()
        for t in mine:
            expect += b"\0" * (-len(expect) % 16)
            expect += t.tobytes()
        assert wire.tobytes() == bytes(expect)
        out = reshard.empty_tensors(model, lay, fill=7)
        reshard.unpack(model, lay, lay, wire, out)
        for o, m in zip(out, mine):
            assert np.array_equal(o, m)


def test_contiguous_source_case_wire_is_concatenated_shards():
    """TP=4 holders 2,3 -> TP=2 reader 1: the reader needs the holders' tensors whole."""
    model = synth.MODELS["dense_small"]
    rng = np.random.default_rng(5)
    dst = L(2, 1, f32_store="bf16")
    for s in (2, 3):
        src = L(4, s)
        regs = layouts.registered_tensors(model, src)
        lts = layouts.logical_tensors(model)
        tensors = [rng.integers(0, 1 << 16, size=(t["rows"], t["cols"])).astype(reshard.NPBITS[t["dtype"]])
                   for t in regs]
        for t, a in zip(regs, tensors):
            if t["dtype"] == "f32":
                a[...] = 0x3F800000
        wire = reshard.pack(model, src, dst, tensors)
        expect = bytearray()
        for t, a in zip(regs, tensors):
            if lts[t["parts"][0][0]]["part"] == "repl":
                if s != 2:
                    continue  # only the primary holder sends replicated tensors
                a = np.full(a.shape, 0x3F80, dtype=np.uint16)  # fp32 one narrowed to bf16
            expect += b"\0" * (-len(expect) % 16)
            expect += a.tobytes()
        assert wire.tobytes() == bytes(expect)


# ---- (v) brute force with a closed form -----------------------------------------------------

def closed_form_global(model, leaf, T, r, i, j, R, C):
    """Global (I, J) of local element (i, j) of rank r, written per convention with plain arithmetic."""
    hd, nq, nkv = model["head_dim"], model["n_q_heads"], model["n_kv_heads"]
    if leaf in ("embed_tokens", "lm_head"):
        return r * (R // T) + i, j
    if leaf in ("o_proj", "down_proj", "w2"):
        return i, r * (C // T) + j
    if leaf == "qkv_proj":
        q, kv = nq // T * hd, nkv // T * hd
        if i < q:
            return r * q + i, j
        if i < q + kv:
            return nq * hd + r * kv + (i - q), j
        return (nq + nkv) * hd + r * kv + (i - q - kv), j
    if leaf in ("gate_up_proj", "w13"):
        F = R // 2
        f = F // T
        return (r * f + i, j) if i < f else (F + r * f + (i - f), j)
    return i, j


@pytest.mark.parametrize("S,D", PAIRS)
def test_brute_force_closed_form(S, D):
    model = tiny_model(n_kv_heads=4, n_q_heads=4)
    full = full_weights(model)
    lts = layouts.logical_tensors(model)
    for d in range(D):
        dst, out, _, _ = run_reader(model, S, D, d, full)
        for t, o in zip(layouts.registered_tensors(model, dst), out):
            li = t["parts"][0][0]
            lt = lts[li]
            leaf = lt["name"].split(".")[-1]
            for i in range(o.shape[0]):
                for j in range(o.shape[1]):
                    I, J = closed_form_global(model, leaf, D, d, i, j, lt["rows"], lt["cols"])
                    assert o[i, j] == (li << 20) + I * lt["cols"] + J, (lt["name"], i, j)


def test_moe_expert_parallel_to_stacked_tensor_parallel():
    model = tiny_moe()
    full = full_weights(model)
    lts = layouts.logical_tensors(model)
    P, D = 4, 2
    for d in range(D):
        dst = L(D, d, experts_stacked=1)
        out = reshard.empty_tensors(model, dst, fill=0xFFFFFFFF)
        counts = [np.zeros(t.shape, dtype=np.int32) for t in out]
        for p in range(P):
            src = L(1, 0, ep_size=P, ep_rank=p)
            wire = reshard.pack(model, src, dst, shard_of(model, src, full))
            reshard.unpack(model, src, dst, wire, out, counts)
            if p == 0:
                # after the first holder only its two experts' slabs (and all non-expert data) are filled
                by = {t["name"]: c for t, c in zip(layouts.registered_tensors(model, dst), counts)}
                w13 = by["layers.0.experts.w13"]
                per = w13.shape[0] // 8
                assert np.all(w13[:2 * per] == 1) and np.all(w13[2 * per:] == 0)
                assert np.all(by["layers.0.qkv_proj"] == 1)
        want = shard_of(model, dst, full)
        for t, o, w, c in zip(layouts.registered_tensors(model, dst), out, want, counts):
            assert np.all(c == 1), t["name"]
            assert np.array_equal(o, w), t["name"]
        # slab e of the stacked tensor is expert e's own tensor-parallel shard
        by = {t["name"]: o for t, o in zip(layouts.registered_tensors(model, dst), out)}
        w2 = by["layers.0.experts.w2"].reshape(8, model["hidden"], -1)
        for e in range(8):
            li = [i for i, lt in enumerate(lts) if lt["name"] == "layers.0.experts.%d.w2" % e][0]
            assert np.array_equal(w2[e], np.split(full[li], D, axis=1)[d])


def test_wire_equals_definition_without_wire():
    """pack -> unpack lands exactly what the wire-free result definition gives, incl. narrowing of norms."""
    for name in ("small_dense_tp1_to_tp4", "small_dense_tp4_to_tp2", "small_moe_ep4_to_tp2",
                 "small_dense_trainer_to_rollout", "small_dense_rollout_to_trainer",
                 "small_moe_stacked_to_per_expert", "small_dense_kvrep_tp8_to_tp2",
                 "small_dense_kvrep_tp2_to_tp16"):
        w = synth.workload(name)
        model, dst = w["model"], w["reader"]
        rng = np.random.default_rng(w["seed"])
        tensors = []
        for src in w["holders"]:
            ts = []
            for t in layouts.registered_tensors(model, src):
                if t["dtype"] == "f32":
                    ts.append(rng.integers(0, 1 << 32, size=(t["rows"], t["cols"]), dtype=np.uint64).astype(np.uint32))
                else:
                    ts.append(rng.integers(0, 1 << 16, size=(t["rows"], t["cols"])).astype(np.uint16))
            tensors.append(ts)
        want, mask = reshard.reshard_by_definition(model, w["holders"], tensors, dst)
        out = reshard.empty_tensors(model, dst, fill=0)
        counts = [np.zeros(t.shape, dtype=np.int32) for t in out]
        for src, ts in zip(w["holders"], tensors):
            wire = reshard.pack(model, src, dst, ts)
            reshard.unpack(model, src, dst, wire, out, counts)
        for o, x, m, c in zip(out, want, mask, counts):
            assert np.array_equal(c == 1, m) and np.all(c <= 1)
            assert np.array_equal(o, x)


# ---- stream lengths: closed forms from the shapes ----------------------------------------------

def test_stream_length_closed_forms_full_size_configs():
    # 8B, TP=1 -> TP=4 rank 0, norms narrowed to bf16; every run is a multiple of 16 bytes
    H, V, F, hd = 4096, 128256, 14336, 128
    per_layer = ((8 + 2 + 2) * hd * H) + (H * 32 * hd // 4) + (2 * F // 4 * H) + (H * F // 4) + 2 * H
    elems = 2 * (V // 4) * H + 32 * per_layer + H
    assert elems * 2 == 4_015_529_984
    w = synth.workload("cfg2_8b_tp1_to_tp4")
    assert reshard.wire_bytes(w["model"], w["holders"][0], w["reader"]) == elems * 2
    # 70B, TP=8 holders 0/1 -> TP=4 rank 0: each holder sends its whole shard; holder 0 adds the norms
    H, V, F = 8192, 128256, 28672
    shard = 2 * (V // 8) * H + 80 * (((8 + 1 + 1) * hd * H) + (H * 64 * hd // 8) + (2 * F // 8 * H) + (H * F // 8))
    norms = 80 * 2 * H + H
    w = synth.workload("cfg3_70b_tp8_to_tp4")
    assert (shard + norms) * 2 == 17_640_734_720 and shard * 2 == 17_638_096_896
    assert reshard.wire_bytes(w["model"], w["holders"][0], w["reader"]) == (shard + norms) * 2
    assert reshard.wire_bytes(w["model"], w["holders"][1], w["reader"]) == shard * 2


def test_stream_length_closed_form_moe():
    H, V, Fe, hd = 2048, 102400, 1408, 128
    attn = (16 * 3 * hd * H) // 2 + (H * 16 * hd) // 2
    experts = (8 + 2) * ((2 * Fe // 2) * H + H * (Fe // 2))
    per_layer = attn + experts + 64 * H + 2 * H
    elems = 2 * (V // 2) * H + 24 * per_layer + H
    assert elems * 2 == 2_904_756_224
    w = synth.workload("cfg4_moe_ep8_to_tp2")
    assert reshard.wire_bytes(w["model"], w["holders"][0], w["reader"]) == elems * 2


def test_narrowing_at_unpack_gives_the_same_reader_tensors_over_a_wider_wire():
    """The wire carries fp32 for the norms and the reader narrows: same destination bits, and the
    stream is longer by exactly 2 bytes per narrowed element."""
    for name in ("small_dense_tp1_to_tp4", "small_dense_trainer_to_rollout"):
        w = synth.workload(name)
        model, dst = w["model"], w["reader"]
        rng = np.random.default_rng(3)
        for src in w["holders"]:
            ts = []
            for t in layouts.registered_tensors(model, src):
                hi = 1 << (32 if t["dtype"] == "f32" else 16)
                ts.append(rng.integers(0, hi, size=(t["rows"], t["cols"]), dtype=np.uint64).astype(reshard.NPBITS[t["dtype"]]))
            a = reshard.empty_tensors(model, dst, fill=0)
            b = reshard.empty_tensors(model, dst, fill=0)
            w_pack = reshard.pack(model, src, dst, ts)
            w_unpack = reshard.pack(model, src, dst, ts, narrow_at="unpack")
            reshard.unpack(model, src, dst, w_pack, a)
            reshard.unpack(model, src, dst, w_unpack, b, narrow_at="unpack")
            for x, y in zip(a, b):
                assert np.array_equal(x, y)
            narrowed = sum(len(it["src_r"]) * len(it["src_c"]) for it in reshard.plan_items(model, src, dst)
                           if it["src_dtype"] != it["dst_dtype"])
            if narrowed:
                assert len(w_unpack) > len(w_pack)
                # runs stay 16-byte aligned, so the difference is the extra payload up to alignment gaps
                assert 0 <= len(w_unpack) - len(w_pack) - 2 * narrowed < 16 * len(ts)
            assert len(w_unpack) == reshard.wire_bytes(model, src, dst, narrow_at="unpack")


def test_chunks_tile_the_stream():
    wire = np.arange(1000, dtype=np.uint8)
    cs = reshard.chunks(wire, 256)
    assert [len(c) for c in cs] == [256, 256, 256, 232]
    assert np.array_equal(np.concatenate(cs), wire)
    with pytest.raises(ValueError):
        reshard.chunks(wire, 100)


def test_alignment_gap_is_zero_and_at_most_14_bytes():
    # hidden 9 in fp32 -> runs that are not multiples of 16 bytes
    model = tiny_model(hidden=9, n_q_heads=2, n_kv_heads=2, head_dim=1, ffn=3, vocab=5, weight_dtype="bf16")
    lay = L(1, 0)
    regs = layouts.registered_tensors(model, lay)
    tensors = [np.full((t["rows"], t["cols"]), 0xFFFF if t["dtype"] == "bf16" else 0xFFFFFFFF,
                       dtype=reshard.NPBITS[t["dtype"]]) for t in regs]
    wire = reshard.pack(model, lay, L(1, 0, f32_store="bf16"), tensors)
    items = list(reshard.plan_items(model, lay, L(1, 0, f32_store="bf16")))
    end = 0
    for it in items:
        assert it["wire_off"] % 16 == 0 and 0 <= it["wire_off"] - end <= 14
        assert not wire[end:it["wire_off"]].any()
        end = it["wire_off"] + len(it["src_r"]) * len(it["src_c"]) * 2
    assert end == len(wire)
