"""Model shapes and (holder -> reader) layout pairings of the five workloads.

Shapes are public Llama-3-8B / 70B-like and DeepSeek-MoE-like dimensions; they
stand in for the proprietary 9B-1T production models of the paper's Table 3.
A layout here is only a tuple of parallel sizes / ranks; what a rank *holds*
under such a layout is worked out independently by the oracle and by the
library's planner.
"""

MiB = 1 << 20


def layout(tp_size=1, tp_rank=0, ep_size=1, ep_rank=0, experts_stacked=0, f32_store="f32",
           qkv_grouped=0, padded_vocab=0):
    """One worker's place in a model-parallel group.

    f32_store: dtype in which this side keeps tensors whose model dtype is
    fp32 ("f32" keeps them, "bf16" narrows them: the inference-ready format).
    qkv_grouped: the fused QKV tensor is stored per KV group (trainer style)
    instead of all Q, then all K, then all V.
    padded_vocab: vocabulary size the embedding / output tables are padded to
    on this side before they are split over ranks (0 = not padded).
    """
    assert f32_store in ("f32", "bf16")
    return dict(tp_size=tp_size, tp_rank=tp_rank, ep_size=ep_size, ep_rank=ep_rank,
                experts_stacked=experts_stacked, f32_store=f32_store, qkv_grouped=qkv_grouped,
                padded_vocab=padded_vocab)


def _dense(n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab, tied):
    return dict(kind="dense", n_layers=n_layers, hidden=hidden, n_q_heads=n_q_heads,
                n_kv_heads=n_kv_heads, head_dim=head_dim, ffn=ffn, vocab=vocab,
                tied_embeddings=tied, n_experts=0, n_shared_experts=0, expert_ffn=0,
                weight_dtype="bf16", norm_dtype="f32")


MODELS = {
    # config 1: tiny Llama-style, tied embeddings
    "tiny": _dense(2, 256, 4, 2, 64, 1024, 1000, 1),
    # config 2: 8B-shaped dense
    "dense8b": _dense(32, 4096, 32, 8, 128, 14336, 128256, 0),
    # config 3: 70B-shaped dense
    "dense70b": _dense(80, 8192, 64, 8, 128, 28672, 128256, 0),
    # config 4: MoE-shaped, 64 routed + 2 shared experts per layer
    "moe": dict(kind="moe", n_layers=24, hidden=2048, n_q_heads=16, n_kv_heads=16, head_dim=128,
                ffn=0, vocab=102400, tied_embeddings=0, n_experts=64, n_shared_experts=2,
                expert_ffn=1408, weight_dtype="bf16", norm_dtype="f32"),
    # reduced shapes of the same families, for CPU tests and quick GPU parity
    "dense_small": _dense(3, 512, 8, 4, 64, 1536, 4096, 0),
    "dense_small_v4000": _dense(2, 512, 8, 4, 64, 1536, 4000, 0),
    "dense_small_kv": _dense(2, 512, 16, 4, 32, 1024, 2048, 0),  # 16 query heads over 4 KV heads
    "moe_small": dict(kind="moe", n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64,
                      ffn=0, vocab=2048, tied_embeddings=0, n_experts=16, n_shared_experts=2,
                      expert_ffn=176, weight_dtype="bf16", norm_dtype="f32"),
}

WORKLOADS = {
    # tiny Llama, both TP=2 holders -> one TP=1 reader, 1 MiB chunks
    "cfg1_tiny_tp2_to_tp1": dict(
        model="tiny", seed=1, chunk_bytes=1 * MiB,
        holders=[layout(2, 0), layout(2, 1)],
        reader=layout(1, 0, f32_store="bf16")),
    # 8B, TP=1 holder -> TP=4 rank-0 reader, 64 MiB chunks
    "cfg2_8b_tp1_to_tp4": dict(
        model="dense8b", seed=2, chunk_bytes=64 * MiB,
        holders=[layout(1, 0)],
        reader=layout(4, 0, f32_store="bf16")),
    # 70B, TP=8 holders 0 and 1 -> TP=4 rank-0 reader, 256 MiB chunks
    "cfg3_70b_tp8_to_tp4": dict(
        model="dense70b", seed=3, chunk_bytes=256 * MiB,
        holders=[layout(8, 0), layout(8, 1)],
        reader=layout(4, 0, f32_store="bf16")),
    # MoE, EP=8 rank-0 holder (per-expert tensors, TP=1 attention) -> TP=2 rank-0
    # reader with stacked experts, 4 MiB chunks
    "cfg4_moe_ep8_to_tp2": dict(
        model="moe", seed=4, chunk_bytes=4 * MiB,
        holders=[layout(1, 0, ep_size=8, ep_rank=0)],
        reader=layout(2, 0, experts_stacked=1, f32_store="bf16")),
    # 100,000 fp32 master tensors (tilted size distribution, ~40 GB), 2-D strided sub-slices in a
    # random wire order, narrowed to bf16 through 16 MiB chunks into a dense arena
    "cfg5_scatter_fp32_to_bf16": dict(kind="scatter", n_tensors=100_000, seed=5, chunk_bytes=16 * MiB),
    "small_scatter": dict(kind="scatter", n_tensors=2_000, seed=15, chunk_bytes=1 * MiB),
    # thousands of tiny tensors in one launch: 400,000 fp32 tensors of 256 B to 4 KiB (log-uniform), the
    # same strided sub-slices, wire order and dense bf16 arena as the scattered sweep
    "tiny_tensors_fp32_to_bf16": dict(kind="scatter", n_tensors=400_000, seed=6, chunk_bytes=16 * MiB,
                                      sizes=dict(min_bytes=256, max_bytes=4096, alpha=0.0)),
    # whole-model sweeps of the same three models: every reader rank the resident holders can feed
    # (parts = independent (holders -> reader) groups; holders named twice are resident once)
    "cfg2_8b_tp1_to_tp4_all_readers": dict(
        model="dense8b", seed=2, chunk_bytes=64 * MiB,
        parts=[dict(holders=[layout(1, 0)], reader=layout(4, r, f32_store="bf16")) for r in range(4)]),
    "cfg3_70b_tp8_to_tp4_two_readers": dict(
        model="dense70b", seed=3, chunk_bytes=256 * MiB,
        parts=[dict(holders=[layout(8, 2 * r), layout(8, 2 * r + 1)], reader=layout(4, r, f32_store="bf16"))
               for r in range(2)]),
    "cfg4_moe_ep8_to_tp2_all_holders": dict(
        model="moe", seed=4, chunk_bytes=4 * MiB,
        holders=[layout(1, 0, ep_size=8, ep_rank=p) for p in range(8)],
        reader=layout(2, 0, experts_stacked=1, f32_store="bf16")),
    # reduced variants
    "small_dense_tp1_to_tp4": dict(
        model="dense_small", seed=12, chunk_bytes=1 * MiB,
        holders=[layout(1, 0)],
        reader=layout(4, 0, f32_store="bf16")),
    "small_dense_tp4_to_tp2": dict(
        model="dense_small", seed=13, chunk_bytes=256 * 1024,
        holders=[layout(4, 2), layout(4, 3)],
        reader=layout(2, 1, f32_store="bf16")),
    # trainer-style source: group-interleaved QKV, vocabulary 4000 padded to 4096 over 4 ranks
    "small_dense_trainer_to_rollout": dict(
        model="dense_small_v4000", seed=16, chunk_bytes=256 * 1024,
        holders=[layout(4, 2, qkv_grouped=1, padded_vocab=4096), layout(4, 3, qkv_grouped=1, padded_vocab=4096)],
        reader=layout(2, 1, f32_store="bf16")),
    # and back: rollout-style source into a trainer-style reader (fp32 norms kept)
    "small_dense_rollout_to_trainer": dict(
        model="dense_small_v4000", seed=17, chunk_bytes=512 * 1024,
        holders=[layout(1, 0)],
        reader=layout(4, 3, qkv_grouped=1, padded_vocab=4096)),
    # more ranks than KV heads on the holder side (each KV head kept by two ranks)
    "small_dense_kvrep_tp8_to_tp2": dict(
        model="dense_small_kv", seed=19, chunk_bytes=128 * 1024,
        holders=[layout(8, 4), layout(8, 5), layout(8, 6), layout(8, 7)],
        reader=layout(2, 1, f32_store="bf16")),
    # ... and on the reader side
    "small_dense_kvrep_tp2_to_tp16": dict(
        model="dense_small_kv", seed=20, chunk_bytes=128 * 1024,
        holders=[layout(2, 1)],
        reader=layout(16, 13, f32_store="bf16")),
    # stacked experts at the source, per-expert tensors at the reader
    "small_moe_stacked_to_per_expert": dict(
        model="moe_small", seed=18, chunk_bytes=128 * 1024,
        holders=[layout(2, 1, experts_stacked=1)],
        reader=layout(1, 0, ep_size=2, ep_rank=1, f32_store="bf16")),
    "small_moe_ep4_to_tp2": dict(
        model="moe_small", seed=14, chunk_bytes=128 * 1024,
        holders=[layout(1, 0, ep_size=4, ep_rank=1)],
        reader=layout(2, 1, experts_stacked=1, f32_store="bf16")),
}


def workload(name):
    w = dict(WORKLOADS[name])
    w["name"] = name
    w.setdefault("kind", "model")
    if w["kind"] == "model":
        w["model_name"] = w["model"]
        w["model"] = dict(MODELS[w["model"]])
        if "parts" not in w:
            w["parts"] = [dict(holders=w["holders"], reader=w["reader"])]
        else:  # the first part doubles as the workload's plain (holders, reader) pair
            w["holders"], w["reader"] = w["parts"][0]["holders"], w["parts"][0]["reader"]
    else:
        w["model_name"] = "scattered fp32 tensors"
        w.setdefault("sizes", {})  # keyword arguments of scatter_description beyond (n_tensors, seed)
    return w
