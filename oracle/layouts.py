"""Oracle: which elements of each logical weight a rank holds.

The paper treats a replica as a set of opaque shards, one per worker of a
model-parallel group (Sec. 4.1), and says nothing about their shapes.  The
conventions below are the common tensor-parallel / expert-parallel ones and are
a reading, not the paper's text:

  * every weight is a logical row-major matrix W[out, in]; vectors are [1, n];
  * column-parallel (split rows):   lm_head;  vocab-parallel: embed_tokens;
  * row-parallel (split columns):   o_proj, down_proj, expert/shared w2;
  * fused QKV, global rows [Q heads | K heads | V heads]; rank r keeps its
    contiguous range of Q heads and of K/V heads, stored as [Q_r; K_r; V_r],
    or - "grouped", the trainer-side convention - per KV head g of the rank as
    [Q heads of group g; K_g; V_g], group after group; with more ranks than KV
    heads (T a multiple of n_kv) rank r keeps its Q heads and a copy of the one
    KV head they use, head r // (T / n_kv);
  * a side may pad the vocabulary of embed_tokens / lm_head to a larger size
    before splitting it; padding rows exist in the rank's tensor but belong to
    no logical weight: they are never sent and never written;
  * fused gate_up (and expert/shared w13), global rows [gate | up]; rank r keeps
    [gate_r; up_r];
  * replicated: norms, MoE router;
  * expert-parallel rank p of P keeps routed experts [p*E/P, (p+1)*E/P) whole;
    everything else is replicated across expert-parallel ranks.

A shard is described the plainest way possible: the vector of global row
indices and the vector of global column indices it keeps, in local order, so
that   local = global[np.ix_(rows, cols)].   No rectangles, no offsets.
Test infrastructure only.
"""
import numpy as np


def logical_tensors(model):
    """All logical weights of the model in registration order.

    Each entry: name, rows, cols, part (how tensor-parallel ranks split it),
    role ("weight" or "norm", selects the model dtype), expert (routed-expert
    index or None)."""
    H = model["hidden"]
    hd = model["head_dim"]
    nq, nkv = model["n_q_heads"], model["n_kv_heads"]
    out = []

    def add(name, rows, cols, part, role="weight", expert=None):
        out.append(dict(name=name, rows=rows, cols=cols, part=part, role=role, expert=expert))

    add("embed_tokens", model["vocab"], H, "vocab")
    for l in range(model["n_layers"]):
        p = "layers.%d." % l
        add(p + "input_norm", 1, H, "repl", role="norm")
        add(p + "qkv_proj", (nq + 2 * nkv) * hd, H, "qkv")
        add(p + "o_proj", H, nq * hd, "row")
        add(p + "post_attn_norm", 1, H, "repl", role="norm")
        if model["kind"] == "moe":
            F = model["expert_ffn"]
            add(p + "router", model["n_experts"], H, "repl")
            for e in range(model["n_experts"]):
                add(p + "experts.%d.w13" % e, 2 * F, H, "gate_up", expert=e)
                add(p + "experts.%d.w2" % e, H, F, "row", expert=e)
            for s in range(model["n_shared_experts"]):
                add(p + "shared.%d.w13" % s, 2 * F, H, "gate_up")
                add(p + "shared.%d.w2" % s, H, F, "row")
        else:
            F = model["ffn"]
            add(p + "gate_up_proj", 2 * F, H, "gate_up")
            add(p + "down_proj", H, F, "row")
    add("final_norm", 1, H, "repl", role="norm")
    if not model["tied_embeddings"]:
        add("lm_head", model["vocab"], H, "col")
    return out


def _split(n, parts, what):
    if n % parts:
        raise ValueError("%s = %d does not divide into %d parts" % (what, n, parts))
    return n // parts


def holds(model, lt, lay):
    """Does this rank hold (a shard of) the logical tensor at all?"""
    if lt["expert"] is None:
        return True
    per = _split(model["n_experts"], lay["ep_size"], "n_experts")
    return lt["expert"] // per == lay["ep_rank"]


def shard_index(model, lt, lay):
    """(rows, cols): global row / column indices kept by this rank, local order."""
    T, r = lay["tp_size"], lay["tp_rank"]
    R, C = lt["rows"], lt["cols"]
    rows, cols = np.arange(R), np.arange(C)
    part = lt["part"]
    if part == "repl":
        pass
    elif part in ("col", "vocab"):
        padded = lay.get("padded_vocab", 0) or R
        if padded < R:
            raise ValueError("padded vocabulary %d is smaller than the vocabulary %d" % (padded, R))
        n = _split(padded, T, lt["name"] + " rows")
        rows = np.arange(r * n, (r + 1) * n)
        rows = rows[rows < R]  # the rest of the rank's n rows is padding
    elif part == "row":
        n = _split(C, T, lt["name"] + " cols")
        cols = np.arange(r * n, (r + 1) * n)
    elif part == "qkv":
        hd = model["head_dim"]
        nq, nkv = model["n_q_heads"], model["n_kv_heads"]
        q = _split(nq, T, "n_q_heads")
        if T > nkv:
            # KV heads are replicated: T / n_kv consecutive ranks share one
            rep = _split(T, nkv, "tp_size over n_kv_heads")
            g = r // rep
            rows = np.concatenate([np.arange(r * q * hd, (r + 1) * q * hd),
                                   nq * hd + np.arange(g * hd, (g + 1) * hd),
                                   (nq + nkv) * hd + np.arange(g * hd, (g + 1) * hd)])
            return rows, cols
        kv = _split(nkv, T, "n_kv_heads")
        if lay.get("qkv_grouped", 0):
            per = nq // nkv  # query heads per KV head
            pieces = []
            for g in range(r * kv, (r + 1) * kv):  # the rank's KV heads
                pieces.append(np.arange(g * per * hd, (g + 1) * per * hd))
                pieces.append(nq * hd + np.arange(g * hd, (g + 1) * hd))
                pieces.append((nq + nkv) * hd + np.arange(g * hd, (g + 1) * hd))
            rows = np.concatenate(pieces)
        else:
            q_rows = np.arange(r * q * hd, (r + 1) * q * hd)
            k_rows = nq * hd + np.arange(r * kv * hd, (r + 1) * kv * hd)
            v_rows = (nq + nkv) * hd + np.arange(r * kv * hd, (r + 1) * kv * hd)
            rows = np.concatenate([q_rows, k_rows, v_rows])
    elif part == "gate_up":
        F = R // 2
        n = _split(F, T, lt["name"] + " ffn")
        gate = np.arange(r * n, (r + 1) * n)
        rows = np.concatenate([gate, F + gate])
    else:
        raise ValueError(part)
    return rows, cols


def storage_rows(model, lt, lay):
    """Rows the rank's tensor has for this logical weight: the kept rows, plus padding rows for a
    padded vocabulary (they follow the kept rows)."""
    rows, _ = shard_index(model, lt, lay)
    if lt["part"] in ("col", "vocab") and lay.get("padded_vocab", 0):
        return lay["padded_vocab"] // lay["tp_size"]
    return len(rows)


def storage_dtype(model, lt, lay):
    d = model["norm_dtype"] if lt["role"] == "norm" else model["weight_dtype"]
    return lay["f32_store"] if d == "f32" else d


def registered_tensors(model, lay):
    """The rank's registered tensors in registration order.

    Each entry: name, dtype, rows, cols (local 2-D shape; a stacked expert
    tensor [E, r, c] is listed as [E*r, c]) and parts = [(logical index,
    first local row)], the logical tensors stored in it, top to bottom."""
    lts = logical_tensors(model)
    out = []
    stacked = {}
    for i, lt in enumerate(lts):
        if not holds(model, lt, lay):
            continue
        rows, cols = shard_index(model, lt, lay)
        dt = storage_dtype(model, lt, lay)
        if lt["expert"] is not None and lay["experts_stacked"]:
            # "layers.L.experts.E.w13" -> one tensor "layers.L.experts.w13" per layer
            head, _, leaf = lt["name"].rpartition(".")
            name = head.rpartition(".")[0] + "." + leaf
            if name not in stacked:
                stacked[name] = dict(name=name, dtype=dt, rows=0, cols=len(cols), parts=[])
                out.append(stacked[name])
            t = stacked[name]
            t["parts"].append((i, t["rows"]))
            t["rows"] += len(rows)
        else:
            out.append(dict(name=lt["name"], dtype=dt, rows=storage_rows(model, lt, lay), cols=len(cols),
                            parts=[(i, 0)]))
    return out


def row_supply_mask(model, lt, src, dst):
    """For data that only some of the holder ranks replicate - K/V heads when the holders have
    more ranks than KV heads - which of this holder's rows it sends to reader `dst`: of the rep_s
    holders that keep a head, reader number j of the rep_d readers that want it (rep_d = 1 if the
    readers do not replicate) pulls from copy floor(j * rep_s / rep_d)."""
    rows, _ = shard_index(model, lt, src)
    mask = np.ones(len(rows), dtype=bool)
    nkv = model["n_kv_heads"]
    if lt["part"] == "qkv" and src["tp_size"] > nkv:
        rep_s = src["tp_size"] // nkv
        rep_d = max(1, dst["tp_size"] // nkv)
        mine = src["tp_rank"] % rep_s
        wanted = ((dst["tp_rank"] % rep_d) * rep_s) // rep_d
        is_kv = rows >= model["n_q_heads"] * model["head_dim"]
        mask[is_kv] = mine == wanted
    return mask


def supplies(model, lt, src, dst):
    """Exactly-once rule for replicated data: of all holders that keep a copy,
    only the primary one sends it to reader `dst`."""
    if lt["part"] == "repl" and src["tp_rank"] != (dst["tp_rank"] * src["tp_size"]) // dst["tp_size"]:
        return False
    if lt["expert"] is None and src["ep_rank"] != (dst["ep_rank"] * src["ep_size"]) // dst["ep_size"]:
        return False
    return True
