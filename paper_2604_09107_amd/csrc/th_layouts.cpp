// Model-level layouts: what each rank's registered tensors hold, as rectangles
// ("blocks") of the logical weights, and the rectangles that move from a holder
// rank to a reader rank.
//
// The paper treats shards as opaque (Sec. 4.1: a replica is divided into shards,
// one per worker) and only says that weights are resharded before transfer
// (Sec. 2.1, step 4).  The shard shapes used here are the common tensor- /
// expert-parallel conventions documented in th.h.
#include <algorithm>
#include <array>
#include <cstdarg>
#include <exception>
#include <map>
#include <new>

#include "th_internal.hpp"

namespace th {
namespace {

enum Part { P_REPL, P_SPLIT_ROWS, P_SPLIT_COLS, P_QKV, P_GATE_UP, P_VOCAB_ROWS };

struct Logical {
    std::string name;
    int64_t rows, cols;
    Part part;
    bool norm;
    int expert;  // routed expert index, -1 otherwise
};

// A rectangle of logical weight `logical` ([g_r0, g_r0+nr) x [g_c0, g_c0+nc)) stored at local
// position (l_r0, l_c0) of a registered tensor.
struct Block {
    int logical;
    int64_t g_r0, g_c0, nr, nc, l_r0, l_c0;
    int rep_index = 0, rep_count = 1;  // this rank's copy number among the ranks that keep the block
};

struct Reg {
    TensorInfo info;
    std::vector<Block> blocks;
};

std::vector<Logical> build_logicals(const th_model_desc& m) {
    std::vector<Logical> v;
    const int64_t H = m.hidden, hd = m.head_dim;
    auto add = [&](std::string name, int64_t r, int64_t c, Part p, bool norm = false, int e = -1) {
        v.push_back(Logical{std::move(name), r, c, p, norm, e});
    };
    add("embed_tokens", m.vocab, H, P_VOCAB_ROWS);
    for (int l = 0; l < m.n_layers; ++l) {
        const std::string p = "layers." + std::to_string(l) + ".";
        add(p + "input_norm", 1, H, P_REPL, true);
        add(p + "qkv_proj", (int64_t)(m.n_q_heads + 2 * m.n_kv_heads) * hd, H, P_QKV);
        add(p + "o_proj", H, (int64_t)m.n_q_heads * hd, P_SPLIT_COLS);
        add(p + "post_attn_norm", 1, H, P_REPL, true);
        if (m.kind == TH_MODEL_MOE) {
            const int64_t F = m.expert_ffn;
            add(p + "router", m.n_experts, H, P_REPL);
            for (int e = 0; e < m.n_experts; ++e) {
                const std::string q = p + "experts." + std::to_string(e) + ".";
                add(q + "w13", 2 * F, H, P_GATE_UP, false, e);
                add(q + "w2", H, F, P_SPLIT_COLS, false, e);
            }
            for (int s = 0; s < m.n_shared_experts; ++s) {
                const std::string q = p + "shared." + std::to_string(s) + ".";
                add(q + "w13", 2 * F, H, P_GATE_UP);
                add(q + "w2", H, F, P_SPLIT_COLS);
            }
        } else {
            add(p + "gate_up_proj", 2 * (int64_t)m.ffn, H, P_GATE_UP);
            add(p + "down_proj", H, m.ffn, P_SPLIT_COLS);
        }
    }
    add("final_norm", 1, H, P_REPL, true);
    if (!m.tied_embeddings) add("lm_head", m.vocab, H, P_VOCAB_ROWS);
    return v;
}

int check_div(int64_t n, int64_t parts, const std::string& what) {
    if (n % parts) {
        set_error("%s = %lld does not split evenly over %lld ranks", what.c_str(), (long long)n,
                  (long long)parts);
        return TH_ERR_INDIVISIBLE;
    }
    return TH_OK;
}

// Global rectangles that tensor-parallel rank r of T keeps of `lt`, top to bottom in local order.
// *kv_rep: > 1 when the rectangles after the first are K/V heads that kv_rep ranks keep copies of.
// *storage_rows receives the rows of the rank's tensor (more than the rectangles' rows when the
// vocabulary is padded: the padding rows follow the kept ones).
int shard_rects(const th_model_desc& m, const Logical& lt, const th_layout& lay,
                std::vector<std::array<int64_t, 4>>& out, int64_t* storage_rows, int* kv_rep) {
    out.clear();
    *kv_rep = 1;
    const int T = lay.tp_size, r = lay.tp_rank;
    const int64_t R = lt.rows, C = lt.cols;
    int rc;
    *storage_rows = -1;
    switch (lt.part) {
        case P_REPL:
            out.push_back({0, 0, R, C});
            break;
        case P_SPLIT_ROWS:
            if ((rc = check_div(R, T, lt.name + " rows"))) return rc;
            out.push_back({r * (R / T), 0, R / T, C});
            break;
        case P_VOCAB_ROWS: {
            const int64_t padded = lay.padded_vocab ? lay.padded_vocab : R;
            if (padded < R) {
                set_error("padded_vocab %lld is smaller than the vocabulary %lld", (long long)padded, (long long)R);
                return TH_ERR_ARG;
            }
            if ((rc = check_div(padded, T, lt.name + " (padded) rows"))) return rc;
            const int64_t n = padded / T, lo = r * n, hi = std::min<int64_t>(R, lo + n);
            if (hi > lo) out.push_back({lo, 0, hi - lo, C});
            *storage_rows = n;
            break;
        }
        case P_SPLIT_COLS:
            if ((rc = check_div(C, T, lt.name + " columns"))) return rc;
            out.push_back({0, r * (C / T), R, C / T});
            break;
        case P_QKV: {
            if ((rc = check_div(m.n_q_heads, T, "n_q_heads"))) return rc;
            const int64_t hd = m.head_dim;
            if (T > m.n_kv_heads) {
                // more ranks than KV heads: T / n_kv consecutive ranks keep copies of one KV head
                if (T % m.n_kv_heads) {
                    set_error("tp_size %d is neither a divisor nor a multiple of n_kv_heads %d", T, m.n_kv_heads);
                    return TH_ERR_UNSUPPORTED;
                }
                const int rep = T / m.n_kv_heads;
                const int64_t g = r / rep, qrows = (int64_t)m.n_q_heads / T * hd;
                out.push_back({r * qrows, 0, qrows, C});
                out.push_back({(int64_t)m.n_q_heads * hd + g * hd, 0, hd, C});
                out.push_back({(int64_t)(m.n_q_heads + m.n_kv_heads) * hd + g * hd, 0, hd, C});
                *kv_rep = rep;
                break;
            }
            if (m.n_kv_heads % T) {
                set_error("tp_size %d is neither a divisor nor a multiple of n_kv_heads %d", T, m.n_kv_heads);
                return TH_ERR_UNSUPPORTED;
            }
            const int64_t q = (int64_t)m.n_q_heads / T * hd, kv = (int64_t)m.n_kv_heads / T * hd;
            const int64_t k_base = (int64_t)m.n_q_heads * hd, v_base = k_base + (int64_t)m.n_kv_heads * hd;
            if (lay.qkv_grouped) {
                // per KV head of the rank: its query heads, its K head, its V head
                const int64_t per = (int64_t)(m.n_q_heads / m.n_kv_heads) * hd;
                const int64_t g0 = (int64_t)r * (m.n_kv_heads / T), g1 = g0 + m.n_kv_heads / T;
                for (int64_t g = g0; g < g1; ++g) {
                    out.push_back({g * per, 0, per, C});
                    out.push_back({k_base + g * hd, 0, hd, C});
                    out.push_back({v_base + g * hd, 0, hd, C});
                }
            } else {
                out.push_back({r * q, 0, q, C});
                out.push_back({k_base + r * kv, 0, kv, C});
                out.push_back({v_base + r * kv, 0, kv, C});
            }
            break;
        }
        case P_GATE_UP: {
            const int64_t F = R / 2;
            if ((rc = check_div(F, T, lt.name + " ffn"))) return rc;
            const int64_t f = F / T;
            out.push_back({r * f, 0, f, C});
            out.push_back({F + r * f, 0, f, C});
            break;
        }
    }
    return TH_OK;
}

int storage_dtype(const th_model_desc& m, const Logical& lt, const th_layout& lay) {
    const int d = lt.norm ? m.norm_dtype : m.weight_dtype;
    return d == TH_F32 ? lay.f32_store : d;
}

int build_regs(const th_model_desc& m, const std::vector<Logical>& lts, const th_layout& lay,
               std::vector<Reg>& regs) {
    regs.clear();
    std::map<std::string, size_t> stacked;  // stacked tensor name -> index in regs
    std::vector<std::array<int64_t, 4>> rects;
    int64_t experts_per_rank = 0;
    if (m.kind == TH_MODEL_MOE) {
        if (int rc = check_div(m.n_experts, lay.ep_size, "n_experts")) return rc;
        experts_per_rank = m.n_experts / lay.ep_size;
    }
    for (size_t i = 0; i < lts.size(); ++i) {
        const Logical& lt = lts[i];
        if (lt.expert >= 0 && lt.expert / experts_per_rank != lay.ep_rank) continue;
        int64_t storage_rows = -1;
        int kv_rep = 1;
        if (int rc = shard_rects(m, lt, lay, rects, &storage_rows, &kv_rep)) return rc;
        const int dt = storage_dtype(m, lt, lay);
        const uint64_t cols = lt.part == P_SPLIT_COLS ? (uint64_t)(lt.cols / lay.tp_size) : (uint64_t)lt.cols;
        Reg* reg;
        if (lt.expert >= 0 && lay.experts_stacked) {
            // "layers.L.experts.E.w13" -> "layers.L.experts.w13"
            const size_t leaf = lt.name.rfind('.');
            const size_t idx = lt.name.rfind('.', leaf - 1);
            const std::string name = lt.name.substr(0, idx) + lt.name.substr(leaf);
            auto it = stacked.find(name);
            if (it == stacked.end()) {
                it = stacked.emplace(name, regs.size()).first;
                regs.emplace_back();
                regs.back().info.name = name;
                regs.back().info.dtype = dt;
                regs.back().info.cols = cols;
            }
            reg = &regs[it->second];
        } else {
            regs.emplace_back();
            reg = &regs.back();
            reg->info.name = lt.name;
            reg->info.dtype = dt;
            reg->info.cols = cols;
        }
        const uint64_t rows_before = reg->info.rows;
        for (size_t k = 0; k < rects.size(); ++k) {
            const auto& q = rects[k];
            Block b{(int)i, q[0], q[1], q[2], q[3], (int64_t)reg->info.rows, 0};
            if (kv_rep > 1 && k > 0) {
                b.rep_index = lay.tp_rank % kv_rep;
                b.rep_count = kv_rep;
            }
            reg->blocks.push_back(b);
            reg->info.rows += (uint64_t)q[2];
        }
        if (storage_rows >= 0) reg->info.rows = rows_before + (uint64_t)storage_rows;  // padding rows follow
    }
    return TH_OK;
}

// Of all holders that keep a copy of replicated data, only one sends it to a given reader.
bool supplies(const Logical& lt, const th_layout& src, const th_layout& dst) {
    if (lt.part == P_REPL && src.tp_rank != (int)((int64_t)dst.tp_rank * src.tp_size / dst.tp_size))
        return false;
    if (lt.expert < 0 && src.ep_rank != (int)((int64_t)dst.ep_rank * src.ep_size / dst.ep_size))
        return false;
    return true;
}

int check_layout(const th_layout& l, const char* who) {
    if (l.tp_size < 1 || l.ep_size < 1 || l.tp_rank < 0 || l.tp_rank >= l.tp_size || l.ep_rank < 0 ||
        l.ep_rank >= l.ep_size || (l.f32_store != TH_BF16 && l.f32_store != TH_F32) || l.padded_vocab < 0) {
        set_error("%s layout: bad parallel size / rank / f32_store / padded_vocab", who);
        return TH_ERR_ARG;
    }
    return TH_OK;
}

struct Piece {  // a needed rectangle in holder-tensor coordinates and where it lands
    int64_t s_r0, s_c0, nr, nc;
    uint32_t dst_tensor;
    int64_t d_r0, d_c0;
};

}  // namespace

static int build_model_segments_impl(const th_model_desc& m, const th_layout& src, const th_layout& dst,
                                     bool narrow_at_unpack, Manifest& man) {
    if ((m.kind != TH_MODEL_DENSE && m.kind != TH_MODEL_MOE) || m.n_layers < 0 || m.hidden < 1 ||
        m.n_q_heads < 1 || m.n_kv_heads < 1 || m.head_dim < 1 || m.vocab < 1 ||
        (m.weight_dtype != TH_BF16 && m.weight_dtype != TH_F32) ||
        (m.norm_dtype != TH_BF16 && m.norm_dtype != TH_F32)) {
        set_error("model description: bad kind, dimension or dtype");
        return TH_ERR_ARG;
    }
    if (m.kind == TH_MODEL_DENSE && m.ffn < 1) {
        set_error("model description: dense model needs ffn >= 1");
        return TH_ERR_ARG;
    }
    if (m.kind == TH_MODEL_MOE && (m.n_experts < 1 || m.expert_ffn < 1 || m.n_shared_experts < 0)) {
        set_error("model description: MoE model needs n_experts >= 1 and expert_ffn >= 1");
        return TH_ERR_ARG;
    }
    if (m.n_q_heads % m.n_kv_heads) {
        set_error("n_q_heads %d is not a multiple of n_kv_heads %d", m.n_q_heads, m.n_kv_heads);
        return TH_ERR_ARG;
    }
    if (int rc = check_layout(src, "source")) return rc;
    if (int rc = check_layout(dst, "destination")) return rc;

    const std::vector<Logical> lts = build_logicals(m);
    std::vector<Reg> sregs, dregs;
    if (int rc = build_regs(m, lts, src, sregs)) return rc;
    if (int rc = build_regs(m, lts, dst, dregs)) return rc;
    for (auto& r : sregs) man.tensors[0].push_back(r.info);
    for (auto& r : dregs) man.tensors[1].push_back(r.info);

    // logical weight -> the reader's blocks of it
    std::vector<std::vector<std::pair<uint32_t, Block>>> dst_of(lts.size());
    for (size_t d = 0; d < dregs.size(); ++d)
        for (const Block& b : dregs[d].blocks) dst_of[b.logical].push_back({(uint32_t)d, b});

    uint64_t wire = 0;
    std::vector<Piece> pieces;
    for (size_t s = 0; s < sregs.size(); ++s) {
        const Reg& sr = sregs[s];
        pieces.clear();
        for (const Block& b : sr.blocks) {
            if (!supplies(lts[b.logical], src, dst)) continue;
            if (b.rep_count > 1) {
                // of the holders that keep a copy, reader number j of the rep_d readers that want the
                // block pulls from copy floor(j * rep_s / rep_d)
                const int rep_d = std::max(1, dst.tp_size / m.n_kv_heads);
                if (b.rep_index != (dst.tp_rank % rep_d) * b.rep_count / rep_d) continue;
            }
            for (const auto& db : dst_of[b.logical]) {
                const Block& d = db.second;
                const int64_t r0 = std::max(b.g_r0, d.g_r0), r1 = std::min(b.g_r0 + b.nr, d.g_r0 + d.nr);
                const int64_t c0 = std::max(b.g_c0, d.g_c0), c1 = std::min(b.g_c0 + b.nc, d.g_c0 + d.nc);
                if (r0 >= r1 || c0 >= c1) continue;
                pieces.push_back(Piece{b.l_r0 + (r0 - b.g_r0), b.l_c0 + (c0 - b.g_c0), r1 - r0, c1 - c0,
                                       db.first, d.l_r0 + (r0 - d.g_r0), d.l_c0 + (c0 - d.g_c0)});
            }
        }
        if (pieces.empty()) continue;

        // Wire order is the holder tensor's row-major order over the needed elements.  Cut the
        // needed rows into bands whose set of needed column intervals is constant; inside a band
        // a wire row is the concatenation of the band's column intervals.
        std::vector<int64_t> cuts;
        for (const Piece& p : pieces) {
            cuts.push_back(p.s_r0);
            cuts.push_back(p.s_r0 + p.nr);
        }
        std::sort(cuts.begin(), cuts.end());
        cuts.erase(std::unique(cuts.begin(), cuts.end()), cuts.end());

        wire = (wire + 15) / 16 * 16;
        const uint64_t run_start = wire;
        const size_t first_seg = man.segments.size();
        std::vector<size_t> open;  // segments of the previous band, by column order
        std::vector<const Piece*> band;
        for (size_t k = 0; k + 1 < cuts.size(); ++k) {
            const int64_t a = cuts[k], b = cuts[k + 1];
            band.clear();
            for (const Piece& p : pieces)
                if (p.s_r0 <= a && b <= p.s_r0 + p.nr) band.push_back(&p);
            if (band.empty()) {
                open.clear();
                continue;
            }
            std::sort(band.begin(), band.end(), [](const Piece* x, const Piece* y) { return x->s_c0 < y->s_c0; });
            uint64_t width = 0;
            for (const Piece* p : band) width += (uint64_t)p->nc;
            std::vector<size_t> now;
            uint64_t prefix = 0;
            for (size_t j = 0; j < band.size(); ++j) {
                const Piece& p = *band[j];
                const TensorInfo& dt = man.tensors[1][p.dst_tensor];
                const int wire_dtype = narrow_at_unpack ? sr.info.dtype : dt.dtype;
                const unsigned es = esize(wire_dtype);
                if (sr.info.dtype == TH_BF16 && dt.dtype == TH_F32) {
                    set_error("tensor %s: bf16 -> fp32 widening is not supported", sr.info.name.c_str());
                    return TH_ERR_UNSUPPORTED;
                }
                Segment g;
                g.src_tensor = (uint32_t)s;
                g.dst_tensor = p.dst_tensor;
                g.src_off = (uint64_t)a * sr.info.cols + (uint64_t)p.s_c0;
                g.src_stride = sr.info.cols;
                g.dst_off = (uint64_t)(p.d_r0 + (a - p.s_r0)) * dt.cols + (uint64_t)p.d_c0;
                g.dst_stride = dt.cols;
                g.nrows = (uint64_t)(b - a);
                g.row_len = (uint64_t)p.nc;
                g.wire_off = wire + prefix * es;
                g.wire_stride = width * es;
                g.src_dtype = (uint8_t)sr.info.dtype;
                g.dst_dtype = (uint8_t)dt.dtype;
                g.wire_dtype = (uint8_t)wire_dtype;
                g.run_start = run_start;
                prefix += (uint64_t)p.nc;
                // continue the segment of the previous band if this one extends it downwards
                bool merged = false;
                if (open.size() == band.size()) {
                    Segment& o = man.segments[open[j]];
                    if (o.dst_tensor == g.dst_tensor && o.row_len == g.row_len && o.src_stride == g.src_stride &&
                        o.dst_stride == g.dst_stride && o.wire_stride == g.wire_stride &&
                        o.src_off + o.nrows * o.src_stride == g.src_off &&
                        o.dst_off + o.nrows * o.dst_stride == g.dst_off &&
                        o.wire_off + o.nrows * o.wire_stride == g.wire_off) {
                        o.nrows += g.nrows;
                        now.push_back(open[j]);
                        merged = true;
                    }
                }
                if (!merged) {
                    now.push_back(man.segments.size());
                    man.segments.push_back(g);
                }
            }
            open.swap(now);
            // all pieces of one holder tensor land in tensors of one dtype, so one element size per band
            wire += (uint64_t)(b - a) * width *
                    esize(narrow_at_unpack ? sr.info.dtype : man.tensors[1][band[0]->dst_tensor].dtype);
        }
        // the alignment gap that follows this tensor's run is written by whoever holds its last element
        const uint64_t gap = (16 - wire % 16) % 16;
        if (gap) {
            for (size_t i = first_seg; i < man.segments.size(); ++i) {
                Segment& g = man.segments[i];
                const uint64_t end = g.wire_off + (g.nrows - 1) * g.wire_stride + g.row_len * esize(g.wire_dtype);
                if (end == wire) g.pad_after = (uint8_t)gap;
            }
        }
    }
    // no gap is owed after the last run of the stream
    uint64_t last_end = 0;
    for (const Segment& g : man.segments)
        last_end = std::max(last_end, g.wire_off + (g.nrows - 1) * g.wire_stride + g.row_len * esize(g.wire_dtype));
    for (Segment& g : man.segments)
        if (g.wire_off + (g.nrows - 1) * g.wire_stride + g.row_len * esize(g.wire_dtype) == last_end) g.pad_after = 0;
    return TH_OK;
}

// Nothing may leave this file as an exception: the callers are extern "C".
int build_model_segments(const th_model_desc& m, const th_layout& src, const th_layout& dst,
                         bool narrow_at_unpack, Manifest& man) {
    try {
        return build_model_segments_impl(m, src, dst, narrow_at_unpack, man);
    } catch (const std::bad_alloc&) {
        set_error("out of memory");
        return TH_ERR_NOMEM;
    } catch (const std::exception& e) {
        set_error("layout planner failed: %s", e.what());
        return TH_ERR_NOMEM;
    } catch (...) {
        set_error("layout planner failed");
        return TH_ERR_NOMEM;
    }
}

}  // namespace th
