// Host planner: turns wire-ordered segments into the chunk manifest (runs) and the
// device work list (tiles).  Integer arithmetic only.
#include <algorithm>
#include <cstring>
#include <exception>
#include <new>
#include <thread>

#include "th_internal.hpp"

namespace th {
namespace {

typedef unsigned __int128 u128;

uint64_t seg_wire_end(const Segment& g) {
    return g.wire_off + (g.nrows - 1) * g.wire_stride + g.row_len * esize(g.wire_dtype);
}

unsigned ceil_log2(uint64_t v) {
    unsigned l = 0;
    while ((1ull << l) < v) ++l;
    return l;
}

struct Side {  // one end of a copy, in bytes
    uint32_t buf;
    uint64_t off, stride;
    unsigned es;
};

// Append the tiles of one run, seen as a copy S -> D of nrows x ncols elements.
// outs[0] receives the tiles of vector-path runs, outs[1] those of other runs, outs[2] those of
// short runs of either kind (one wavefront each); a run's tiles are all of one class.
void tile_run(std::vector<Tile>* outs, Side S, Side D, uint64_t nrows, uint64_t ncols, unsigned pad,
              bool bases_aligned16, const Tuning& tune, bool& used_vec) {
    // rows that follow each other without a gap on both ends are one long row
    if (nrows > 1 && S.stride == ncols * S.es && D.stride == ncols * D.es) {
        ncols *= nrows;
        nrows = 1;
    }
    const bool narrows = S.es == 4 && D.es == 2;
    // Vector path: every address a multiple of 16 bytes on both sides and the same dtype; or, when
    // narrowing, 16 bytes of source (four elements) for every 8 bytes of destination.
    const uint64_t unit_elems = 16 / S.es;  // elements per column unit of the vector path
    const uint64_t vs = 16, vd = unit_elems * D.es;  // unit bytes on either side: 16 / 16, or 16 / 8
    const bool vec = bases_aligned16 && pad == 0 && (S.es == D.es || narrows) && S.off % vs == 0 &&
                     D.off % vd == 0 && ncols % unit_elems == 0 &&
                     (nrows == 1 || (S.stride % vs == 0 && D.stride % vd == 0));
    used_vec = vec;
    // A run that is short as a whole (at most short_slots of the kernel's units of work per thread:
    // 16-byte vectors, or destination slots of 16 bytes, 8 when narrowing, one more per row for the
    // slot a row end can straddle) goes to the short class, whose tiles get one wavefront each.  The
    // last piece of a long run stays with the run's own class.
    const uint64_t slot_bytes = narrows ? 8 : 16;
    const uint64_t run_slots = vec ? nrows * (ncols / unit_elems) : nrows * ((ncols * D.es + slot_bytes - 1) / slot_bytes + 1);
    std::vector<Tile>& out = outs[run_slots <= tune.short_slots ? 2 : vec ? 0 : 1];
    const uint64_t tile_bytes = vec ? tune.tile_bytes : narrows ? tune.tile_bytes_narrow : tune.tile_bytes_any;
    uint32_t flags = vec ? TILE_KIND_VEC : TILE_KIND_ANY;
    if (S.es == 4) flags |= TILE_SRC_F32;
    if (D.es == 4) flags |= TILE_DST_F32;
    const uint64_t unit_d = vec ? vd : D.es, unit_s = vec ? vs : S.es;  // bytes per column unit
    const uint64_t units = ncols * D.es / unit_d;                        // column units per row
    const uint64_t row_bytes = ncols * D.es;

    if (vec) {
        // Cut the rectangle's vectors, taken in row-major order, into equal runs: every tile is
        // full whatever the row length; a tile may start mid-row and wrap over row ends.
        const uint64_t cap = tile_bytes / 16;  // units per tile: one per thread at the default size
        const uint64_t total = nrows * units;
        // When row length and row stride are whole 128-byte lines of the destination, a run that
        // starts mid-line gets a shorter first tile, so that every later tile starts on a line
        // (the kernel then stores whole lines per wavefront).
        const bool lines_repeat = nrows == 1 || ((units * vd) % 128 == 0 && D.stride % 128 == 0);
        const uint64_t first_short = lines_repeat ? (D.off % 128) / vd : 0;
        for (uint64_t v0 = 0, n; v0 < total; v0 += n) {
            n = std::min(v0 ? cap : cap - first_short, total - v0);
            Tile t;
            std::memset(&t, 0, sizeof t);
            const uint64_t row0 = nrows == 1 ? 0 : v0 / units;
            const uint64_t col0 = nrows == 1 ? 0 : v0 % units;
            // a single row needs no wrapping: the tile starts v0 units into it
            t.src_off = S.off + row0 * S.stride + (nrows == 1 ? v0 * vs : 0);
            t.dst_off = D.off + row0 * D.stride + (nrows == 1 ? v0 * vd : 0);
            t.src_stride = S.stride;
            t.dst_stride = D.stride;
            t.src_buf = S.buf;
            t.dst_buf = D.buf;
            t.count = (uint32_t)n;
            t.flags = flags;
            if (nrows == 1 || units >= cap || units == 1) {
                // at most one wrap inside a tile: the kernel compares instead of dividing
                t.ncols = nrows == 1 ? 0xFFFFFFFFu : (uint32_t)units;
                t.magic = 0;
            } else {
                t.ncols = (uint32_t)units;
                t.magic = (uint32_t)((1ull << 32) / units) + 1;
            }
            t.col0 = (uint32_t)col0;
            out.push_back(t);
        }
        return;
    }

    if (nrows == 1 || D.stride == ncols * D.es) {
        // Dense destination (every wire run of an explicit-segment plan, every one-row run): cut the
        // destination bytes at 16-byte boundaries so that each thread owns one aligned 16-byte slot
        // and gathers its elements from the source rows, wrapping at row ends.
        const uint64_t total = nrows * ncols;          // elements
        const uint64_t end = D.off + total * D.es;     // bytes
        // at most 32768 elements per tile keeps the kernel's multiply-high division exact
        const uint64_t tb = std::min<uint64_t>(tile_bytes, 32768ull * D.es);
        const uint64_t cap = tb / D.es;                // elements a tile can hold
        uint64_t pos = D.off;
        while (pos < end) {
            // Tiles end on 128-byte lines of the destination buffer (the first tile of a run is up
            // to a line short): with a line-aligned base pointer every later tile of the run starts
            // on a line, its slots need no shifting and each wavefront stores whole lines.
            uint64_t stop = std::min(end, pos / 128 * 128 + tb);
            // a tile that is not the last of its run writes the 16-byte slot straddling its end
            // whole, so at least 16 more bytes of the run must follow it
            if (end - stop < 16) stop = end;
            const uint64_t e0 = (pos - D.off) / D.es;
            Tile t;
            std::memset(&t, 0, sizeof t);
            const uint64_t row0 = nrows == 1 ? 0 : e0 / ncols;
            const uint64_t col0 = nrows == 1 ? 0 : e0 % ncols;
            t.src_off = S.off + row0 * S.stride + (nrows == 1 ? e0 * S.es : 0);
            t.dst_off = pos;
            t.src_stride = S.stride;
            t.dst_stride = 0;
            t.src_buf = S.buf;
            t.dst_buf = D.buf;
            t.count = (uint32_t)((stop - pos) / D.es);
            t.flags = (flags & ~TILE_KIND_MASK) | TILE_KIND_DENSE;
            if (nrows == 1 || ncols >= cap + 16 || ncols == 1) {
                // at most one row end inside the elements a tile touches (its own plus one slot)
                t.ncols = nrows == 1 ? 0xFFFFFFFFu : (uint32_t)ncols;
                t.magic = 0;
            } else {
                t.ncols = (uint32_t)ncols;
                t.magic = (uint32_t)((1ull << 32) / ncols) + 1;
            }
            t.col0 = (uint32_t)col0;
            if (pos != D.off) t.flags |= TILE_HEAD_SKIP;
            if (stop != end) t.flags |= TILE_TAIL_OK;
            if (stop == end && pad) t.flags |= (uint32_t)pad << TILE_PAD_SHIFT;
            out.push_back(t);
            pos = stop;
        }
        return;
    }

    auto emit = [&](uint64_t r0, uint64_t nr, uint64_t u0, uint64_t nu, bool last) {
        Tile t;
        std::memset(&t, 0, sizeof t);
        t.src_off = S.off + r0 * S.stride + u0 * unit_s;
        t.dst_off = D.off + r0 * D.stride + u0 * unit_d;
        t.src_stride = S.stride;
        t.dst_stride = D.stride;
        t.src_buf = S.buf;
        t.dst_buf = D.buf;
        t.count = (uint32_t)nr;
        t.ncols = (uint32_t)nu;
        t.flags = flags;
        const uint64_t slots = (nu * D.es + 15) / 16 + 1;  // 16-byte destination slots a row can touch
        // threads that share a row: a power of two, at most the workgroup of the kernel that runs these tiles
        t.flags |= std::min(ceil_log2((uint64_t)kBlockThreadsAny), ceil_log2(slots)) << TILE_LG_LANES_SHIFT;
        if (last && pad) t.flags |= (uint32_t)pad << TILE_PAD_SHIFT;
        out.push_back(t);
    };

    if (nrows == 1 || row_bytes >= tile_bytes) {
        // long rows: each row is cut into equal column pieces of at most one tile
        const uint64_t k = (row_bytes + tile_bytes - 1) / tile_bytes;
        const uint64_t per = ((units + k - 1) / k + 7) / 8 * 8;
        for (uint64_t r = 0; r < nrows; ++r)
            for (uint64_t u = 0; u < units; u += per)
                emit(r, 1, u, std::min(per, units - u), r + 1 == nrows && u + per >= units);
    } else {
        // short rows: several whole rows per tile, evenly
        const uint64_t fit = std::max<uint64_t>(1, tile_bytes / row_bytes);
        const uint64_t nt = (nrows + fit - 1) / fit;
        const uint64_t per = (nrows + nt - 1) / nt;
        for (uint64_t r = 0; r < nrows; r += per)
            emit(r, std::min(per, nrows - r), 0, units, r + per >= nrows);
    }
}

}  // namespace

static int segments_from_user_impl(const th_segment* segs, size_t n, const uint64_t* src_elems, uint32_t n_src,
                                   const uint64_t* dst_elems, uint32_t n_dst, bool narrow_at_unpack, Manifest& m) {
    if ((n && !segs) || (n_src && !src_elems) || (n_dst && !dst_elems)) {
        set_error("null segment or tensor-size array");
        return TH_ERR_ARG;
    }
    for (int side = 0; side < 2; ++side) {
        const uint32_t cnt = side ? n_dst : n_src;
        m.tensors[side].resize(cnt);
        for (uint32_t i = 0; i < cnt; ++i) {
            TensorInfo& t = m.tensors[side][i];
            t.name = (side ? "dst." : "src.") + std::to_string(i);
            t.rows = 1;
            t.cols = side ? dst_elems[i] : src_elems[i];
            t.dtype = 0;
        }
    }
    uint64_t wire = 0, run_start = 0;
    int64_t prev_tensor = -1;
    for (size_t k = 0; k < n; ++k) {
        const th_segment& u = segs[k];
        if (u.src_tensor >= n_src || u.dst_tensor >= n_dst) {
            set_error("segment %zu: tensor id out of range", k);
            return TH_ERR_RANGE;
        }
        if ((u.src_dtype != TH_BF16 && u.src_dtype != TH_F32) || (u.dst_dtype != TH_BF16 && u.dst_dtype != TH_F32)) {
            set_error("segment %zu: bad dtype", k);
            return TH_ERR_ARG;
        }
        if (u.src_dtype == TH_BF16 && u.dst_dtype == TH_F32) {
            set_error("segment %zu: bf16 -> fp32 widening is not supported", k);
            return TH_ERR_UNSUPPORTED;
        }
        TensorInfo& st = m.tensors[0][u.src_tensor];
        TensorInfo& dt = m.tensors[1][u.dst_tensor];
        if ((st.dtype && st.dtype != u.src_dtype) || (dt.dtype && dt.dtype != u.dst_dtype)) {
            set_error("segment %zu: a tensor is used with two dtypes", k);
            return TH_ERR_ARG;
        }
        st.dtype = u.src_dtype;
        dt.dtype = u.dst_dtype;
        if (u.nrows == 0 || u.row_len == 0) continue;
        if (u.nrows > 1 && u.dst_row_stride < u.row_len) {
            set_error("segment %zu: destination rows overlap (stride < row length)", k);
            return TH_ERR_ARG;
        }
        const u128 s_last = (u128)u.src_elem_off + (u128)(u.nrows - 1) * u.src_row_stride + u.row_len;
        const u128 d_last = (u128)u.dst_elem_off + (u128)(u.nrows - 1) * u.dst_row_stride + u.row_len;
        if (s_last > st.cols || d_last > dt.cols) {
            set_error("segment %zu reaches outside its %s tensor", k, s_last > st.cols ? "source" : "destination");
            return TH_ERR_RANGE;
        }
        if ((u128)u.nrows * u.row_len > ((u128)1 << 60)) {
            set_error("segment %zu is too large", k);
            return TH_ERR_RANGE;
        }
        // a tile record keeps a rectangle's row length, and the kernels a position in a row plus a tile's
        // length, in 32 bits (a single row needs neither)
        if (u.nrows > 1 && u.row_len >= (1ull << 31)) {
            set_error("segment %zu: rows of 2^31 elements or more are supported only as single-row segments", k);
            return TH_ERR_UNSUPPORTED;
        }
        if ((int64_t)u.src_tensor != prev_tensor) {
            const uint64_t aligned = (wire + 15) / 16 * 16;
            if (!m.segments.empty()) m.segments.back().pad_after = (uint8_t)(aligned - wire);
            wire = aligned;
            run_start = wire;
            prev_tensor = u.src_tensor;
        }
        Segment g;
        g.src_tensor = u.src_tensor;
        g.dst_tensor = u.dst_tensor;
        g.src_off = u.src_elem_off;
        g.src_stride = u.src_row_stride;
        g.dst_off = u.dst_elem_off;
        g.dst_stride = u.dst_row_stride;
        g.nrows = u.nrows;
        g.row_len = u.row_len;
        g.src_dtype = u.src_dtype;
        g.dst_dtype = u.dst_dtype;
        g.wire_dtype = narrow_at_unpack ? u.src_dtype : u.dst_dtype;
        g.wire_off = wire;
        g.run_start = run_start;
        g.wire_stride = u.row_len * esize(g.wire_dtype);
        m.segments.push_back(g);
        wire += u.nrows * u.row_len * esize(g.wire_dtype);
    }
    return TH_OK;
}

static int finish_manifest_impl(Manifest& m, uint64_t CB, bool ptrs_aligned16, const Tuning& tune) {
    if (CB == 0 || CB % 16) {
        set_error("chunk_bytes must be a positive multiple of 16");
        return TH_ERR_ARG;
    }
    m.chunk_bytes = CB;
    m.wire_bytes = m.payload_bytes = m.src_read_bytes = 0;
    m.tensor_wire_end.assign(m.tensors[0].size(), 0);
    for (const Segment& g : m.segments) {
        m.wire_bytes = std::max(m.wire_bytes, seg_wire_end(g));
        m.tensor_wire_end[g.src_tensor] = std::max(m.tensor_wire_end[g.src_tensor], seg_wire_end(g));
        m.payload_bytes += g.nrows * g.row_len * esize(g.wire_dtype);
        m.src_read_bytes += g.nrows * g.row_len * esize(g.src_dtype);
    }
    const uint64_t nchunks = (m.wire_bytes + CB - 1) / CB;
    if (nchunks > 0x7FFFFFFFull) {
        set_error("too many chunks");
        return TH_ERR_RANGE;
    }
    m.n_chunks = (uint32_t)nchunks;

    // ---- runs: every segment cut so that each piece lies inside one chunk ----
    for (const Segment& g : m.segments) {
        const unsigned es_s = esize(g.src_dtype), es_w = esize(g.wire_dtype), es_d = esize(g.dst_dtype);
        const uint64_t row_bytes = g.row_len * es_w;
        auto emit = [&](uint64_t r0, uint64_t nr, uint64_t c0, uint64_t nc, uint64_t wire_pos) {
            th_run r;
            std::memset(&r, 0, sizeof r);
            r.src_tensor = g.src_tensor;
            r.dst_tensor = g.dst_tensor;
            r.chunk = (uint32_t)(wire_pos / CB);
            r.src_byte_off = (g.src_off + r0 * g.src_stride + c0) * es_s;
            r.src_byte_stride = g.src_stride * es_s;
            r.dst_byte_off = (g.dst_off + r0 * g.dst_stride + c0) * es_d;
            r.dst_byte_stride = g.dst_stride * es_d;
            r.chunk_byte_off = wire_pos % CB;
            r.wire_byte_stride = g.wire_stride;
            r.nrows = nr;
            r.row_len = nc;
            r.src_dtype = g.src_dtype;
            r.dst_dtype = g.dst_dtype;
            r.wire_dtype = g.wire_dtype;
            if (r0 + nr == g.nrows && c0 + nc == g.row_len) r.pad_bytes = g.pad_after;
            m.runs.push_back(r);
            m.run_starts.push_back(g.run_start);
        };
        uint64_t r = 0;
        while (r < g.nrows) {
            const uint64_t start = g.wire_off + r * g.wire_stride;
            const uint64_t lim = (start / CB + 1) * CB;
            if (start + row_bytes <= lim) {
                // this row and maybe more rows end inside the chunk
                const uint64_t cnt = std::min(g.nrows - r, (lim - row_bytes - start) / g.wire_stride + 1);
                emit(r, cnt, 0, g.row_len, start);
                r += cnt;
            } else {
                // the row crosses one or more chunk boundaries: cut it by columns
                uint64_t col = 0;
                while (col < g.row_len) {
                    const uint64_t pos = start + col * es_w;
                    const uint64_t room = ((pos / CB + 1) * CB - pos) / es_w;
                    const uint64_t nc = std::min(g.row_len - col, room);
                    emit(r, 1, col, nc, pos);
                    col += nc;
                }
                r += 1;
            }
        }
    }

    // ---- tiles: one list per direction and the wire-free list, built by three threads (the lists
    // are independent; what they learn about the tensors is merged afterwards) ----
    struct Seen {
        std::vector<uint8_t> used, need16;
    };
    Seen seen[3][2];  // [list][tensor side]
    for (int l = 0; l < 3; ++l)
        for (int s = 0; s < 2; ++s) {
            seen[l][s].used.assign(m.tensors[s].size(), 0);
            seen[l][s].need16.assign(m.tensors[s].size(), 0);
        }
    const size_t guess = (size_t)(m.payload_bytes / std::min({tune.tile_bytes, tune.tile_bytes_any, tune.tile_bytes_narrow}));

    // One list per direction: vector-path tiles first, each sub-list grouped by chunk.  Runs come in
    // wire order, so within a class the tiles are generated in chunk order already: the two classes
    // are collected separately and joined, nothing is sorted or copied twice.
    // The short class is one more launch per call, with a tail of its own: it pays when short runs
    // are a good part of the list (thousands of tiny tensors: 3 to 7 times faster), not when a few
    // percent of the tiles are short (the scattered sweep loses 0.8 % to it).  A list gets the class
    // when at least one piece of work in eight is a short run; `bytes` are a list's destination bytes.
    auto tuning_for = [&](uint64_t short_runs, uint64_t bytes) {
        Tuning t = tune;
        const uint64_t est_tiles = bytes / std::max<uint64_t>(4096, std::min({t.tile_bytes, t.tile_bytes_any, t.tile_bytes_narrow})) + short_runs;
        if (short_runs * 8 < est_tiles) t.short_slots = 0;
        return t;
    };
    auto run_is_short = [&](uint64_t nrows, uint64_t ncols, unsigned es_src, unsigned es_dst) {
        const uint64_t slot = (es_src == 4 && es_dst == 2) ? 8 : 16;
        return nrows * ((ncols * es_dst + slot - 1) / slot + 1) <= tune.short_slots;
    };

    auto build_side = [&](int side) {
        uint64_t short_runs = 0, list_bytes = 0;
        for (const th_run& r : m.runs) {
            const unsigned es_from = esize(side == 0 ? r.src_dtype : r.wire_dtype);
            const unsigned es_to = esize(side == 0 ? r.wire_dtype : r.dst_dtype);
            short_runs += run_is_short(r.nrows, r.row_len, es_from, es_to);
            list_bytes += r.nrows * r.row_len * es_to;
        }
        const Tuning tune = tuning_for(short_runs, list_bytes);  // shadows the plan's: this list's
        std::vector<Tile> tiles[kPathClasses];
        std::vector<uint64_t> base[kPathClasses];
        bool reserved[kPathClasses] = {false, false, false};
        Seen& mine = seen[side][side];  // pack learns about source tensors, unpack about destination tensors
        for (unsigned k = 0; k < kPathClasses; ++k) m.chunk_tile0[side][k].assign((size_t)m.n_chunks + 1, 0);
        for (size_t ri = 0; ri < m.runs.size(); ++ri) {
            const th_run& r = m.runs[ri];
            const unsigned es_s = esize(r.src_dtype), es_w = esize(r.wire_dtype), es_d = esize(r.dst_dtype);
            Side S, D;
            if (side == 0) {
                S = Side{r.src_tensor, r.src_byte_off, r.src_byte_stride, es_s};
                D = Side{r.chunk, r.chunk_byte_off, r.wire_byte_stride, es_w};
            } else {
                S = Side{r.chunk, r.chunk_byte_off, r.wire_byte_stride, es_w};
                D = Side{r.dst_tensor, r.dst_byte_off, r.dst_byte_stride, es_d};
            }
            bool vec = false;
            size_t before[kPathClasses];
            for (unsigned k = 0; k < kPathClasses; ++k) before[k] = tiles[k].size();
            tile_run(tiles, S, D, r.nrows, r.row_len, side == 0 ? r.pad_bytes : 0, ptrs_aligned16, tune, vec);
            for (unsigned k = 0; k < kPathClasses; ++k) {
                if (tiles[k].size() == before[k]) continue;
                if (!reserved[k]) {  // first run of this class (most plans use one class only)
                    reserved[k] = true;
                    tiles[k].reserve(guess + 2 * m.runs.size());
                    base[k].reserve(guess + 2 * m.runs.size());
                }
                for (size_t i = before[k]; i < tiles[k].size(); ++i) {
                    Tile& t = tiles[k][i];
                    t.src_tensor = r.src_tensor;
                    const uint64_t wire_off = (uint64_t)r.chunk * CB + (side == 0 ? t.dst_off : t.src_off);
                    base[k].push_back((wire_off - m.run_starts[ri]) / 2);
                }
                m.chunk_tile0[side][k][r.chunk + 1] += tiles[k].size() - before[k];
            }
            const uint32_t tensor = side == 0 ? r.src_tensor : r.dst_tensor;
            mine.used[tensor] = 1;
            if (vec) mine.need16[tensor] = 1;
        }
        const int classes_in_use = !tiles[0].empty() + !tiles[1].empty() + !tiles[2].empty();
        if (tune.single_list && classes_in_use > 1) {
            // A plan that publishes progress finishes chunk after chunk, which launches class after
            // class cannot: when its tiles are of more than one class they all go into one list in
            // chunk order, run by the kernel that holds every path.  (A plan with vector-path tiles
            // only, the usual case for model weights, keeps the vector-only kernel.)
            std::vector<Tile> all;
            std::vector<uint64_t> all_base;
            all.reserve(tiles[0].size() + tiles[1].size() + tiles[2].size());
            all_base.reserve(all.capacity());
            size_t pos[kPathClasses] = {0, 0, 0};
            for (size_t c = 0; c < m.n_chunks; ++c) {
                uint64_t total = 0;
                for (unsigned k = 0; k < kPathClasses; ++k) {
                    const uint64_t cnt = m.chunk_tile0[side][k][c + 1];
                    all.insert(all.end(), tiles[k].begin() + pos[k], tiles[k].begin() + pos[k] + cnt);
                    all_base.insert(all_base.end(), base[k].begin() + pos[k], base[k].begin() + pos[k] + cnt);
                    pos[k] += cnt;
                    total += cnt;
                    m.chunk_tile0[side][k][c + 1] = 0;
                }
                m.chunk_tile0[side][1][c + 1] = total;
            }
            tiles[0].clear(), tiles[2].clear(), base[0].clear(), base[2].clear();
            tiles[1] = std::move(all);
            base[1] = std::move(all_base);
        }
        uint64_t class_start = 0;
        for (unsigned k = 0; k < kPathClasses; ++k) {
            std::vector<uint64_t>& first = m.chunk_tile0[side][k];
            first[0] = class_start;
            for (size_t c = 0; c < m.n_chunks; ++c) first[c + 1] += first[c];
            class_start += tiles[k].size();
        }
        unsigned lead = 0;  // the first class that has tiles keeps its storage, the others are appended
        while (lead + 1 < kPathClasses && tiles[lead].empty()) ++lead;
        m.tiles[side] = std::move(tiles[lead]);
        m.tile_base[side] = std::move(base[lead]);
        for (unsigned k = lead + 1; k < kPathClasses; ++k) {
            m.tiles[side].insert(m.tiles[side].end(), tiles[k].begin(), tiles[k].end());
            m.tile_base[side].insert(m.tile_base[side].end(), base[k].begin(), base[k].end());
        }
    };

    // direct list: holder tensors -> reader tensors without the wire, one pass over the segments
    auto build_direct = [&]() {
        uint64_t short_runs = 0, list_bytes = 0;
        for (const Segment& g : m.segments) {
            short_runs += run_is_short(g.nrows, g.row_len, esize(g.src_dtype), esize(g.dst_dtype));
            list_bytes += g.nrows * g.row_len * esize(g.dst_dtype);
        }
        const Tuning tune = tuning_for(short_runs, list_bytes);
        std::vector<Tile> tiles[kPathClasses];
        bool reserved = false;
        for (const Segment& g : m.segments) {
            const unsigned es_s = esize(g.src_dtype), es_d = esize(g.dst_dtype);
            const Side S{g.src_tensor, g.src_off * es_s, g.src_stride * es_s, es_s};
            const Side D{g.dst_tensor, g.dst_off * es_d, g.dst_stride * es_d, es_d};
            bool vec = false;
            tile_run(tiles, S, D, g.nrows, g.row_len, 0, ptrs_aligned16, tune, vec);
            if (!reserved) {
                reserved = true;
                tiles[vec ? 0 : 1].reserve(guess + 2 * m.segments.size());
            }
            if (vec) seen[2][0].need16[g.src_tensor] = seen[2][1].need16[g.dst_tensor] = 1;
        }
        unsigned lead = 0;
        while (lead + 1 < kPathClasses && tiles[lead].empty()) ++lead;
        for (unsigned k = 0; k < kPathClasses; ++k) m.direct_n[k] = tiles[k].size();
        m.tiles[2] = std::move(tiles[lead]);
        for (unsigned k = lead + 1; k < kPathClasses; ++k)
            m.tiles[2].insert(m.tiles[2].end(), tiles[k].begin(), tiles[k].end());
    };

    // The three lists are independent.  Large plans build the two per-direction lists on threads of
    // their own; an exception inside a list builder is caught where it is thrown and handed back
    // after the join, and a thread that cannot be started leaves its list to this thread.
    int status[3] = {TH_OK, TH_OK, TH_OK};
    auto guarded = [&](int which) {
        try {
            if (which < 2)
                build_side(which);
            else
                build_direct();
        } catch (...) {
            status[which] = TH_ERR_NOMEM;
        }
    };
    std::thread workers[2];
    bool started[2] = {false, false};
    if (guess >= 4096 && tune.planner_threads > 1) {  // small plans: not worth two threads
        for (int k = 0; k < 2; ++k) {
            try {
                workers[k] = std::thread(guarded, k);
                started[k] = true;
            } catch (...) {
            }
        }
    }
    guarded(2);
    for (int k = 0; k < 2; ++k)
        if (!started[k]) guarded(k);
    for (int k = 0; k < 2; ++k)
        if (started[k]) workers[k].join();
    for (int k = 0; k < 3; ++k)
        if (status[k] != TH_OK) {
            set_error("out of memory while building the tile lists");
            return status[k];
        }
    for (int l = 0; l < 3; ++l)
        for (int s = 0; s < 2; ++s)
            for (size_t i = 0; i < m.tensors[s].size(); ++i) {
                if (seen[l][s].used[i]) m.tensors[s][i].used = true;
                if (seen[l][s].need16[i]) m.tensors[s][i].need16 = true;
            }
    return TH_OK;
}

// Nothing may leave the planner as an exception: the callers are extern "C".
template <class F>
static int no_throw(F&& body) {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        set_error("out of memory");
        return TH_ERR_NOMEM;
    } catch (const std::exception& e) {
        set_error("planner failed: %s", e.what());
        return TH_ERR_NOMEM;
    } catch (...) {
        set_error("planner failed");
        return TH_ERR_NOMEM;
    }
}

int segments_from_user(const th_segment* segs, size_t n, const uint64_t* src_elems, uint32_t n_src,
                       const uint64_t* dst_elems, uint32_t n_dst, bool narrow_at_unpack, Manifest& m) {
    return no_throw([&] {
        return segments_from_user_impl(segs, n, src_elems, n_src, dst_elems, n_dst, narrow_at_unpack, m);
    });
}

int finish_manifest(Manifest& m, uint64_t CB, bool ptrs_aligned16, const Tuning& tune) {
    return no_throw([&] { return finish_manifest_impl(m, CB, ptrs_aligned16, tune); });
}

}  // namespace th
