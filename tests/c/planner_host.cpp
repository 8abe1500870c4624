// Host-only driver of the planner (th_layouts.cpp + th_planner.cpp, no HIP): built by
// tests/test_planner_sanitizers.py with -fsanitize=address,undefined.  It plans the full-size
// workloads and a few thousand odd explicit segments, checks that one planner thread and three
// build identical tile lists, and lets every allocation of a plan fail in turn: each attempt must
// end in TH_OK or TH_ERR_NOMEM, never in std::terminate, a leak or a report from the sanitizers.
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "th_internal.hpp"

namespace th {
static char g_last[512];
void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last, sizeof g_last, fmt, ap);
    va_end(ap);
}
Tuning current_tuning() { return Tuning(); }
}  // namespace th
using namespace th;

// ---- allocation failure injection: the k-th allocation from now throws (any thread) ----
static std::atomic<long> g_countdown{-1};
static std::atomic<long> g_failed{0};
static void maybe_fail() {
    if (g_countdown.load(std::memory_order_relaxed) >= 0 && g_countdown.fetch_sub(1) == 0) {
        g_failed.fetch_add(1);
        throw std::bad_alloc();
    }
}
void* operator new(std::size_t n) {
    maybe_fail();
    void* p = std::malloc(n ? n : 1);
    if (!p) throw std::bad_alloc();
    return p;
}
void* operator new(std::size_t n, std::align_val_t a) {
    maybe_fail();
    void* p = nullptr;
    if (posix_memalign(&p, (std::size_t)a < sizeof(void*) ? sizeof(void*) : (std::size_t)a, n ? n : 1)) throw std::bad_alloc();
    return p;
}
void operator delete(void* p) noexcept { std::free(p); }
void operator delete(void* p, std::size_t) noexcept { std::free(p); }
void operator delete(void* p, std::align_val_t) noexcept { std::free(p); }
void operator delete(void* p, std::size_t, std::align_val_t) noexcept { std::free(p); }

#define CHECK(c)                                                                          \
    do {                                                                                  \
        if (!(c)) {                                                                       \
            std::fprintf(stderr, "line %d: %s (last error: %s)\n", __LINE__, #c, g_last); \
            return 1;                                                                     \
        }                                                                                 \
    } while (0)

static th_layout L(int T, int r, int P = 1, int p = 0, int st = 0, int f32 = TH_F32, int grp = 0, int pad = 0) {
    th_layout l{T, r, P, p, st, f32, grp, pad};
    return l;
}

static std::vector<th_segment> odd_segments(int n, uint64_t src_elems, uint64_t* dst_elems) {
    std::vector<th_segment> segs;
    uint64_t d = 0;
    for (int k = 0; k < n; ++k) {
        th_segment s{};
        s.src_tensor = (uint32_t)(k / 40);
        s.dst_tensor = 0;
        s.row_len = 1 + (k * 7) % 97;
        s.nrows = 1 + (k * 13) % 50;
        s.src_row_stride = s.row_len + (k % 5);
        s.dst_row_stride = s.row_len + (k % 3);
        s.src_elem_off = (uint64_t)(k * 37) % (src_elems - 50 * 110);
        s.dst_elem_off = d;
        d += s.nrows * s.dst_row_stride + 1;
        s.src_dtype = TH_F32;
        s.dst_dtype = (k / 40) % 2 ? TH_BF16 : TH_F32;  // one dtype per destination use; one per source tensor
        s.dst_tensor = (k / 40) % 2;
        segs.push_back(s);
    }
    *dst_elems = d;
    return segs;
}

static bool same_lists(const Manifest& a, const Manifest& b) {
    for (int l = 0; l < 3; ++l) {
        if (a.tiles[l].size() != b.tiles[l].size()) return false;
        if (!a.tiles[l].empty() && std::memcmp(a.tiles[l].data(), b.tiles[l].data(), a.tiles[l].size() * sizeof(Tile)))
            return false;
    }
    for (int s = 0; s < 2; ++s)
        for (int k = 0; k < kPathClasses; ++k)
            if (a.chunk_tile0[s][k] != b.chunk_tile0[s][k]) return false;
    return a.tile_base[0] == b.tile_base[0] && a.tile_base[1] == b.tile_base[1];
}

int main() {
    th_model_desc m8{TH_MODEL_DENSE, 32, 4096, 32, 8, 128, 14336, 128256, 0, 0, 0, 0, TH_BF16, TH_F32};
    th_model_desc m70{TH_MODEL_DENSE, 80, 8192, 64, 8, 128, 28672, 128256, 0, 0, 0, 0, TH_BF16, TH_F32};
    th_model_desc moe{TH_MODEL_MOE, 24, 2048, 16, 16, 128, 0, 102400, 0, 64, 2, 1408, TH_BF16, TH_F32};
    th_model_desc small{TH_MODEL_DENSE, 2, 512, 16, 4, 32, 1024, 2048, 0, 0, 0, 0, TH_BF16, TH_F32};
    struct Case {
        th_model_desc* m;
        th_layout s, d;
        uint64_t cb;
    } cases[] = {{&m8, L(1, 0), L(4, 0, 1, 0, 0, TH_BF16), 64u << 20},
                 {&m70, L(8, 1), L(4, 0, 1, 0, 0, TH_BF16), 256u << 20},
                 {&moe, L(1, 0, 8, 0), L(2, 0, 1, 0, 1, TH_BF16), 4u << 20},
                 {&small, L(8, 5), L(2, 1, 1, 0, 0, TH_BF16), 4096},
                 {&small, L(2, 1, 1, 0, 0, TH_F32, 1, 4096), L(16, 13, 1, 0, 0, TH_BF16), 1u << 16}};
    // 1. full-size and small model plans, three threads against one
    for (auto& c : cases) {
        Manifest a, b;
        CHECK(build_model_segments(*c.m, c.s, c.d, false, a) == TH_OK);
        CHECK(build_model_segments(*c.m, c.s, c.d, false, b) == TH_OK);
        Tuning t3, t1;
        t1.planner_threads = 1;
        CHECK(finish_manifest(a, c.cb, true, t3) == TH_OK);
        CHECK(finish_manifest(b, c.cb, true, t1) == TH_OK);
        CHECK(same_lists(a, b));
        std::printf("segments %zu runs %zu tiles %zu/%zu/%zu wire %llu\n", a.segments.size(), a.runs.size(),
                    a.tiles[0].size(), a.tiles[1].size(), a.tiles[2].size(), (unsigned long long)a.wire_bytes);
    }
    // 1b. the order in which a launch walks a tile range in prefix order: every record exactly once,
    //     blocks in launch order, one run of consecutive records per XCD and block, the tail as it comes
    const uint32_t B = kOrderBlock, G = kOrderGroup;
    for (uint32_t n : {0u, 1u, 7u, B - 1, B, B + 1, 2 * B - 1, 2 * B, 3 * B + 17, 4096u, 100003u}) {
        std::vector<uint8_t> hit(n, 0);
        for (uint32_t q = 0; q < n; ++q) {
            const uint32_t r = prefix_order_record(q, n);
            CHECK(r < n && !hit[r]);
            hit[r] = 1;
            if (q >= n / B * B) {
                CHECK(r == q);
            } else {
                CHECK(r / B == q / B);                                          // its own block
                CHECK((r % B) / G == q % 8);                                    // XCD q mod 8 owns one piece of the block
                if (q % B >= 8) CHECK(r == prefix_order_record(q - 8, n) + 1);  // ... and walks it in order
            }
        }
    }
    // 2. odd explicit segments (rows of 1..97 elements, every alignment), small tiles and chunks
    const uint64_t src_n = 1000000;
    uint64_t dst_n = 0;
    std::vector<th_segment> segs = odd_segments(4000, src_n, &dst_n);
    std::vector<uint64_t> se(100, src_n), de(2, dst_n);
    {
        Manifest a, b;
        CHECK(segments_from_user(segs.data(), segs.size(), se.data(), 100, de.data(), 2, false, a) == TH_OK);
        CHECK(segments_from_user(segs.data(), segs.size(), se.data(), 100, de.data(), 2, true, b) == TH_OK);
        Tuning t;
        t.tile_bytes_any = t.tile_bytes_narrow = 4096;
        CHECK(finish_manifest(a, 4096, false, t) == TH_OK);
        t.planner_threads = 1;
        CHECK(finish_manifest(b, 1u << 16, false, t) == TH_OK);
        std::printf("explicit: runs %zu / %zu tiles %zu / %zu\n", a.runs.size(), b.runs.size(), a.tiles[0].size(),
                    b.tiles[0].size());
        CHECK(a.tiles[0].size() >= 4096);  // large enough for the threaded build
    }
    // 3. every allocation fails in turn: serial build of a small model plan, threaded build of the
    //    explicit-segment plan (workers included)
    long attempts = 0, refused = 0;
    for (int threaded = 0; threaded < 2; ++threaded) {
        for (long k = 0;; k += (k < 300 ? 1 : 23)) {
            int rc;
            {
                Manifest m;
                g_countdown.store(k);
                if (threaded) {
                    rc = segments_from_user(segs.data(), segs.size(), se.data(), 100, de.data(), 2, false, m);
                    Tuning t;
                    t.tile_bytes_any = t.tile_bytes_narrow = 4096;
                    if (rc == TH_OK) rc = finish_manifest(m, 4096, false, t);
                } else {
                    rc = build_model_segments(small, L(8, 5), L(2, 1, 1, 0, 0, TH_BF16), false, m);
                    Tuning t;
                    if (rc == TH_OK) rc = finish_manifest(m, 4096, true, t);
                }
            }
            const bool fired = g_countdown.load() < 0;
            g_countdown.store(-1);
            ++attempts;
            CHECK(rc == TH_OK || rc == TH_ERR_NOMEM);
            if (rc == TH_ERR_NOMEM) {
                ++refused;
                CHECK(fired);
            }
            if (!fired) {  // the plan needed fewer than k allocations: it was built whole
                CHECK(rc == TH_OK);
                break;
            }
        }
    }
    std::printf("allocation failures: %ld attempts, %ld refused with TH_ERR_NOMEM, %ld injected\n", attempts, refused,
                g_failed.load());
    CHECK(refused > 50);
    std::printf("planner host ok\n");
    return 0;
}
