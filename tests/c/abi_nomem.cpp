// Allocation failures at the C ABI (no GPU needed): this program replaces the global operator new,
// which the shared library then uses too, and lets the k-th allocation inside th_plan_create* fail
// for every k.  Each call must come back with TH_OK or TH_ERR_NOMEM and a message; nothing may
// throw through the extern "C" boundary or terminate the process.
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "th.h"

static std::atomic<long> g_countdown{-1};
static void maybe_fail() {
    if (g_countdown.load(std::memory_order_relaxed) >= 0 && g_countdown.fetch_sub(1) == 0) throw std::bad_alloc();
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

#define CHECK(c)                                                                                     \
    do {                                                                                             \
        if (!(c)) {                                                                                  \
            std::fprintf(stderr, "line %d: %s (last error: %s)\n", __LINE__, #c, th_last_error());   \
            return 1;                                                                                \
        }                                                                                            \
    } while (0)

int main() {
    // a model plan (small dense model, TP=2 holder rank 1 -> TP=1 reader) and an explicit-segment plan
    // large enough for the threaded list build
    th_model_desc model;
    std::memset(&model, 0, sizeof model);
    model.kind = TH_MODEL_DENSE;
    model.n_layers = 2, model.hidden = 256, model.n_q_heads = 4, model.n_kv_heads = 2, model.head_dim = 64;
    model.ffn = 1024, model.vocab = 1000, model.tied_embeddings = 1;
    model.weight_dtype = TH_BF16, model.norm_dtype = TH_F32;
    th_layout src = {2, 1, 1, 0, 0, TH_F32, 0, 0}, dst = {1, 0, 1, 0, 0, TH_BF16, 0, 0};
    std::vector<th_segment> segs(3000);
    std::vector<uint64_t> se(3000, 5000), de(1, 3000ull * 5000);
    for (size_t k = 0; k < segs.size(); ++k) {
        std::memset(&segs[k], 0, sizeof segs[k]);
        segs[k].src_tensor = (uint32_t)k;
        segs[k].nrows = 40, segs[k].row_len = 100 + k % 20, segs[k].src_row_stride = 125, segs[k].dst_row_stride = 120;
        segs[k].dst_elem_off = k * 5000;
        segs[k].src_dtype = TH_F32, segs[k].dst_dtype = TH_BF16;
    }
    long refused = 0, built = 0;
    for (int which = 0; which < 2; ++which) {
        for (long k = 0;; k += (k < 200 ? 1 : 17)) {
            th_plan* plan = nullptr;
            g_countdown.store(k);
            const int rc = which == 0
                               ? th_plan_create(&model, &src, &dst, 1 << 16, TH_FLAG_HOST_ONLY, &plan)
                               : th_plan_create_from_segments(segs.data(), segs.size(), se.data(), 3000, de.data(), 1,
                                                              1 << 20, TH_FLAG_HOST_ONLY, &plan);
            const bool fired = g_countdown.load() < 0;
            g_countdown.store(-1);
            CHECK(rc == TH_OK || rc == TH_ERR_NOMEM);
            if (rc == TH_ERR_NOMEM) {
                CHECK(fired && plan == nullptr && std::strlen(th_last_error()) > 0);
                ++refused;
            } else {
                CHECK(plan != nullptr && th_plan_num_chunks(plan) > 0);
                CHECK(th_plan_destroy(plan) == TH_OK);
            }
            if (!fired) {
                ++built;
                break;
            }
        }
    }
    CHECK(built == 2 && refused > 40);
    std::printf("c abi nomem ok: %ld calls refused with TH_ERR_NOMEM\n", refused);
    return 0;
}
